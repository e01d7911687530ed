// Verify attention on the matrix cores (gfx950), head_dim 128, bf16 queries, bf16 or e4m3 cache.
//
// Work decomposition.  The KV cache of one (request, KV head) pair ("unit") is a run of
// 16-token tiles, one per cache block.  All tiles of all units form one flat sequence (unit
// major).  A plan kernel writes that sequence out as a flat list of tile addresses (physical
// block * kv heads + kv head) and cuts it into `num_waves` equal contiguous spans; every
// wavefront streams one span, so the load is balanced whatever the mix of context lengths, and
// the load side of the kernel is a plain linear walk that never stops at a unit boundary.  A
// span may cover the tail of one unit, several whole units and the head of another; for every
// unit it touches the wave emits one partial result (softmax reference, sum, unnormalised
// output) into slot `wave + unit` (that sum is unique along the sequence).  A last kernel
// merges the partials of each unit by their log-sum-exp and writes the rounded output.
//
// Per tile, with rows = (k+1) * (query heads per KV head) padded to a multiple of 16:
//   S^T[token][row] = K[token][:] . Q[row][:]   v_mfma_f32_16x16x32_bf16, K tile as A operand
//   online softmax on S^T in registers (a row's 16 scores sit in 4 lanes x 4 registers)
//   O^T[d][row]    += V[token][d] * P[row][token]   v_mfma_f32_16x16x16_bf16, P taken straight
//                     from the S^T accumulator layout, V as A operand
// Both K and V are read from HBM directly in operand layout with 16-byte loads: for K a lane
// holds 8 consecutive d of one token; for V a lane holds d = 8*i .. 8*i+7 of four tokens and
// the eight M-blocks of O^T are the eight interleaved d-phases, so no transpose through LDS is
// needed (only a 16-bit pack per operand register).
#include "common.h"

namespace ss {
namespace {

// ---------------------------------------------------------------------------------------------
// plan: workgroup (b, g) sums the tile counts of the requests in front of b, writes the flat tile
// address list of its unit, and (b, 0) / the last one publish the prefix and the partition count
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_plan_kernel(AttnArgs a)
{
    __shared__ int sh[8];
    const int b = blockIdx.x / a.num_kv_heads, g = blockIdx.x % a.num_kv_heads;
    const int tid = threadIdx.x;
    int before = 0, rest = 0;   // tiles (per kv head) of the requests in front of b, and from b on
    for (int i = tid; i < a.batch; i += 256) {
        const int t = window_tiles(a.kv_len[i], a.q_indptr[i + 1] - a.q_indptr[i], a.q_lo);
        if (i < b) before += t; else rest += t;
    }
    for (int off = 32; off; off >>= 1) {
        before += __shfl_xor(before, off);
        rest += __shfl_xor(rest, off);
    }
    if ((tid & 63) == 0) {
        sh[tid >> 6] = before;
        sh[4 + (tid >> 6)] = rest;
    }
    __syncthreads();
    const int pre = sh[0] + sh[1] + sh[2] + sh[3];
    const long long total = (long long)(pre + sh[4] + sh[5] + sh[6] + sh[7]) * a.num_kv_heads;
    long long nw = total / kMinTilesPerWave;
    if (nw < 1) nw = 1;
    if (nw > a.launch_waves) nw = a.launch_waves;

    const int n = window_tiles(a.kv_len[b], a.q_indptr[b + 1] - a.q_indptr[b], a.q_lo);
    const long long off = (long long)pre * a.num_kv_heads + (long long)g * n;   // this unit's place in the flat list
    const int32_t *bt = a.block_table + (long long)b * a.max_blocks;
    int32_t *dst = a.tile_addr + off;
    for (int t = tid; t < n; t += 256) dst[t] = bt[t] * a.num_kv_heads + g;

    // waves whose span [w*total/nw, (w+1)*total/nw) starts inside this unit get their descriptor here
    const long long w_lo = (off * nw + total - 1) / total;             // first w with w*total/nw >= off
    const long long w_hi = ((off + n) * nw + total - 1) / total;       // first w with w*total/nw >= off + n
    // Descriptor: {request, kv head, first tile, tiles of the unit, span begin, span end, kv_len,
    // first query row, end query row, addresses of the span's first kDescAddrs tiles}: everything
    // the wave's first loads depend on, so that they go out after a single read.
    for (long long w = w_lo + tid; w < w_hi && w < nw; w += 256) {
        const long long x0 = w * total / nw, x1 = (w + 1) * total / nw;
        int32_t *d = a.wave_desc + w * kDescInts;
        d[0] = b; d[1] = g; d[2] = (int)(x0 - off); d[3] = n;
        d[4] = (int)x0; d[5] = (int)x1;
        d[6] = a.kv_len[b]; d[7] = a.q_indptr[b]; d[8] = a.q_indptr[b + 1];
        // walk forward from (b, g, tile) over unit boundaries; past the last unit repeat the last tile
        int bb = b, gg = g, tt = (int)(x0 - off), nn = n, last = 0;
        const int32_t *tb = bt;
        for (int j = 0; j < kDescAddrs; ++j) {
            while (bb < a.batch && tt >= nn) {
                tt -= nn;
                if (++gg == a.num_kv_heads) {
                    gg = 0;
                    if (++bb < a.batch) {
                        nn = window_tiles(a.kv_len[bb], a.q_indptr[bb + 1] - a.q_indptr[bb], a.q_lo);
                        tb = a.block_table + (long long)bb * a.max_blocks;
                    }
                }
            }
            if (bb < a.batch) last = tb[tt] * a.num_kv_heads + gg;
            d[9 + j] = last;
            ++tt;
        }
    }
    if (blockIdx.x == 0) {   // launched waves beyond the partition count get an empty span
        for (long long w = nw + tid; w < a.launch_waves; w += 256) {
            int32_t *d = a.wave_desc + w * kDescInts;
            d[4] = 0;
            d[5] = 0;
        }
    }
    if (g == 0 && tid == 0) {
        a.tile_prefix[b] = pre;
        if (b == a.batch - 1) {
            a.tile_prefix[a.batch] = pre + n;
            a.plan->total_tiles = (int)total;
            a.plan->num_waves = (int)nw;
        }
    }
}

}  // namespace

size_t attn_workspace_bytes(int batch, int max_blocks, int num_q_heads, int num_kv_heads, int head_dim, int launch_waves,
                            int max_q_len)
{
    const int G = num_q_heads / num_kv_heads;
    const size_t rows_pad = (size_t)attn_rows_pad(max_q_len, G);
    const size_t slots = (size_t)launch_waves + (size_t)batch * num_kv_heads;
    size_t n = 256;
    n += align_up(sizeof(int32_t) * ((size_t)batch + 1), 256);
    n += align_up(sizeof(int32_t) * kDescInts * (size_t)launch_waves, 256);
    n += align_up(sizeof(int32_t) * (size_t)batch * max_blocks * num_kv_heads, 256);
    n += align_up(slots * rows_pad * 2 * sizeof(float), 256);
    n += align_up(slots * rows_pad * (size_t)head_dim * sizeof(float), 256);
    return n;
}

bool attn_mfma_supported(const AttnArgs &a)
{
    const int G = a.num_q_heads / a.num_kv_heads;
    return a.head_dim == kMfmaHeadDim && a.q_dtype == SS_BF16 && (a.kv_dtype == SS_BF16 || a.kv_dtype == SS_FP8_E4M3) &&
           (G == 1 || G == 2 || G == 4 || G == 8) && a.launch_waves % kWavesPerWg == 0;
}

int32_t attn_mfma_launch(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1)
{
    const int G = a.num_q_heads / a.num_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return fail(SS_ERR_UNSUPPORTED, "head grouping not built for the MFMA kernel");
    // A wavefront holds at most 16 * kMaxRowBlocks query rows of a KV head.  A batch whose row bound
    // exceeds that is served in several passes over equal windows of query tokens, each a full
    // plan / stream / merge sequence on the same workspace (the stream orders them).
    const int win_max = 16 * kMaxRowBlocks / G;
    const int passes = (a.max_q_len + win_max - 1) / win_max;
    AttnArgs p = a;
    p.q_win = (a.max_q_len + passes - 1) / passes;
    for (p.q_lo = 0; p.q_lo < a.max_q_len; p.q_lo += p.q_win) {
        if (!(a.reuse_plan && passes == 1)) {   // a stored plan describes one window only
            hipLaunchKernelGGL(attn_plan_kernel, dim3((unsigned)a.batch * a.num_kv_heads), dim3(256), 0, stream, p);
            SS_HIP_CHECK(hipGetLastError(), "launch attn_plan_kernel");
        }
        // the streaming and merge kernels of each grouping live in their own translation unit; a
        // profile's event pair goes to the first pass
        hipEvent_t e0 = p.q_lo ? nullptr : ev0, e1 = p.q_lo ? nullptr : ev1;
        int32_t rc;
        switch (G) {
        case 1: rc = attn_mfma_launch_g1(p, stream, e0, e1); break;
        case 2: rc = attn_mfma_launch_g2(p, stream, e0, e1); break;
        case 4: rc = attn_mfma_launch_g4(p, stream, e0, e1); break;
        default: rc = attn_mfma_launch_g8(p, stream, e0, e1); break;
        }
        if (rc != SS_OK) return rc;
    }
    return SS_OK;
}

}  // namespace ss
