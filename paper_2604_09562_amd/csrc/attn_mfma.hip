// Verify attention on the matrix cores (gfx950), head_dim 128, bf16 queries, bf16 or e4m3 cache.
//
// Work decomposition.  The KV cache of one (request, KV head) pair ("unit") is a run of
// 16-token tiles, one per cache block.  All tiles of all units form one flat sequence (unit
// major).  A plan kernel writes that sequence out as a flat list of tile addresses (physical
// block * kv heads + kv head) and cuts it into `num_waves` contiguous spans of equal cost (a
// tile costs one, opening a unit a fixed number of tiles; span_cuts.h); every wavefront streams
// one span, so the load is balanced whatever the mix of context lengths, and the load side of
// the kernel is a plain linear walk that never stops at a unit boundary.  A span may cover the
// tail of one unit, several whole units and the head of another; for every unit it touches the
// wave has one partial result (softmax reference, sum, unnormalised output).  What the streaming
// kernel cannot finish itself (attn_mfma_kernels.h) goes to a partial slot, `wave + unit` or
// `workgroup + unit` (unique along the sequence), and a last kernel merges the partials of each
// such unit by their log-sum-exp and writes the rounded output.
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
#include "span_cuts.h"

namespace ss {
namespace {

// ---------------------------------------------------------------------------------------------
// plan: workgroup (b, g) writes the flat tile address list of its unit and the descriptors of the waves
// whose span starts inside it; (b, 0) / the last one publish the prefix and the partition count.
//
// Where the spans are cut.  A wave pays a fixed price for every unit it opens (query loads, a drained
// tile pipeline, the partial of the unit before: about the time of kUnitWeight tiles), so equal tile
// counts do not finish together: on a ragged batch the waves that cross ten short units were 10 % late.
// The cuts are therefore equal in a weighted coordinate in which every unit is kUnitWeight virtual
// tiles followed by its real ones; a cut that falls into a unit's virtual part becomes the unit's first
// tile.  The cuts depend on the batch's lengths only, so results do not vary from run to run.
// ---------------------------------------------------------------------------------------------
constexpr int kPlanMaxBatch = 4096;   // requests whose tile prefix fits the plan kernel's LDS; beyond that the cuts are unweighted

__global__ __launch_bounds__(256) void attn_plan_kernel(AttnArgs a)
{
    __shared__ int32_t prefix[kPlanMaxBatch + 1];
    __shared__ int sh[4];
    const int b = blockIdx.x / a.num_kv_heads, g = blockIdx.x % a.num_kv_heads;
    const int tid = threadIdx.x;
    const bool weighted = a.batch <= kPlanMaxBatch && a.unit_weight > 0;

    // exclusive prefix of the tile counts of all requests (every workgroup builds its own copy), or,
    // for a batch too large for that, just the sums in front of and from request b on
    int pre = 0;
    long long total = 0;
    if (a.batch <= kPlanMaxBatch) {
        int carry = 0;
        for (int base = 0; base < a.batch; base += 256) {
            const int i = base + tid;
            const int t = i < a.batch ? window_tiles(a.kv_len[i], a.q_indptr[i + 1] - a.q_indptr[i], a.q_lo) : 0;
            int incl = t;
            for (int off = 1; off < 64; off <<= 1) {
                const int o = __shfl_up(incl, off);
                if ((tid & 63) >= off) incl += o;
            }
            if ((tid & 63) == 63) sh[tid >> 6] = incl;
            __syncthreads();
            int before = carry;
            for (int wv = 0; wv < (tid >> 6); ++wv) before += sh[wv];
            if (i < a.batch) prefix[i] = before + incl - t;
            const int chunk_total = sh[0] + sh[1] + sh[2] + sh[3];
            __syncthreads();
            carry += chunk_total;
        }
        if (tid == 0) prefix[a.batch] = carry;
        __syncthreads();
        pre = prefix[b];
        total = (long long)prefix[a.batch] * a.num_kv_heads;
    } else {
        int before = 0, rest = 0;
        for (int i = tid; i < a.batch; i += 256) {
            const int t = window_tiles(a.kv_len[i], a.q_indptr[i + 1] - a.q_indptr[i], a.q_lo);
            if (i < b) before += t; else rest += t;
        }
        for (int off = 32; off; off >>= 1) {
            before += __shfl_xor(before, off);
            rest += __shfl_xor(rest, off);
        }
        __shared__ int sh2[8];
        if ((tid & 63) == 0) {
            sh2[tid >> 6] = before;
            sh2[4 + (tid >> 6)] = rest;
        }
        __syncthreads();
        pre = sh2[0] + sh2[1] + sh2[2] + sh2[3];
        total = (long long)(pre + sh2[4] + sh2[5] + sh2[6] + sh2[7]) * a.num_kv_heads;
    }
    long long nw = total / kMinTilesPerWave;
    if (nw < 1) nw = 1;
    if (nw > a.launch_waves) nw = a.launch_waves;
    const int weight = weighted ? a.unit_weight : 0;
    const long long total_w = total + (long long)weight * a.batch * a.num_kv_heads;

    const int n = window_tiles(a.kv_len[b], a.q_indptr[b + 1] - a.q_indptr[b], a.q_lo);
    const long long off = (long long)pre * a.num_kv_heads + (long long)g * n;   // this unit's place in the flat list
    const int32_t *bt = a.block_table + (long long)b * a.max_blocks;
    int32_t *dst = a.tile_addr + off;
    for (int t = tid; t < n; t += 256) dst[t] = bt[t] * a.num_kv_heads + g;

    // waves whose cut falls into this unit's stretch [ya, ya + weight + n) of the weighted coordinate
    SpanCuts cuts;
    cuts.prefix = prefix;   // (only read when weight > 0, i.e. when the prefix was built)
    cuts.batch = a.batch;
    cuts.hkv = a.num_kv_heads;
    cuts.weight = weight;
    cuts.total = total;
    cuts.total_w = total_w;
    cuts.nw = nw;
    const long long ya = off + (long long)weight * ((long long)b * a.num_kv_heads + g);
    const long long w_lo = cuts.first_cut_at_or_after(ya);                // first w with w*total_w/nw >= ya
    const long long w_hi = cuts.first_cut_at_or_after(ya + weight + n);   // first w at or past the unit's end
    // Descriptor: {request, kv head, first tile, tiles of the unit, span begin, span end, kv_len,
    // first query row, end query row, addresses of the span's first kDescAddrs tiles}: everything
    // the wave's first loads depend on, so that they go out after a single read.
    for (long long w = w_lo + tid; w < w_hi && w < nw; w += 256) {
        const int t0 = cuts.first_tile(cuts.cut(w), ya);
        const long long x0 = off + t0;
        const long long x1 = cuts.span_end(w);
        int32_t *d = a.wave_desc + w * kDescInts;
        d[0] = b; d[1] = g; d[2] = t0; d[3] = n;
        d[4] = (int)x0; d[5] = (int)x1;
        d[6] = a.kv_len[b]; d[7] = a.q_indptr[b]; d[8] = a.q_indptr[b + 1];
        // walk forward from (b, g, tile) over unit boundaries; past the last unit repeat the last tile
        int bb = b, gg = g, tt = t0, nn = n, last = 0;
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
            a.plan->unit_weight = weight;
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
