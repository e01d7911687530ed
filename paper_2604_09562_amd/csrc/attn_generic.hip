// Plain fp32 vector-ALU verify attention: the path for fp32 caches/queries, head_dim 64 and any
// head grouping the matrix-core kernel is not built for.  One 256-lane workgroup per
// (query row, query head); every lane walks its own tokens with a running (max, sum, output)
// triple and the 256 triples are merged at the end.  All arithmetic is fp32.
#include "common.h"

namespace ss {
namespace {

__device__ __forceinline__ float load_as_float(const void *p, int64_t i, int dtype)
{
    if (dtype == SS_F32) return static_cast<const float *>(p)[i];
    if (dtype == SS_BF16) {
        uint32_t w = (uint32_t) static_cast<const uint16_t *>(p)[i] << 16;
        return __uint_as_float(w);
    }
    // e4m3fn byte: the gfx950 converter implements the OCP format
    return __builtin_amdgcn_cvt_f32_fp8((uint32_t) static_cast<const uint8_t *>(p)[i], 0);
}

template <int D>
__global__ __launch_bounds__(256) void attn_generic_kernel(AttnArgs a)
{
    __shared__ float q_s[D];
    __shared__ float red_m[4], red_l[4];
    __shared__ float red_o[4][D];

    const int row = blockIdx.x / a.num_q_heads;
    const int h = blockIdx.x % a.num_q_heads;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int g = h / G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // request owning this row: largest b with q_indptr[b] <= row
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (a.q_indptr[mid] <= row) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int q0 = a.q_indptr[b], q_len = a.q_indptr[b + 1] - q0;
    // Visible cache positions: everything before this step's new tokens, then the new tokens the
    // row's mask word names (its own node and its ancestors); for a chain those are tokens 0..i.
    const int ctx = a.kv_len[b] - q_len;
    const uint32_t newmask = a.tree_mask ? a.tree_mask[row] : (2u << (row - q0)) - 1u;
    const int visible = ctx + 32 - __builtin_clz(newmask | 1u);  // one past the last visible position
    const int64_t qoff = ((int64_t)row * a.num_q_heads + h) * D;

    for (int d = tid; d < D; d += 256) q_s[d] = load_as_float(a.q, qoff + d, a.q_dtype);
    __syncthreads();

    float m = -INFINITY, l = 0.f;
    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;

    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks;
    for (int t = tid; t < visible; t += 256) {
        if (t >= ctx && !((newmask >> (t - ctx)) & 1u)) continue;
        const int64_t phys = bt[t / kTile];
        const int64_t base = ((phys * a.num_kv_heads + g) * kTile + (t % kTile)) * D;
        float s = 0.f;
#pragma unroll 8
        for (int d = 0; d < D; ++d) s = fmaf(q_s[d], load_as_float(a.k, base + d, a.kv_dtype), s);
        float vs = 1.f;
        if (a.k_scale) {
            s *= a.k_scale[phys * a.num_kv_heads + g];
            vs = a.v_scale[phys * a.num_kv_heads + g];
        }
        s *= a.sm_scale;
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new);  // exp(-inf) = 0 on the first token
        const float p = expf(s - m_new);
        l = l * alpha + p;
        const float pv = p * vs;
#pragma unroll 8
        for (int d = 0; d < D; ++d) o[d] = fmaf(pv, load_as_float(a.v, base + d, a.kv_dtype), o[d] * alpha);
        m = m_new;
    }

    // merge the 256 per-lane states: common max, rescale, sum
    float wm = m;
    for (int off = 32; off; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
    if (lane == 0) red_m[wave] = wm;
    __syncthreads();
    const float gm = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));  // finite: visible >= 1
    const float sc = (m == -INFINITY) ? 0.f : expf(m - gm);
    float wl = l * sc;
    for (int off = 32; off; off >>= 1) wl += __shfl_xor(wl, off);
    if (lane == 0) red_l[wave] = wl;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float x = o[d] * sc;
        for (int off = 32; off; off >>= 1) x += __shfl_xor(x, off);
        if (lane == 0) red_o[wave][d] = x;
    }
    __syncthreads();
    const float lsum = (red_l[0] + red_l[1]) + (red_l[2] + red_l[3]);
    for (int d = tid; d < D; d += 256) {
        const float x = ((red_o[0][d] + red_o[1][d]) + (red_o[2][d] + red_o[3][d])) / lsum;
        if (a.q_dtype == SS_F32)
            static_cast<float *>(a.out)[qoff + d] = x;
        else
            static_cast<__bf16 *>(a.out)[qoff + d] = (__bf16)x;  // round to nearest even
    }
    if (a.lse && tid == 0) a.lse[(int64_t)row * a.num_q_heads + h] = gm + logf(lsum);
}

}  // namespace

int32_t attn_generic_launch(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1)
{
    const unsigned grid = (unsigned)a.total_rows * (unsigned)a.num_q_heads;
    if (ev0) SS_HIP_CHECK(hipEventRecord(ev0, stream), "hipEventRecord");
    if (a.head_dim == 64)
        hipLaunchKernelGGL(attn_generic_kernel<64>, dim3(grid), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(attn_generic_kernel<128>, dim3(grid), dim3(256), 0, stream, a);
    SS_HIP_CHECK(hipGetLastError(), "launch attn_generic_kernel");
    if (ev1) SS_HIP_CHECK(hipEventRecord(ev1, stream), "hipEventRecord");
    return SS_OK;
}

}  // namespace ss
