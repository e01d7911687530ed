// KV append before the verify step, compaction of an accepted tree path and commit after acceptance
// (decode KV = prefill KV with the new tokens appended).  One wavefront per (request, new token, KV head); a lane owns head_dim/64
// consecutive elements of the key and of the value.
#include "common.h"

#include <type_traits>

namespace ss {
namespace {

typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr float kFp8Max = 448.0f;   // largest finite e4m3fn value

template <int NEW_DT, int EPL>
__device__ __forceinline__ void load_new(const void *src, int64_t base, int lane, float (&x)[EPL])
{
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int64_t i = base + lane * EPL + e;
        if constexpr (NEW_DT == SS_F32)
            x[e] = static_cast<const float *>(src)[i];
        else
            x[e] = __uint_as_float((uint32_t) static_cast<const uint16_t *>(src)[i] << 16);
    }
}

__device__ __forceinline__ uint16_t to_bf16_rne(float f)
{
    const float2v v = {f, 0.f};
    return (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2)) & 0xffffu);
}

__device__ __forceinline__ uint8_t to_e4m3_rne(float x, float scale)
{
    float q = x / scale;                       // one IEEE division, as the reference encoder takes it
    q = fminf(fmaxf(q, -kFp8Max), kFp8Max);    // saturate: the cache never holds the NaN byte for finite input
    return (uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(q, 0.f, 0, false) & 0xffu);
}

// grid: batch * max_q_len * kv heads; workgroup = one wavefront
template <int KV_DT, int NEW_DT, int EPL>
__global__ __launch_bounds__(64) void kv_append_kernel(KvAppendArgs a)
{
    const int lane = threadIdx.x;
    const int h = blockIdx.x % a.num_kv_heads;
    const int bi = blockIdx.x / a.num_kv_heads, i = bi % a.max_q_len, b = bi / a.max_q_len;
    const int r0 = a.q_indptr[b], q_len = a.q_indptr[b + 1] - r0;
    if (i >= q_len) return;
    const int D = a.head_dim;
    const int P = a.kv_len[b] - q_len;          // cache position of the request's first new token
    const int pos = P + i, blk = pos / kTile, slot = pos % kTile;
    const int phys = a.block_table[(int64_t)b * a.max_blocks + blk];
    const int64_t src = ((int64_t)(r0 + i) * a.num_kv_heads + h) * D;
    const int64_t dst = (((int64_t)phys * a.num_kv_heads + h) * kTile + slot) * D + lane * EPL;

#pragma unroll
    for (int side = 0; side < 2; ++side) {
        const void *nw = side ? a.v_new : a.k_new;
        void *cache = side ? a.v : a.k;
        float *scales = side ? a.v_scale : a.k_scale;
        float x[EPL];
        load_new<NEW_DT, EPL>(nw, src, lane, x);
        if constexpr (KV_DT == SS_F32) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) static_cast<float *>(cache)[dst + e] = x[e];
        } else if constexpr (KV_DT == SS_BF16) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) static_cast<uint16_t *>(cache)[dst + e] = to_bf16_rne(x[e]);
        } else {
            // A block whose slot 0 is written by this call takes a new scale, amax/448 over the new
            // tokens that land in it; every wavefront of the block computes the same value itself,
            // the one at slot 0 stores it.  A block that holds older tokens keeps its scale.
            float scale;
            if (blk * kTile >= P) {
                float amax = 0.f;
                const int i_lo = blk * kTile - P;                                  // first new token of the block
                const int i_hi = min(q_len, (blk + 1) * kTile - P);               // one past its last
                for (int j = i_lo; j < i_hi; ++j) {
                    float y[EPL];
                    load_new<NEW_DT, EPL>(nw, ((int64_t)(r0 + j) * a.num_kv_heads + h) * D, lane, y);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(y[e]));
                }
                for (int off = 32; off; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
                scale = amax > 0.f ? amax / kFp8Max : 1.0f;
                if (slot == 0 && lane == 0) scales[(int64_t)phys * a.num_kv_heads + h] = scale;
            } else {
                scale = scales[(int64_t)phys * a.num_kv_heads + h];
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) static_cast<uint8_t *>(cache)[dst + e] = to_e4m3_rne(x[e], scale);
        }
    }
}

__global__ __launch_bounds__(256) void kv_commit_kernel(int batch, const int32_t *q_indptr, const int32_t *accepted_len,
                                                         int32_t *kv_len)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= batch) return;
    const int k = q_indptr[b + 1] - q_indptr[b] - 1;
    kv_len[b] = kv_len[b] - k + accepted_len[b];   // the accepted drafts stay, the rejected slots fall past the end
}

// Compaction after acceptance over a draft tree: the accepted nodes a_1 < .. < a_n of a request move
// from cache positions P + a_j to P + j, where a chain would have put them.  grid: batch * kv heads,
// one wavefront each; a lane owns the same EPL elements of every token row, and walks the moves in
// path order, so its own loads and stores keep the order the moves need (a_j >= j: a move never reads
// a slot that an earlier one wrote).  e4m3 bytes that change block are rescaled from the source
// block's scale to the destination's.
template <int KV_DT, int EPL>
__global__ __launch_bounds__(64) void kv_compact_kernel(KvAppendArgs a, const int32_t *accepted_nodes,
                                                        const int32_t *accepted_len)
{
    typedef typename std::conditional<KV_DT == SS_F32, float,
                                      typename std::conditional<KV_DT == SS_BF16, uint16_t, uint8_t>::type>::type elem_t;
    const int lane = threadIdx.x;
    const int h = blockIdx.x % a.num_kv_heads, b = blockIdx.x / a.num_kv_heads;
    const int q_len = a.q_indptr[b + 1] - a.q_indptr[b];
    const int P = a.kv_len[b] - q_len;
    const int n = min(accepted_len[b], q_len - 1);
    const int D = a.head_dim;
    const int32_t *bt = a.block_table + (int64_t)b * a.max_blocks;
    int prev = 0;
    for (int j = 1; j <= n; ++j) {
        const int node = accepted_nodes[(int64_t)b * SS_MAX_DEPTH + j - 1];
        if (node <= prev || node >= q_len) break;   // not a path: leave the rest alone
        prev = node;
        if (node == j) continue;
        const int ps = P + node, pd = P + j;
        const int64_t blk_s = bt[ps / kTile], blk_d = bt[pd / kTile];
        const int64_t src = ((blk_s * a.num_kv_heads + h) * kTile + ps % kTile) * D + lane * EPL;
        const int64_t dst = ((blk_d * a.num_kv_heads + h) * kTile + pd % kTile) * D + lane * EPL;
#pragma unroll
        for (int side = 0; side < 2; ++side) {
            elem_t *cache = static_cast<elem_t *>(side ? a.v : a.k);
            elem_t x[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) x[e] = cache[src + e];
            if constexpr (KV_DT == SS_FP8_E4M3) {
                if (blk_s != blk_d) {
                    const float *scales = side ? a.v_scale : a.k_scale;
                    const float s_src = scales[blk_s * a.num_kv_heads + h], s_dst = scales[blk_d * a.num_kv_heads + h];
#pragma unroll
                    for (int e = 0; e < EPL; ++e)
                        x[e] = to_e4m3_rne(__builtin_amdgcn_cvt_f32_fp8((uint32_t)x[e], 0) * s_src, s_dst);
                }
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) cache[dst + e] = x[e];
        }
    }
}

template <int KV_DT, int NEW_DT>
int32_t launch_append(const KvAppendArgs &a, hipStream_t stream)
{
    const unsigned grid = (unsigned)a.batch * a.max_q_len * a.num_kv_heads;
    if (a.head_dim == 128)
        hipLaunchKernelGGL((kv_append_kernel<KV_DT, NEW_DT, 2>), dim3(grid), dim3(64), 0, stream, a);
    else
        hipLaunchKernelGGL((kv_append_kernel<KV_DT, NEW_DT, 1>), dim3(grid), dim3(64), 0, stream, a);
    SS_HIP_CHECK(hipGetLastError(), "launch kv_append_kernel");
    return SS_OK;
}

template <int KV_DT>
int32_t launch_append_kv(const KvAppendArgs &a, hipStream_t stream)
{
    if (a.new_dtype == SS_F32) return launch_append<KV_DT, SS_F32>(a, stream);
    return launch_append<KV_DT, SS_BF16>(a, stream);
}

}  // namespace

int32_t kv_append_launch(const KvAppendArgs &a, hipStream_t stream)
{
    if (a.batch == 0) return SS_OK;
    switch (a.kv_dtype) {
    case SS_F32: return launch_append_kv<SS_F32>(a, stream);
    case SS_BF16: return launch_append_kv<SS_BF16>(a, stream);
    default: return launch_append_kv<SS_FP8_E4M3>(a, stream);
    }
}

int32_t kv_compact_launch(const KvAppendArgs &a, const int32_t *accepted_nodes, const int32_t *accepted_len,
                          hipStream_t stream)
{
    if (a.batch == 0) return SS_OK;
    const dim3 grid((unsigned)a.batch * a.num_kv_heads), wg(64);
    const bool wide = a.head_dim == 128;
    switch (a.kv_dtype) {
    case SS_F32:
        if (wide) hipLaunchKernelGGL((kv_compact_kernel<SS_F32, 2>), grid, wg, 0, stream, a, accepted_nodes, accepted_len);
        else hipLaunchKernelGGL((kv_compact_kernel<SS_F32, 1>), grid, wg, 0, stream, a, accepted_nodes, accepted_len);
        break;
    case SS_BF16:
        if (wide) hipLaunchKernelGGL((kv_compact_kernel<SS_BF16, 2>), grid, wg, 0, stream, a, accepted_nodes, accepted_len);
        else hipLaunchKernelGGL((kv_compact_kernel<SS_BF16, 1>), grid, wg, 0, stream, a, accepted_nodes, accepted_len);
        break;
    default:
        if (wide) hipLaunchKernelGGL((kv_compact_kernel<SS_FP8_E4M3, 2>), grid, wg, 0, stream, a, accepted_nodes, accepted_len);
        else hipLaunchKernelGGL((kv_compact_kernel<SS_FP8_E4M3, 1>), grid, wg, 0, stream, a, accepted_nodes, accepted_len);
    }
    SS_HIP_CHECK(hipGetLastError(), "launch kv_compact_kernel");
    return SS_OK;
}

int32_t kv_commit_launch(int batch, const int32_t *q_indptr, const int32_t *accepted_len, int32_t *kv_len,
                         hipStream_t stream)
{
    if (batch == 0) return SS_OK;
    hipLaunchKernelGGL(kv_commit_kernel, dim3((unsigned)(batch + 255) / 256), dim3(256), 0, stream, batch, q_indptr,
                       accepted_len, kv_len);
    SS_HIP_CHECK(hipGetLastError(), "launch kv_commit_kernel");
    return SS_OK;
}

}  // namespace ss
