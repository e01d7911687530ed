// Pieces shared by the acceptance kernels (chain rule in accept.hip, sampled tree walk in accept_tree.hip):
// constants, the workspace carve-up of the row-statistics and resampling passes, vocabulary loads, block
// reductions with a fixed order and the fp64 exponential.
#pragma once

#include "common.h"

namespace ss {
namespace {

constexpr int kThreads = 256;
constexpr int kSub = 2048;                     // vocabulary entries per workgroup in the fp64 passes
constexpr int kSubPer = kSub / kThreads;       // 8 logits per lane there
constexpr int kMaxRows = 2 * SS_MAX_DEPTH + 1; // rows of one request: k+1 target, k draft
constexpr double kLog2eD = 1.4426950408889634;

struct RowPick {      // written by decide, read by the resampling passes
    int32_t p_row;    // target row the new token is drawn from
    int32_t q_row;    // draft row of the rejected position, -1 if every draft was accepted
    float m_p, m_q;   // exact row maxima
    float temperature;
    int32_t n;        // accepted length
    double rho;       // Zp/Zq as known from the fp32 row statistics (relative error below 2e-5)
};

constexpr int kAmbCap = 4096;       // listed boundary entries per request; beyond that the slow exact path runs
constexpr double kAmbEps = 1.0e-4;  // relative half-width of the boundary zone around p == q
constexpr int kPickWgs = 8;         // workgroups per request in the last pass (all but one idle unless the list overflowed)

struct Workspace {
    float *cmax, *csum;   // [rows][nchunks]
    int32_t *carg;        // [rows][nchunks]
    RowPick *pick;        // [batch]
    double *zp, *zq, *sc; // [batch][nsub]: sums of exp over all entries of the block (p row, q row), block mass
    double *pp, *qq;      // [batch][nsub]: the same sums over the entries with p clearly above q
    int32_t *amb_cnt;     // [batch] entries in the boundary zone (may exceed kAmbCap: then the list is not used)
    int32_t *done;        // [batch] workgroups of the last pass that have delivered their block masses
    int32_t *blk_base, *blk_cnt;  // [batch][nsub] where in the list a block's entries start, and how many they are
    double *amb_ep, *amb_eq;  // [batch][kAmbCap] their unnormalised exponentials, each block's entries contiguous
    int nchunks, nsub, rows;
};

__host__ __device__ inline int num_chunks(int vocab) { return (vocab + kChunk - 1) / kChunk; }
__host__ __device__ inline int num_sub(int vocab) { return (vocab + kSub - 1) / kSub; }

__host__ Workspace carve(void *ws, int batch, int total_rows, int vocab)
{
    Workspace w;
    w.nchunks = num_chunks(vocab);
    w.nsub = num_sub(vocab);
    w.rows = 2 * total_rows - batch;
    char *p = static_cast<char *>(ws);
    const size_t per = align_up(sizeof(float) * (size_t)w.rows * w.nchunks, 256);
    w.cmax = reinterpret_cast<float *>(p); p += per;
    w.csum = reinterpret_cast<float *>(p); p += per;
    w.carg = reinterpret_cast<int32_t *>(p); p += per;
    w.pick = reinterpret_cast<RowPick *>(p); p += align_up(sizeof(RowPick) * (size_t)batch, 256);
    const size_t perd = align_up(sizeof(double) * (size_t)batch * w.nsub, 256);
    w.zp = reinterpret_cast<double *>(p); p += perd;
    w.zq = reinterpret_cast<double *>(p); p += perd;
    w.sc = reinterpret_cast<double *>(p); p += perd;
    w.pp = reinterpret_cast<double *>(p); p += perd;
    w.qq = reinterpret_cast<double *>(p); p += perd;
    const size_t pera = align_up(sizeof(double) * (size_t)batch * kAmbCap, 256);
    w.amb_ep = reinterpret_cast<double *>(p); p += pera;
    w.amb_eq = reinterpret_cast<double *>(p); p += pera;
    const size_t peri = align_up(sizeof(int32_t) * (size_t)batch * w.nsub, 256);
    w.blk_base = reinterpret_cast<int32_t *>(p); p += peri;
    w.blk_cnt = reinterpret_cast<int32_t *>(p); p += peri;
    w.amb_cnt = reinterpret_cast<int32_t *>(p); p += align_up(sizeof(int32_t) * (size_t)batch, 256);
    w.done = reinterpret_cast<int32_t *>(p); p += align_up(sizeof(int32_t) * (size_t)batch, 256);
    return w;
}

// ---- loading one lane's share of a block of N*256 vocabulary entries -------------------------
// Coalesced order: lane t owns entries base + it*(256*vec) + t*vec + j (vec = 8 for bf16, 4 for f32).
// Sequential order (the inverse-CDF search): lane t owns base + t*N .. + N-1.
// Out-of-vocabulary positions read as -inf.  index_of() gives the vocabulary id of slot s.
// DT is the logit dtype (SS_BF16 or SS_F32): the kernels are compiled once per dtype.
template <int DT, int N, bool SEQ>
__device__ __forceinline__ int index_of(int base, int tid, int s)
{
    if (SEQ) return base + tid * N + s;
    constexpr int vec = DT == SS_BF16 ? 8 : 4;
    return base + (s / vec) * (kThreads * vec) + tid * vec + (s % vec);
}

template <int DT, int N, bool SEQ>
__device__ __forceinline__ void load_slots(const void *row, int vocab, int base, int tid, float (&x)[N])
{
    constexpr int vec = DT == SS_BF16 ? 8 : 4;
    if (base + N * kThreads <= vocab) {   // whole block inside the vocabulary (uniform): plain 16-byte loads
        uint4 w[N / vec];
#pragma unroll
        for (int it = 0; it < N / vec; ++it) {
            const int i0 = index_of<DT, N, SEQ>(base, tid, it * vec);
            if constexpr (DT == SS_BF16)
                w[it] = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(row) + i0);
            else
                w[it] = *reinterpret_cast<const uint4 *>(static_cast<const float *>(row) + i0);
        }
#pragma unroll
        for (int it = 0; it < N / vec; ++it) {
            const uint32_t ww[4] = {w[it].x, w[it].y, w[it].z, w[it].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (DT == SS_BF16) {
                    x[it * 8 + 2 * j] = __uint_as_float(ww[j] << 16);
                    x[it * 8 + 2 * j + 1] = __uint_as_float(ww[j] & 0xffff0000u);
                } else {
                    x[it * 4 + j] = __uint_as_float(ww[j]);
                }
            }
        }
        return;
    }
    // The block that holds the end of the vocabulary.  Every lane still issues 16-byte loads (from a
    // clamped, in-bounds address, so that they pipeline); lanes whose vector lies past the end drop
    // the data, and the one vector that straddles the end is read element by element.
    const int last_full = vocab >= vec ? (vocab - vec) / vec * vec : -1;
#pragma unroll
    for (int it = 0; it < N / vec; ++it) {
        const int i0 = index_of<DT, N, SEQ>(base, tid, it * vec);
        uint4 w = make_uint4(0, 0, 0, 0);
        if (last_full >= 0) {
            const int ic = i0 < last_full ? i0 : last_full;
            if constexpr (DT == SS_BF16)
                w = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(row) + ic);
            else
                w = *reinterpret_cast<const uint4 *>(static_cast<const float *>(row) + ic);
        }
        const bool whole = i0 + vec <= vocab;
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (DT == SS_BF16) {
                x[it * 8 + 2 * j] = whole ? __uint_as_float(ww[j] << 16) : -INFINITY;
                x[it * 8 + 2 * j + 1] = whole ? __uint_as_float(ww[j] & 0xffff0000u) : -INFINITY;
            } else {
                x[it * 4 + j] = whole ? __uint_as_float(ww[j]) : -INFINITY;
            }
        }
        if (!whole && i0 < vocab) {
#pragma unroll
            for (int j = 0; j < vec; ++j) {
                if (i0 + j < vocab) {
                    if constexpr (DT == SS_BF16)
                        x[it * vec + j] = __uint_as_float((uint32_t) static_cast<const uint16_t *>(row)[i0 + j] << 16);
                    else
                        x[it * vec + j] = static_cast<const float *>(row)[i0 + j];
                }
            }
        }
    }
}

__device__ __forceinline__ const void *row_ptr(const void *base, int64_t row, int64_t stride, int dtype)
{
    return static_cast<const char *>(base) + row * stride * (dtype == SS_BF16 ? 2 : 4);
}

__device__ __forceinline__ float load_logit(const void *base, int64_t row, int64_t stride, int dtype, int v)
{
    const void *r = row_ptr(base, row, stride, dtype);
    if (dtype == SS_BF16) return __uint_as_float((uint32_t) static_cast<const uint16_t *>(r)[v] << 16);
    return static_cast<const float *>(r)[v];
}

// ---- block reductions with a fixed order ---------------------------------------------------
__device__ __forceinline__ float block_max(float v, float *sh)
{
    for (int off = 32; off; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}
template <typename T>
__device__ __forceinline__ T block_sum(T v, T *sh)
{
    for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// ---- fp64 exponential for non-positive arguments -----------------------------------------------
// exp(x) = 2^e * 2^(j/64) * exp(r), x = (64 e + j) ln2/64 + r, |r| <= ln2/128, with a 64-entry
// table of 2^(j/64) in LDS and a degree-5 Taylor polynomial (remainder < 4e-17 relative).
// 2^(j/64), j = 0..63, each the double nearest to the exact value (tests/test_exp_table.py recomputes them)
static __device__ const double kExp2Sixtyfourths[64] = {
    0x1.0000000000000p+0, 0x1.02c9a3e778061p+0, 0x1.059b0d3158574p+0, 0x1.0874518759bc8p+0,
    0x1.0b5586cf9890fp+0, 0x1.0e3ec32d3d1a2p+0, 0x1.11301d0125b51p+0, 0x1.1429aaea92de0p+0,
    0x1.172b83c7d517bp+0, 0x1.1a35beb6fcb75p+0, 0x1.1d4873168b9aap+0, 0x1.2063b88628cd6p+0,
    0x1.2387a6e756238p+0, 0x1.26b4565e27cddp+0, 0x1.29e9df51fdee1p+0, 0x1.2d285a6e4030bp+0,
    0x1.306fe0a31b715p+0, 0x1.33c08b26416ffp+0, 0x1.371a7373aa9cbp+0, 0x1.3a7db34e59ff7p+0,
    0x1.3dea64c123422p+0, 0x1.4160a21f72e2ap+0, 0x1.44e086061892dp+0, 0x1.486a2b5c13cd0p+0,
    0x1.4bfdad5362a27p+0, 0x1.4f9b2769d2ca7p+0, 0x1.5342b569d4f82p+0, 0x1.56f4736b527dap+0,
    0x1.5ab07dd485429p+0, 0x1.5e76f15ad2148p+0, 0x1.6247eb03a5585p+0, 0x1.6623882552225p+0,
    0x1.6a09e667f3bcdp+0, 0x1.6dfb23c651a2fp+0, 0x1.71f75e8ec5f74p+0, 0x1.75feb564267c9p+0,
    0x1.7a11473eb0187p+0, 0x1.7e2f336cf4e62p+0, 0x1.82589994cce13p+0, 0x1.868d99b4492edp+0,
    0x1.8ace5422aa0dbp+0, 0x1.8f1ae99157736p+0, 0x1.93737b0cdc5e5p+0, 0x1.97d829fde4e50p+0,
    0x1.9c49182a3f090p+0, 0x1.a0c667b5de565p+0, 0x1.a5503b23e255dp+0, 0x1.a9e6b5579fdbfp+0,
    0x1.ae89f995ad3adp+0, 0x1.b33a2b84f15fbp+0, 0x1.b7f76f2fb5e47p+0, 0x1.bcc1e904bc1d2p+0,
    0x1.c199bdd85529cp+0, 0x1.c67f12e57d14bp+0, 0x1.cb720dcef9069p+0, 0x1.d072d4a07897cp+0,
    0x1.d5818dcfba487p+0, 0x1.da9e603db3285p+0, 0x1.dfc97337b9b5fp+0, 0x1.e502ee78b3ff6p+0,
    0x1.ea4afa2a490dap+0, 0x1.efa1bee615a27p+0, 0x1.f50765b6e4540p+0, 0x1.fa7c1819e90d8p+0,
};

struct ExpTable {
    double t[64];
    __device__ void init()
    {
        if (threadIdx.x < 64) t[threadIdx.x] = kExp2Sixtyfourths[threadIdx.x];
        __syncthreads();
    }
    __device__ __forceinline__ double operator()(double x) const
    {
        x = fmax(x, -746.0);   // exp underflows to 0 from there on (also covers -inf)
        const double kd = rint(x * 92.33248261689366);  // 64 / ln 2
        double r = fma(kd, -0x1.62e42fee00000p-7, x);    // ln2/64: high part with 21 trailing zero bits
        r = fma(kd, -0x1.a39ef35793c76p-39, r);          //         low part
        const int k = (int)kd;
        const double p = fma(fma(fma(fma(fma(r, 1.0 / 120.0, 1.0 / 24.0), r, 1.0 / 6.0), r, 0.5), r, 1.0), r, 1.0);
        return ldexp(t[k & 63] * p, k >> 6);
    }
};


}  // namespace
}  // namespace ss
