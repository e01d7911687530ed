// spec_accept: acceptance walk and resampling over full-vocabulary logits.
//
// Pass 1 (rowstats) streams every target and draft row once (the HBM-bound part): per
// 8192-entry chunk it leaves the chunk maximum and the sum of exp2((x - max) * log2e/T) in fp32
// (greedy mode: maximum and lowest-index argmax of target rows only).
// decide      one workgroup per request merges the chunk statistics of all its rows in parallel,
//             evaluates u < p/q for every draft in fp64 and fixes the accepted length and the
//             row(s) the new token is drawn from; in greedy mode it compares arg-maxima instead,
//             along the chain or, given parent pointers, down a draft tree.
// Passes 2a-2b touch only those one or two rows per request and work in fp64, so that the drawn
// token can be reproduced by an fp64 reference.  2a leaves, per 2048-entry block, the sums of the
// unnormalised exponentials of both rows (the exact normalisers Zp, Zq once added up) and the same
// sums restricted to the entries whose residual p - q is positive; which entries those are follows
// from Zp/Zq as known from pass 1, except for entries within 1e-4 of the boundary, which are set
// aside in a list (each block's entries contiguous).  2b turns the sums into block masses
// P/Zp - Q/Zq, adds the listed entries with the exact normalisers, and does the inverse-CDF search
// inside the block that holds u * mass.
// All reductions have a fixed order (no atomics): results are run-to-run identical.
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
struct ExpTable {
    double t[64];
    __device__ void init()
    {
        if (threadIdx.x < 64) t[threadIdx.x] = exp2((double)threadIdx.x * (1.0 / 64.0));
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

// ---- pass 1 ---------------------------------------------------------------------------------
// grid: batch * rows_max * ceil(nchunks / 4), rows_max from the caller's bound of k+1; workgroup (b, j, group): wave wv of it streams chunk
// 4 * group + wv of request b's row j (j <= k: target row j; k < j <= 2k: draft row j-k-1; larger j:
// nothing to do).  A wave owns its chunk alone: all of its 16-byte loads go out first, then the
// values are folded vector by vector into a per-lane running (max, sum) and reduced across the wave
// with shuffles, so the streaming pass has no barrier and no LDS traffic.
template <int DT>
__device__ __forceinline__ void unpack(const uint4 &w, float (&x)[DT == SS_BF16 ? 8 : 4])
{
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if constexpr (DT == SS_BF16) {
            x[2 * j] = __uint_as_float(ww[j] << 16);
            x[2 * j + 1] = __uint_as_float(ww[j] & 0xffff0000u);
        } else {
            x[j] = __uint_as_float(ww[j]);
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kThreads) void accept_rowstats_kernel(AcceptArgs a, Workspace w)
{
    constexpr int vec = DT == SS_BF16 ? 8 : 4;       // logits per 16-byte load
    constexpr int NV = kChunk / (64 * vec);          // loads per lane and chunk
    constexpr int STEP = 4;                          // vectors folded per update of the running maximum
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int groups = (w.nchunks + 3) / 4;
    const int chunk = (blockIdx.x % groups) * 4 + wv;
    const int rows_max = a.greedy ? a.max_q_len : 2 * a.max_q_len - 1;   // rows a request can have
    const int bj = blockIdx.x / groups, b = bj / rows_max, j = bj % rows_max;
    const int t0 = a.q_indptr[b], k = a.q_indptr[b + 1] - t0 - 1;
    if (j > (a.greedy ? k : 2 * k) || chunk >= w.nchunks) return;
    const bool is_draft = j > k;
    const int r = is_draft ? t0 - b + (j - k - 1) : t0 + j;
    const int64_t ry = is_draft ? (int64_t)a.total_rows + r : r;
    const void *row = row_ptr(is_draft ? a.draft : a.target, r, a.row_stride, DT);
    const int base = chunk * kChunk;
    const int64_t o = ry * w.nchunks + chunk;
    const float T = a.greedy ? 1.f : (a.temperature ? a.temperature[b] : a.temperature_scalar);
    const float sc = 1.4426950408889634f / T;

    // vector v of this lane starts at vocabulary id base + v * (64 * vec) + lane * vec
    uint4 raw[NV];
    const bool full = base + kChunk <= a.vocab;       // uniform: the chunk lies inside the vocabulary
    const int last_full = a.vocab >= vec ? (a.vocab - vec) / vec * vec : -1;
    if (full) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int i0 = base + v * (64 * vec) + lane * vec;
            raw[v] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(row) + (int64_t)i0 * (DT == SS_BF16 ? 2 : 4));
        }
    } else {
        // the chunk that holds the end of the vocabulary: loads from a clamped, in-bounds address
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int i0 = base + v * (64 * vec) + lane * vec;
            const int ic = i0 < last_full ? i0 : last_full;
            raw[v] = make_uint4(0, 0, 0, 0);
            if (last_full >= 0)
                raw[v] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(row) + (int64_t)ic * (DT == SS_BF16 ? 2 : 4));
        }
    }

    float m = -INFINITY, z = 0.f;
    int best = 0x7fffffff;
#pragma unroll
    for (int s0 = 0; s0 < NV; s0 += STEP) {
        float x[STEP][vec];
#pragma unroll
        for (int v = 0; v < STEP; ++v) {
            unpack<DT>(raw[s0 + v], x[v]);
            if (!full) {
                const int i0 = base + (s0 + v) * (64 * vec) + lane * vec;
                if (i0 + vec > a.vocab) {   // past the end, or the one vector that straddles it
#pragma unroll
                    for (int e = 0; e < vec; ++e) {
                        float val = -INFINITY;
                        if (i0 + e < a.vocab) {
                            if constexpr (DT == SS_BF16)
                                val = __uint_as_float((uint32_t) static_cast<const uint16_t *>(row)[i0 + e] << 16);
                            else
                                val = static_cast<const float *>(row)[i0 + e];
                        }
                        x[v][e] = val;
                    }
                }
            }
        }
        float mx = x[0][0];
#pragma unroll
        for (int v = 0; v < STEP; ++v)
#pragma unroll
            for (int e = 0; e < vec; ++e) mx = fmaxf(mx, x[v][e]);
        if (a.greedy) {
            if (mx > m) {   // a new maximum: its first position within this step, ids ascend with (v, e)
                m = mx;
                best = 0x7fffffff;
#pragma unroll
                for (int v = STEP - 1; v >= 0; --v)
#pragma unroll
                    for (int e = vec - 1; e >= 0; --e)
                        if (x[v][e] == mx) best = base + (s0 + v) * (64 * vec) + lane * vec + e;
            }
        } else {
            const float m_new = fmaxf(m, mx);
            if (m_new != -INFINITY) {
                float acc = 0.f;
#pragma unroll
                for (int v = 0; v < STEP; ++v)
#pragma unroll
                    for (int e = 0; e < vec; ++e) acc += __builtin_amdgcn_exp2f((x[v][e] - m_new) * sc);
                z = z * __builtin_amdgcn_exp2f((m - m_new) * sc) + acc;   // m == -inf: z is 0 and the factor 0
                m = m_new;
            }
        }
    }
    // across the wave
    float cm = m;
    for (int off = 32; off; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off));
    if (a.greedy) {
        int arg = m == cm ? best : 0x7fffffff;   // lowest vocabulary id holding the chunk maximum
        for (int off = 32; off; off >>= 1) arg = min(arg, __shfl_xor(arg, off));
        if (lane == 0) {
            w.cmax[o] = cm;
            w.carg[o] = arg;
        }
        return;
    }
    if (m != -INFINITY) z *= __builtin_amdgcn_exp2f((m - cm) * sc);
    for (int off = 32; off; off >>= 1) z += __shfl_xor(z, off);
    if (lane == 0) {
        w.cmax[o] = cm;
        w.csum[o] = z;
    }
}

// ---- decide ---------------------------------------------------------------------------------
// One 256-lane workgroup per request.  Wave wv merges the chunk statistics of rows wv, wv+4, ...
// (lanes over chunks), then lanes 0..k-1 of wave 0 evaluate their draft and a ballot finds the
// first rejection.
__global__ __launch_bounds__(kThreads) void accept_decide_kernel(AcceptArgs a, Workspace w)
{
    __shared__ float row_m[kMaxRows];
    __shared__ double row_z[kMaxRows];
    __shared__ int row_arg[kMaxRows];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = a.q_indptr[b], k = a.q_indptr[b + 1] - t0 - 1, d0 = t0 - b;
    const float T = a.temperature ? a.temperature[b] : a.temperature_scalar;
    const double inv_t = a.greedy ? 1.0 : 1.0 / (double)T;
    const int nrows = a.greedy ? k + 1 : 2 * k + 1;

    // Wave 0's gathers (draft token, then its two logits) depend on nothing the row merge below
    // produces: they are requested first so that their latency runs under it.
    int x_early = -1;
    float lp_early = 0.f, lq_early = 0.f, u_early = 0.f;
    if (wave == 0 && lane < k && !a.tree_parent) {
        x_early = a.draft_tokens[d0 + lane];
        if (!a.greedy) {
            lp_early = load_logit(a.target, t0 + lane, a.row_stride, a.logit_dtype, x_early);
            lq_early = load_logit(a.draft, d0 + lane, a.row_stride, a.logit_dtype, x_early);
            u_early = a.u_accept[d0 + lane];
        }
    }

    for (int j = wave; j < nrows; j += 4) {
        const int64_t ry = j <= k ? (int64_t)t0 + j : (int64_t)a.total_rows + d0 + (j - k - 1);
        float m = -INFINITY;
        for (int c = lane; c < w.nchunks; c += 64) m = fmaxf(m, w.cmax[ry * w.nchunks + c]);
        for (int off = 32; off; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
        if (a.greedy) {
            int best = 0x7fffffff;
            for (int c = lane; c < w.nchunks; c += 64)
                if (w.cmax[ry * w.nchunks + c] == m) best = min(best, w.carg[ry * w.nchunks + c]);
            for (int off = 32; off; off >>= 1) best = min(best, __shfl_xor(best, off));
            if (lane == 0) row_arg[j] = best;
        } else {
            double z = 0.0;
            for (int c = lane; c < w.nchunks; c += 64) {
                const float cm = w.cmax[ry * w.nchunks + c];
                if (cm != -INFINITY)
                    z += (double)w.csum[ry * w.nchunks + c] * exp2(((double)cm - (double)m) * inv_t * kLog2eD);
            }
            for (int off = 32; off; off >>= 1) z += __shfl_xor(z, off);
            if (lane == 0) {
                row_m[j] = m;
                row_z[j] = z;
            }
        }
    }
    __syncthreads();
    if (wave != 0) return;

    if (a.tree_parent) {
        // Greedy walk over a draft tree: lane i holds node i (1..k) with its parent and token; each
        // step a ballot finds the lowest-numbered child of the current node that carries the token
        // greedy decoding emits there.
        const int par = (lane >= 1 && lane <= k) ? a.tree_parent[t0 + lane] : -2;
        const int x = (lane >= 1 && lane <= k) ? a.draft_tokens[d0 + lane - 1] : -1;
        int cur = 0, n = 0, my_tok = -1, my_node = -1;
        for (;;) {   // at most k steps: every step moves to a higher-numbered node
            const int t = row_arg[cur];
            const unsigned long long hit = __ballot(par == cur && x == t);
            if (!hit) break;
            cur = __ffsll((long long)hit) - 1;
            if (lane == n) {
                my_tok = t;
                my_node = cur;
            }
            ++n;
        }
        if (lane == n) my_tok = row_arg[cur];
        if (lane < SS_OUT_WIDTH) a.out_tokens[(int64_t)b * SS_OUT_WIDTH + lane] = my_tok;
        if (lane < SS_MAX_DEPTH) a.accepted_nodes[(int64_t)b * SS_MAX_DEPTH + lane] = my_node;
        if (lane == 0) a.accepted_len[b] = n;
        return;
    }

    // every draft in parallel: lane i judges draft i
    bool reject = false;
    int x = -1;
    if (lane < k) {
        x = x_early;
        if (a.greedy) {
            reject = row_arg[lane] != x;
        } else {
            const double lp = lp_early, lq = lq_early;
            // p(x)/q(x) = exp((lp-mp)/T - (lq-mq)/T) * Zq/Zp
            const double e = (lp - (double)row_m[lane]) * inv_t - (lq - (double)row_m[k + 1 + lane]) * inv_t;
            const double rho = exp(e) * (row_z[k + 1 + lane] / row_z[lane]);
            if (a.ratio_out) a.ratio_out[d0 + lane] = (float)rho;
            reject = !((double)u_early < rho);
        }
    }
    const unsigned long long rej = __ballot(reject);
    const int n = rej ? __ffsll((long long)rej) - 1 : k;   // first rejection, k if none
    if (lane < SS_OUT_WIDTH) {
        int tok = lane < n ? x : -1;
        if (a.greedy && lane == n) tok = row_arg[n];
        a.out_tokens[(int64_t)b * SS_OUT_WIDTH + lane] = tok;   // slot n is filled by pass 2b when sampling
    }
    if (lane == 0) {
        a.accepted_len[b] = n;
        if (!a.greedy) {
            RowPick pk;
            pk.p_row = t0 + n;
            pk.q_row = n < k ? d0 + n : -1;
            pk.m_p = row_m[n];
            pk.m_q = n < k ? row_m[k + 1 + n] : 0.f;
            pk.temperature = T;
            pk.n = n;
            pk.rho = n < k ? row_z[n] / row_z[k + 1 + n] : 1.0;
            w.pick[b] = pk;
            w.amb_cnt[b] = 0;
            w.done[b] = 0;
        }
    }
}

// ---- pass 2a: fp64 sums per block -------------------------------------------------------------
// N sums in one go (fixed order): lanes, then the four waves.
template <int N>
__device__ __forceinline__ void block_sums(double (&v)[N], double (*sh)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i)
        for (int off = 32; off; off >>= 1) v[i] += __shfl_xor(v[i], off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) sh[threadIdx.x >> 6][i] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = (sh[0][i] + sh[1][i]) + (sh[2][i] + sh[3][i]);
}

template <int DT>
__global__ __launch_bounds__(kThreads) void accept_norm_kernel(AcceptArgs a, Workspace w)
{
    __shared__ double sh[4];
    __shared__ double sh5[4][5];
    __shared__ ExpTable ex;
    ex.init();
    const int sub = blockIdx.x % w.nsub, b = blockIdx.x / w.nsub, tid = threadIdx.x;
    const RowPick pk = w.pick[b];
    const double inv_t = 1.0 / (double)pk.temperature;
    const int64_t o = (int64_t)b * w.nsub + sub;
    float xp[kSubPer], xq[kSubPer];
    load_slots<DT, kSubPer, false>(row_ptr(a.target, pk.p_row, a.row_stride, DT), a.vocab, sub * kSub, tid, xp);
    if (pk.q_row < 0) {   // bonus distribution: only the normaliser of the target row is needed
        double z = 0.0;
#pragma unroll
        for (int s = 0; s < kSubPer; ++s) z += ex(((double)xp[s] - (double)pk.m_p) * inv_t);
        z = block_sum<double>(z, sh);
        if (tid == 0) w.zp[o] = z;
        return;
    }
    load_slots<DT, kSubPer, false>(row_ptr(a.draft, pk.q_row, a.row_stride, DT), a.vocab, sub * kSub, tid, xq);
    // v[0], v[1]: exponentials of all entries (p row, q row); v[2], v[3]: of the entries whose residual
    // p - q is positive for certain, i.e. ep / eq above rho by more than the boundary zone
    double v[5] = {0.0, 0.0, 0.0, 0.0, 0.0};   // [4]: how many entries of the block are too close to call
    const double hi = pk.rho * (1.0 + kAmbEps), lo = pk.rho * (1.0 - kAmbEps);
    unsigned near = 0;   // slots of this lane that are too close to call before Zp/Zq are exact
#pragma unroll
    for (int s = 0; s < kSubPer; ++s) {
        const double ep = ex(((double)xp[s] - (double)pk.m_p) * inv_t);
        const double eq = ex(((double)xq[s] - (double)pk.m_q) * inv_t);
        v[0] += ep;
        v[1] += eq;
        if (ep > hi * eq) {
            v[2] += ep;
            v[3] += eq;
        } else if (ep > 0.0 && ep >= lo * eq) {
            near |= 1u << s;
        }
    }
    // The boundary entries of this block go to the request's list as one contiguous run, in lane and
    // slot order (so their later additions have a fixed order); one counter update per block.
    __shared__ int wave_cnt[4], run_base;
    const int mine = __popc(near);
    v[4] = (double)mine;
    block_sums<5>(v, sh5);
    const int total = (int)v[4];
    if (tid == 0) {
        w.zp[o] = v[0];
        w.zq[o] = v[1];
        w.pp[o] = v[2];
        w.qq[o] = v[3];
        w.blk_cnt[o] = total;
    }
    if (total > 0) {
        int incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(incl, off);
            if ((tid & 63) >= off) incl += t;
        }
        if ((tid & 63) == 63) wave_cnt[tid >> 6] = incl;
        __syncthreads();
        int before = 0;
        for (int wv = 0; wv < (tid >> 6); ++wv) before += wave_cnt[wv];
        if (tid == 0) {
            run_base = atomicAdd(&w.amb_cnt[b], total);
            w.blk_base[o] = run_base;
        }
        __syncthreads();
        if (run_base + total <= kAmbCap) {
            int64_t l = (int64_t)b * kAmbCap + run_base + before + (incl - mine);
#pragma unroll
            for (int s = 0; s < kSubPer; ++s) {
                if (near & (1u << s)) {
                    // evaluated again rather than kept (the same bits): keeping sixteen doubles per lane
                    // alive for this rare branch would halve the kernel's occupancy
                    float yp = xp[s], yq = xq[s];
                    asm volatile("" : "+v"(yp), "+v"(yq));
                    w.amb_ep[l] = ex(((double)yp - (double)pk.m_p) * inv_t);
                    w.amb_eq[l] = ex(((double)yq - (double)pk.m_q) * inv_t);
                    ++l;
                }
            }
        }
    }
}

// Sum of v[0..n) with a fixed association (lane-strided partial sums, then the block tree): every
// workgroup that calls it on the same array gets the same bits.
__device__ __forceinline__ double block_total(const double *v, int n, double *sh)
{
    double s = 0.0;
    for (int c = threadIdx.x; c < n; c += kThreads) s += v[c];
    return block_sum<double>(s, sh);
}

// residual (or bonus) mass of one vocabulary entry
__device__ __forceinline__ double mass(const ExpTable &ex, float lp, float lq, const RowPick &pk, double inv_t,
                                       double inv_zp, double inv_zq)
{
    const double p = ex(((double)lp - (double)pk.m_p) * inv_t) * inv_zp;
    if (pk.q_row < 0) return p;
    const double q = ex(((double)lq - (double)pk.m_q) * inv_t) * inv_zq;
    return p > q ? p - q : 0.0;
}

// ---- pass 2b: block masses and inverse-CDF search ------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(kThreads) void accept_pick_kernel(AcceptArgs a, Workspace w)
{
    __shared__ double wave_tot[4];
    __shared__ int sh_first[4], sh_last[4];
    __shared__ float sh_f[4];
    __shared__ ExpTable ex;
    const int b = blockIdx.x / kPickWgs, part = blockIdx.x % kPickWgs;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowPick pk = w.pick[b];
    int32_t *dst = a.out_tokens + (int64_t)b * SS_OUT_WIDTH + pk.n;
    // block masses live in LDS unless the vocabulary has more blocks than fit there
    constexpr int kScCap = 1024;
    __shared__ double sc_sh[kScCap];
    __shared__ double sh4[4][4];
    const int64_t ob = (int64_t)b * w.nsub;
    // everything that does not depend on anything else is requested up front
    const float u_s = a.u_sample[b];
    const int namb = pk.q_row >= 0 ? w.amb_cnt[b] : 0;
    const bool listed = namb <= kAmbCap;
    if (listed && part != 0) return;   // one workgroup does the whole request unless the list overflowed
    double *sc = listed && w.nsub <= kScCap ? sc_sh : w.sc + ob;
    const bool own = tid < w.nsub;
    const double zp0 = own ? w.zp[ob + tid] : 0.0;
    const double zq0 = own && pk.q_row >= 0 ? w.zq[ob + tid] : 0.0;
    const double pp0 = own && pk.q_row >= 0 ? w.pp[ob + tid] : 0.0;
    const double qq0 = own && pk.q_row >= 0 ? w.qq[ob + tid] : 0.0;
    const int cnt0 = own && pk.q_row >= 0 ? w.blk_cnt[ob + tid] : 0;       // this lane's block: its listed run
    const int base0 = own && pk.q_row >= 0 ? w.blk_base[ob + tid] : 0;
    ex.init();

    // exact normalisers, then the mass of every block
    double tot[4] = {zp0, zq0, 0.0, 0.0};
    for (int c = tid + kThreads; c < w.nsub; c += kThreads) {
        tot[0] += w.zp[ob + c];
        if (pk.q_row >= 0) tot[1] += w.zq[ob + c];
    }
    block_sums<4>(tot, sh4);
    const double zp = tot[0], zq = pk.q_row >= 0 ? tot[1] : 1.0;
    const double inv_t = 1.0 / (double)pk.temperature, inv_zp = 1.0 / zp, inv_zq = 1.0 / zq;
    if (pk.q_row < 0) {
        if (own) sc[tid] = zp0 / zp;
        for (int c = tid + kThreads; c < w.nsub; c += kThreads) sc[c] = w.zp[ob + c] / zp;
    } else if (listed) {
        if (own) {
            const double m = pp0 * inv_zp - qq0 * inv_zq;
            sc[tid] = m > 0.0 ? m : 0.0;
        }
        for (int c = tid + kThreads; c < w.nsub; c += kThreads) {
            const double m = w.pp[ob + c] * inv_zp - w.qq[ob + c] * inv_zq;
            sc[c] = m > 0.0 ? m : 0.0;
        }
        if (namb > 0) {
            // The listed boundary entries, now that Zp and Zq are exact: lane c adds block c's run in its stored order.
            __syncthreads();
            for (int c = tid; c < w.nsub; c += kThreads) {
                const int cnt = c == tid ? cnt0 : w.blk_cnt[ob + c];
                if (cnt > 0) {
                    const int64_t l0 = (int64_t)b * kAmbCap + (c == tid ? base0 : w.blk_base[ob + c]);
                    double add = 0.0;
                    for (int e = 0; e < cnt; ++e) {
                        const double r = w.amb_ep[l0 + e] * inv_zp - w.amb_eq[l0 + e] * inv_zq;
                        add += r > 0.0 ? r : 0.0;
                    }
                    sc[c] += add;
                }
            }
        }
    } else {
        // Too many entries near p == q to list (rows that nearly coincide, or many equal logit pairs on
        // the boundary): the request's workgroups share the blocks and compute every mass entry by
        // entry; the last one to deliver (a counter in device memory) goes on to draw the token.
        for (int c = part; c < w.nsub; c += kPickWgs) {
            float yp[kSubPer], yq[kSubPer];
            load_slots<DT, kSubPer, false>(row_ptr(a.target, pk.p_row, a.row_stride, DT), a.vocab, c * kSub, tid, yp);
            load_slots<DT, kSubPer, false>(row_ptr(a.draft, pk.q_row, a.row_stride, DT), a.vocab, c * kSub, tid, yq);
            double m = 0.0;
#pragma unroll
            for (int i = 0; i < kSubPer; ++i) m += mass(ex, yp[i], yq[i], pk, inv_t, inv_zp, inv_zq);
            m = block_sum<double>(m, wave_tot);
            if (tid == 0) sc[c] = m;
        }
        __shared__ int ticket_sh;
        __threadfence();   // the masses are out before the counter moves
        __syncthreads();
        if (tid == 0) ticket_sh = atomicAdd(&w.done[b], 1);
        __syncthreads();
        if (ticket_sh != kPickWgs - 1) return;
        __threadfence();   // and the other workgroups' masses are read from memory, not from a stale cache line
    }
    __threadfence_block();
    __syncthreads();

    // Inclusive scan of the block masses in index order (lane c holds block c; vocabularies beyond
    // 256 blocks take several rounds), first for the total S, then again to find the first block
    // with mass whose running sum exceeds u * S, together with the mass in front of it.
    __shared__ double scan_tot[4];
    __shared__ double carry_sh, prefix_sh;
    __shared__ int cstar_sh, lastpos_sh;
    double S = 0.0;
    int cand = 0x7fffffff, last = -1;
    double cand_prefix = 0.0, last_prefix = 0.0;
    for (int pass = 0; pass < 2; ++pass) {
        const double thr0 = (double)u_s * S;
        __syncthreads();
        if (tid == 0) { carry_sh = 0.0; cstar_sh = 0x7fffffff; lastpos_sh = -1; }
        __syncthreads();
        for (int base = 0; base < w.nsub; base += kThreads) {
            const int c = base + tid;
            const double v = c < w.nsub ? sc[c] : 0.0;
            double incl = v;
            for (int off = 1; off < 64; off <<= 1) {
                const double t = __shfl_up(incl, off);
                if (lane >= off) incl += t;
            }
            if (lane == 63) scan_tot[wave] = incl;
            __syncthreads();
            double before = carry_sh;
            for (int wv = 0; wv < wave; ++wv) before += scan_tot[wv];
            const double cum = before + incl;   // running sum through block c
            if (pass == 1 && v > 0.0) {
                if (cum > thr0 && c < cand) { cand = c; cand_prefix = cum - v; }
                last = c;
                last_prefix = cum - v;
            }
            __syncthreads();
            if (tid == kThreads - 1) carry_sh = cum;
            __syncthreads();
        }
        if (pass == 0) S = carry_sh;
        if (!(S > 0.0)) break;
    }
    if (!(S > 0.0)) {
        // p_n == q_n exactly: no residual mass; fall back to the lowest-index argmax of the target row
        float best = -INFINITY;
        for (int v = tid; v < a.vocab; v += kThreads)
            best = fmaxf(best, load_logit(a.target, pk.p_row, a.row_stride, DT, v));
        best = block_max(best, sh_f);
        int arg = 0x7fffffff;
        for (int v = tid; v < a.vocab; v += kThreads)
            if (load_logit(a.target, pk.p_row, a.row_stride, DT, v) == best) { arg = v; break; }
        for (int off = 32; off; off >>= 1) arg = min(arg, __shfl_xor(arg, off));
        if (lane == 0) sh_first[wave] = arg;
        __syncthreads();
        if (tid == 0) *dst = min(min(sh_first[0], sh_first[1]), min(sh_first[2], sh_first[3]));
        return;
    }
    atomicMin(&cstar_sh, cand);
    atomicMax(&lastpos_sh, last);
    __syncthreads();
    const bool take_last = cstar_sh == 0x7fffffff;  // rounding left u*S at or past the total: last entry with mass
    const int cstar = take_last ? lastpos_sh : cstar_sh;
    if (!take_last && cand == cstar) prefix_sh = cand_prefix;
    if (take_last && last == cstar) prefix_sh = last_prefix;
    __syncthreads();   // publishes prefix_sh
    const double thr = (double)u_s * S;
    const double prefix = prefix_sh;
    float xp[kSubPer], xq[kSubPer];
    load_slots<DT, kSubPer, true>(row_ptr(a.target, pk.p_row, a.row_stride, DT), a.vocab, cstar * kSub, tid, xp);
    if (pk.q_row >= 0)
        load_slots<DT, kSubPer, true>(row_ptr(a.draft, pk.q_row, a.row_stride, DT), a.vocab, cstar * kSub, tid, xq);
    else {
#pragma unroll
        for (int i = 0; i < kSubPer; ++i) xq[i] = 0.f;
    }
    double r[kSubPer];
    double local = 0.0;
    int my_last = -1;
#pragma unroll
    for (int i = 0; i < kSubPer; ++i) {
        r[i] = mass(ex, xp[i], xq[i], pk, inv_t, inv_zp, inv_zq);
        local += r[i];
        if (r[i] > 0.0) my_last = cstar * kSub + tid * kSubPer + i;
    }
    // exclusive prefix of `local` over lanes in index order
    double incl = local;
    for (int off = 1; off < 64; off <<= 1) {
        const double t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    double before = prefix;
    for (int wv = 0; wv < wave; ++wv) before += wave_tot[wv];
    const double excl = before + (incl - local);
    // first lane whose running sum crosses the threshold
    const bool crosses = !take_last && (excl + local > thr);
    const unsigned long long bal = __ballot(crosses);
    if (lane == 0) sh_first[wave] = bal ? wave * 64 + (__ffsll((long long)bal) - 1) : 0x7fffffff;
    int lw = my_last;
    for (int off = 32; off; off >>= 1) lw = max(lw, __shfl_xor(lw, off));
    if (lane == 0) sh_last[wave] = lw;
    __syncthreads();
    const int first = min(min(sh_first[0], sh_first[1]), min(sh_first[2], sh_first[3]));
    const int last_tok = max(max(sh_last[0], sh_last[1]), max(sh_last[2], sh_last[3]));
    if (first == 0x7fffffff) {
        if (tid == 0) *dst = last_tok;
        return;
    }
    if (tid == first) {
        double c = excl;
        int tok = -1;
#pragma unroll
        for (int i = 0; i < kSubPer; ++i) {
            if (r[i] > 0.0) {
                c += r[i];
                if (tok < 0 && c > thr) tok = cstar * kSub + tid * kSubPer + i;
            }
        }
        // the lane total crossed but the element-wise sum may round differently: then its last entry with mass
        *dst = tok >= 0 ? tok : my_last;
    }
}

// ---- sampled acceptance over a draft tree ------------------------------------------------------------------
// One 1024-lane workgroup per request walks its tree on its own, in fp64: the current distribution r
// lives unnormalised in device memory (value / norm), every child is offered against it with the exact
// ratio r[x]/q[x], a rejection replaces r by the normalised residual max(0, r - q) (written to the
// second buffer, which then becomes current), an acceptance moves on to the accepted node's target
// distribution, and the last token is drawn by the inverse CDF over r.  While r is still a node's own
// target distribution it is not written out: a child is judged from two gathered logits and the row
// statistics of the first pass, and only a rejection (or the final draw) sweeps the vocabulary.  Sweeps
// use the workgroup's lanes and reduce in a fixed order, so the result is run-to-run identical.  This
// path favours exactness over speed: a request costs two or three vocabulary sweeps per rejected
// child and one or two for the draw, all on one compute unit.
constexpr int kTreeThreads = 1024;

struct TreeShared {
    double red[kTreeThreads / 64];
    int ired[kTreeThreads / 64];
};

__device__ __forceinline__ double tree_sum(double v, TreeShared &sh)
{
    for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.red[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < kTreeThreads / 64; ++i) s += sh.red[i];
    return s;
}

__device__ __forceinline__ int tree_min(int v, TreeShared &sh)
{
    for (int off = 32; off; off >>= 1) v = min(v, __shfl_xor(v, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.ired[threadIdx.x >> 6] = v;
    __syncthreads();
    int s = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < kTreeThreads / 64; ++i) s = min(s, sh.ired[i]);
    return s;
}

__device__ __forceinline__ int tree_max(int v, TreeShared &sh) { return -tree_min(-v, sh); }

template <int DT>
__global__ __launch_bounds__(kTreeThreads) void accept_tree_sample_kernel(AcceptArgs a, Workspace w, double *buf)
{
    __shared__ ExpTable ex;
    __shared__ TreeShared sh;
    ex.init();
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.vocab;
    const int t0 = a.q_indptr[b], k = a.q_indptr[b + 1] - t0 - 1, d0 = t0 - b;
    const float T = a.temperature ? a.temperature[b] : a.temperature_scalar;
    const double inv_t = 1.0 / (double)T;
    double *cur_arr = buf + (int64_t)b * 3 * V, *alt = cur_arr + V, *eq = cur_arr + 2 * (int64_t)V;
    double norm = 1.0;

    // Maximum and normaliser of a row from the chunk statistics of the row-statistics pass (every lane
    // computes them).  The maximum is exact; the normaliser carries the fp32 rounding of the chunk sums
    // (relative error below 1e-6) and is only used to judge a child, never in a residual.
    auto row_stats = [&](int64_t ry, float &m, double &z) {
        m = -INFINITY;
        for (int c = 0; c < w.nchunks; ++c) m = fmaxf(m, w.cmax[ry * w.nchunks + c]);
        z = 0.0;
        for (int c = 0; c < w.nchunks; ++c) {
            const float cm = w.cmax[ry * w.nchunks + c];
            if (cm != -INFINITY) z += (double)w.csum[ry * w.nchunks + c] * exp2(((double)cm - (double)m) * inv_t * kLog2eD);
        }
    };
    // cur_arr <- exponentials of a target row, norm <- their exact sum: r = softmax of the row
    auto materialise = [&](int node, float m) {
        double s = 0.0;
        for (int v = tid; v < V; v += kTreeThreads) {
            const double e = ex(((double)load_logit(a.target, t0 + node, a.row_stride, DT, v) - (double)m) * inv_t);
            cur_arr[v] = e;
            s += e;
        }
        norm = tree_sum(s, sh);   // (its barriers also publish cur_arr to the workgroup)
    };

    if (tid < k && a.ratio_out) a.ratio_out[d0 + tid] = __builtin_nanf("");
    int cur = 0, n = 0, my_tok = -1, my_node = -1;
    bool degenerate = false;
    bool pure = true;   // r is still the current node's own target distribution and has not been written out
    float mp;
    double zp;
    row_stats(t0, mp, zp);
    for (;;) {
        bool moved = false;
        for (int c = cur + 1; c <= k && !moved; ++c) {
            if (a.tree_parent[t0 + c] != cur) continue;
            const int x = a.draft_tokens[d0 + c - 1];
            const double u = (double)a.u_accept[d0 + c - 1];
            float mq;
            double zq;
            row_stats((int64_t)a.total_rows + d0 + c - 1, mq, zq);
            const double qx = ex(((double)load_logit(a.draft, d0 + c - 1, a.row_stride, DT, x) - (double)mq) * inv_t) / zq;
            const double rx = pure ? ex(((double)load_logit(a.target, t0 + cur, a.row_stride, DT, x) - (double)mp) * inv_t) / zp
                                   : cur_arr[x] / norm;
            if (tid == 0 && a.ratio_out) a.ratio_out[d0 + c - 1] = (float)(rx / qx);
            if (u * qx < rx) {
                if (tid == n) {
                    my_tok = x;
                    my_node = c;
                }
                ++n;
                cur = c;
                degenerate = false;
                pure = true;
                row_stats((int64_t)t0 + c, mp, zp);
                moved = true;
            } else {
                // the residual is taken exactly: both distributions with their fp64 normalisers
                __syncthreads();   // (lanes may still be reading cur_arr[x])
                if (pure) {
                    materialise(cur, mp);
                    pure = false;
                }
                double s = 0.0;
                for (int v = tid; v < V; v += kTreeThreads) {
                    const double e = ex(((double)load_logit(a.draft, d0 + c - 1, a.row_stride, DT, v) - (double)mq) * inv_t);
                    eq[v] = e;
                    s += e;
                }
                const double zq_exact = tree_sum(s, sh);
                double sr = 0.0;
                for (int v = tid; v < V; v += kTreeThreads) {
                    const double rt = cur_arr[v] / norm, qt = eq[v] / zq_exact;
                    const double res = rt > qt ? rt - qt : 0.0;
                    alt[v] = res;
                    sr += res;
                }
                const double S = tree_sum(sr, sh);
                degenerate = !(S > 0.0);
                if (!degenerate) {
                    double *t = cur_arr;
                    cur_arr = alt;
                    alt = t;
                    norm = S;
                }
            }
        }
        if (!moved) break;
    }

    int y;
    if (degenerate) {   // the residual vanished: lowest-index maximum of the current node's target row
        float m;
        double z;
        row_stats((int64_t)t0 + cur, m, z);
        int best = 0x7fffffff;
        for (int v = tid; v < V; v += kTreeThreads)
            if (load_logit(a.target, t0 + cur, a.row_stride, DT, v) == m) { best = v; break; }
        y = tree_min(best, sh);
    } else {
        if (pure) materialise(cur, mp);
        // inverse CDF in token order: lane t owns the contiguous entries [t*seg, (t+1)*seg)
        const int seg = (V + kTreeThreads - 1) / kTreeThreads;
        const int lo = min(V, tid * seg), hi = min(V, lo + seg);
        double mine = 0.0;
        int my_last = -1;
        for (int v = lo; v < hi; ++v) {
            const double rt = cur_arr[v] / norm;
            if (rt > 0.0) {
                mine += rt;
                my_last = v;
            }
        }
        double incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const double t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        __syncthreads();
        if (lane == 63) sh.red[wave] = incl;
        __syncthreads();
        double before = 0.0, total = 0.0;
#pragma unroll
        for (int i = 0; i < kTreeThreads / 64; ++i) {
            if (i < wave) before += sh.red[i];
            total += sh.red[i];
        }
        const double excl = before + (incl - mine);
        const double thr = (double)a.u_sample[b] * total;
        const int first = tree_min(excl + mine > thr ? tid : 0x7fffffff, sh);
        const int last_tok = tree_max(my_last, sh);
        int tok = -1;
        if (tid == first) {
            double c = excl;
            for (int v = lo; v < hi; ++v) {
                const double rt = cur_arr[v] / norm;
                if (rt > 0.0) {
                    c += rt;
                    if (tok < 0 && c > thr) tok = v;
                }
            }
            if (tok < 0) tok = my_last;   // the lane total crossed but the element-wise sum rounds differently
        }
        y = first == 0x7fffffff ? last_tok : tree_max(tok, sh);
    }
    if (tid == n) my_tok = y;
    if (tid < SS_OUT_WIDTH) a.out_tokens[(int64_t)b * SS_OUT_WIDTH + tid] = tid <= n ? my_tok : -1;
    if (tid < SS_MAX_DEPTH) a.accepted_nodes[(int64_t)b * SS_MAX_DEPTH + tid] = tid < n ? my_node : -1;
    if (tid == 0) a.accepted_len[b] = n;
}

}  // namespace

size_t accept_workspace_bytes(int batch, int total_rows, int vocab)
{
    const size_t nch = num_chunks(vocab), nsub = num_sub(vocab);
    const size_t rows = 2 * (size_t)total_rows - batch;
    size_t n = 3 * align_up(sizeof(float) * rows * nch, 256);
    n += align_up(sizeof(RowPick) * (size_t)batch, 256);
    n += 5 * align_up(sizeof(double) * (size_t)batch * nsub, 256);
    n += 2 * align_up(sizeof(double) * (size_t)batch * kAmbCap, 256);
    n += 2 * align_up(sizeof(int32_t) * (size_t)batch * nsub, 256);
    n += 2 * align_up(sizeof(int32_t) * (size_t)batch, 256);
    return n + 256;
}

template <int DT>
static int32_t accept_launch_dt(const AcceptArgs &a, const Workspace &w, unsigned g1, unsigned g2, hipStream_t stream)
{
    hipLaunchKernelGGL(accept_rowstats_kernel<DT>, dim3(g1), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_rowstats_kernel");
    hipLaunchKernelGGL(accept_decide_kernel, dim3(a.batch), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_decide_kernel");
    if (a.greedy) return SS_OK;
    hipLaunchKernelGGL(accept_norm_kernel<DT>, dim3(g2), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_norm_kernel");
    hipLaunchKernelGGL(accept_pick_kernel<DT>, dim3((unsigned)a.batch * kPickWgs), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_pick_kernel");
    return SS_OK;
}

int32_t accept_launch(const AcceptArgs &a, hipStream_t stream)
{
    const Workspace w = carve(a.workspace, a.batch, a.total_rows, a.vocab);
    const unsigned long long g1 =
        (unsigned long long)a.batch * (a.greedy ? a.max_q_len : 2 * a.max_q_len - 1) * ((w.nchunks + 3) / 4);
    const unsigned long long g2 = (unsigned long long)a.batch * w.nsub;
    if (g1 > 0x7fffffffull || g2 > 0x7fffffffull)
        return fail(SS_ERR_UNSUPPORTED, "batch * vocab too large for one launch");
    if (a.logit_dtype == SS_BF16) return accept_launch_dt<SS_BF16>(a, w, (unsigned)g1, (unsigned)g2, stream);
    return accept_launch_dt<SS_F32>(a, w, (unsigned)g1, (unsigned)g2, stream);
}

size_t accept_tree_workspace_bytes(int batch, int total_rows, int vocab)
{
    return accept_workspace_bytes(batch, total_rows, vocab) + align_up(sizeof(double) * 3 * (size_t)batch * vocab, 256);
}

int32_t accept_tree_sample_launch(const AcceptArgs &a, hipStream_t stream)
{
    const Workspace w = carve(a.workspace, a.batch, a.total_rows, a.vocab);
    double *buf = reinterpret_cast<double *>(static_cast<char *>(a.workspace) +
                                             accept_workspace_bytes(a.batch, a.total_rows, a.vocab));
    const unsigned long long g1 = (unsigned long long)a.batch * (2 * a.max_q_len - 1) * ((w.nchunks + 3) / 4);
    if (g1 > 0x7fffffffull) return fail(SS_ERR_UNSUPPORTED, "batch * vocab too large for one launch");
    if (a.logit_dtype == SS_BF16) {
        hipLaunchKernelGGL(accept_rowstats_kernel<SS_BF16>, dim3((unsigned)g1), dim3(kThreads), 0, stream, a, w);
        SS_HIP_CHECK(hipGetLastError(), "launch accept_rowstats_kernel");
        hipLaunchKernelGGL(accept_tree_sample_kernel<SS_BF16>, dim3(a.batch), dim3(kTreeThreads), 0, stream, a, w, buf);
    } else {
        hipLaunchKernelGGL(accept_rowstats_kernel<SS_F32>, dim3((unsigned)g1), dim3(kThreads), 0, stream, a, w);
        SS_HIP_CHECK(hipGetLastError(), "launch accept_rowstats_kernel");
        hipLaunchKernelGGL(accept_tree_sample_kernel<SS_F32>, dim3(a.batch), dim3(kTreeThreads), 0, stream, a, w, buf);
    }
    SS_HIP_CHECK(hipGetLastError(), "launch accept_tree_sample_kernel");
    return SS_OK;
}

}  // namespace ss
