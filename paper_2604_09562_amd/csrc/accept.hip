// spec_accept: acceptance walk and resampling over full-vocabulary logits.
//
// Pass 1 (rowstats) streams every target and draft row once (the HBM-bound part): per
// 8192-entry chunk it leaves the chunk maximum and sum of exp2((x - max) * log2e/T) in fp32
// (greedy mode: maximum and lowest-index argmax of target rows only).
// decide      one wavefront per request merges the chunk statistics, walks the drafts
//             (u < p/q in fp64) and fixes the accepted length and which rows are resampled.
// Passes 2a-2c touch only the one or two rows the new token is drawn from and work in fp64,
// so the drawn token can be reproduced by an fp64 reference: 2a normalisers per chunk, 2b
// residual mass per chunk, 2c inverse-CDF search inside the chunk that holds u * mass.
// All reductions have a fixed order (no atomics): results are run-to-run identical.
#include "common.h"

namespace ss {
namespace {

constexpr int kThreads = 256;
constexpr int kPerThread = kChunk / kThreads;  // 32 logits per lane
constexpr double kLog2eD = 1.4426950408889634;

struct RowPick {      // written by decide, read by the resampling passes
    int32_t p_row;    // target row the new token is drawn from
    int32_t q_row;    // draft row of the rejected position, -1 if every draft was accepted
    float m_p, m_q;   // exact row maxima
    float temperature;
    int32_t n;        // accepted length
    int32_t pad[2];
};

struct Workspace {
    float *cmax, *csum;   // [rows][nchunks]
    int32_t *carg;        // [rows][nchunks]
    RowPick *pick;        // [batch]
    double *zp, *zq, *sc; // [batch][nchunks]
    int nchunks, rows;
};

__host__ __device__ inline int num_chunks(int vocab) { return (vocab + kChunk - 1) / kChunk; }

__host__ Workspace carve(void *ws, int batch, int total_rows, int vocab)
{
    Workspace w;
    w.nchunks = num_chunks(vocab);
    w.rows = 2 * total_rows - batch;
    char *p = static_cast<char *>(ws);
    const size_t per = align_up(sizeof(float) * (size_t)w.rows * w.nchunks, 256);
    w.cmax = reinterpret_cast<float *>(p); p += per;
    w.csum = reinterpret_cast<float *>(p); p += per;
    w.carg = reinterpret_cast<int32_t *>(p); p += per;
    w.pick = reinterpret_cast<RowPick *>(p); p += align_up(sizeof(RowPick) * (size_t)batch, 256);
    const size_t perd = align_up(sizeof(double) * (size_t)batch * w.nchunks, 256);
    w.zp = reinterpret_cast<double *>(p); p += perd;
    w.zq = reinterpret_cast<double *>(p); p += perd;
    w.sc = reinterpret_cast<double *>(p); p += perd;
    return w;
}

// ---- loading one lane's share of a chunk ---------------------------------------------------
// Coalesced order: lane t owns elements chunk0 + it*(kThreads*8) + t*8 + j  (bf16, it<4, j<8)
//                                   or chunk0 + it*(kThreads*4) + t*4 + j  (f32,  it<8, j<4)
// Sequential order (sampling search): lane t owns chunk0 + t*32 .. +31.
// Out-of-vocabulary positions read as -inf.  index_of() gives the vocabulary id of slot s.
template <bool SEQ>
__device__ __forceinline__ int index_of(int chunk0, int tid, int s, int dtype)
{
    if (SEQ) return chunk0 + tid * kPerThread + s;
    const int vec = dtype == SS_BF16 ? 8 : 4;
    return chunk0 + (s / vec) * (kThreads * vec) + tid * vec + (s % vec);
}

template <bool SEQ>
__device__ __forceinline__ void load_slots(const void *row, int vocab, int chunk0, int tid, int dtype, float (&x)[kPerThread])
{
    if (dtype == SS_BF16) {
#pragma unroll
        for (int it = 0; it < kPerThread / 8; ++it) {
            const int i0 = index_of<SEQ>(chunk0, tid, it * 8, dtype);
            if (i0 + 8 <= vocab) {
                const uint4 w = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(row) + i0);
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[it * 8 + 2 * j] = __uint_as_float(ww[j] << 16);
                    x[it * 8 + 2 * j + 1] = __uint_as_float(ww[j] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    x[it * 8 + j] = (i0 + j < vocab)
                                        ? __uint_as_float((uint32_t) static_cast<const uint16_t *>(row)[i0 + j] << 16)
                                        : -INFINITY;
            }
        }
    } else {
#pragma unroll
        for (int it = 0; it < kPerThread / 4; ++it) {
            const int i0 = index_of<SEQ>(chunk0, tid, it * 4, dtype);
            if (i0 + 4 <= vocab) {
                const float4 w = *reinterpret_cast<const float4 *>(static_cast<const float *>(row) + i0);
                x[it * 4] = w.x; x[it * 4 + 1] = w.y; x[it * 4 + 2] = w.z; x[it * 4 + 3] = w.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    x[it * 4 + j] = (i0 + j < vocab) ? static_cast<const float *>(row)[i0 + j] : -INFINITY;
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

// request owning target row r / draft row j (q_indptr[b] - b is the draft-row start of b)
__device__ __forceinline__ int request_of_row(const int32_t *q_indptr, int batch, int r, bool draft)
{
    int lo = 0, hi = batch;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        const int start = q_indptr[mid] - (draft ? mid : 0);
        if (start <= r) lo = mid; else hi = mid;
    }
    return lo;
}

// ---- pass 1 ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_rowstats_kernel(AcceptArgs a, Workspace w)
{
    __shared__ float sh[4];
    __shared__ int shi[4];
    const int chunk = blockIdx.x % w.nchunks, ry = blockIdx.x / w.nchunks, tid = threadIdx.x;
    const bool is_draft = ry >= a.total_rows;
    const int r = is_draft ? ry - a.total_rows : ry;
    const void *row = row_ptr(is_draft ? a.draft : a.target, r, a.row_stride, a.logit_dtype);
    float x[kPerThread];
    load_slots<false>(row, a.vocab, chunk * kChunk, tid, a.logit_dtype, x);

    float m = x[0];
#pragma unroll
    for (int s = 1; s < kPerThread; ++s) m = fmaxf(m, x[s]);
    const float cm = block_max(m, sh);
    const int64_t o = (int64_t)ry * w.nchunks + chunk;
    if (a.greedy) {
        // lowest vocabulary id holding the chunk maximum
        int best = 0x7fffffff;
#pragma unroll
        for (int s = 0; s < kPerThread; ++s) {
            const int id = index_of<false>(chunk * kChunk, tid, s, a.logit_dtype);
            if (x[s] == cm && id < best) best = id;
        }
        for (int off = 32; off; off >>= 1) best = min(best, __shfl_xor(best, off));
        __syncthreads();
        if ((tid & 63) == 0) shi[tid >> 6] = best;
        __syncthreads();
        if (tid == 0) {
            w.cmax[o] = cm;
            w.carg[o] = min(min(shi[0], shi[1]), min(shi[2], shi[3]));
        }
        return;
    }
    float T = a.temperature_scalar;
    if (a.temperature) T = a.temperature[request_of_row(a.q_indptr, a.batch, r, is_draft)];
    const float sc = 1.4426950408889634f / T;
    float z = 0.f;
    if (cm != -INFINITY) {
#pragma unroll
        for (int s = 0; s < kPerThread; ++s) z += exp2f((x[s] - cm) * sc);
    }
    z = block_sum<float>(z, sh);
    if (tid == 0) {
        w.cmax[o] = cm;
        w.csum[o] = z;
    }
}

// ---- decide ---------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void accept_decide_kernel(AcceptArgs a, Workspace w)
{
    __shared__ float row_m[2 * SS_OUT_WIDTH];
    __shared__ double row_z[2 * SS_OUT_WIDTH];
    __shared__ int row_arg[SS_OUT_WIDTH];
    const int b = blockIdx.x, lane = threadIdx.x;
    const int t0 = a.q_indptr[b], k = a.q_indptr[b + 1] - t0 - 1, d0 = t0 - b;
    const float T = a.temperature ? a.temperature[b] : a.temperature_scalar;
    const double inv_t = a.greedy ? 1.0 : 1.0 / (double)T;

    // merge chunk statistics of the k+1 target rows and k draft rows
    const int nrows = a.greedy ? k + 1 : 2 * k + 1;
    for (int j = 0; j < nrows; ++j) {
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
    if (lane != 0) return;

    int32_t *toks = a.out_tokens + (int64_t)b * SS_OUT_WIDTH;
    int n = k;
    if (a.greedy) {
        n = 0;
        while (n < k && row_arg[n] == a.draft_tokens[d0 + n]) ++n;
    } else {
        for (int i = 0; i < k; ++i) {
            const int x = a.draft_tokens[d0 + i];
            const double lp = load_logit(a.target, t0 + i, a.row_stride, a.logit_dtype, x);
            const double lq = load_logit(a.draft, d0 + i, a.row_stride, a.logit_dtype, x);
            // p(x)/q(x) = exp((lp-mp)/T - (lq-mq)/T) * Zq/Zp
            const double e = (lp - (double)row_m[i]) * inv_t - (lq - (double)row_m[k + 1 + i]) * inv_t;
            const double rho = exp(e) * (row_z[k + 1 + i] / row_z[i]);
            if (a.ratio_out) a.ratio_out[d0 + i] = (float)rho;
            if (n == k && !((double)a.u_accept[d0 + i] < rho)) n = i;
        }
    }
    for (int j = 0; j < SS_OUT_WIDTH; ++j) toks[j] = j < n ? a.draft_tokens[d0 + j] : -1;
    a.accepted_len[b] = n;
    if (a.greedy) {
        toks[n] = row_arg[n];
        return;
    }
    RowPick pk;
    pk.p_row = t0 + n;
    pk.q_row = n < k ? d0 + n : -1;
    pk.m_p = row_m[n];
    pk.m_q = n < k ? row_m[k + 1 + n] : 0.f;
    pk.temperature = T;
    pk.n = n;
    pk.pad[0] = pk.pad[1] = 0;
    w.pick[b] = pk;
}

// ---- pass 2a: fp64 normalisers per chunk ---------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_norm_kernel(AcceptArgs a, Workspace w)
{
    __shared__ double sh[4];
    const int chunk = blockIdx.x % w.nchunks, b = blockIdx.x / w.nchunks, tid = threadIdx.x;
    const RowPick pk = w.pick[b];
    const double inv_t = 1.0 / (double)pk.temperature;
    float x[kPerThread];
    load_slots<false>(row_ptr(a.target, pk.p_row, a.row_stride, a.logit_dtype), a.vocab, chunk * kChunk, tid,
                      a.logit_dtype, x);
    double z = 0.0;
#pragma unroll 4
    for (int s = 0; s < kPerThread; ++s) z += exp(((double)x[s] - (double)pk.m_p) * inv_t);
    z = block_sum<double>(z, sh);
    if (tid == 0) w.zp[(int64_t)b * w.nchunks + chunk] = z;
    if (pk.q_row < 0) return;
    load_slots<false>(row_ptr(a.draft, pk.q_row, a.row_stride, a.logit_dtype), a.vocab, chunk * kChunk, tid,
                      a.logit_dtype, x);
    z = 0.0;
#pragma unroll 4
    for (int s = 0; s < kPerThread; ++s) z += exp(((double)x[s] - (double)pk.m_q) * inv_t);
    z = block_sum<double>(z, sh);
    if (tid == 0) w.zq[(int64_t)b * w.nchunks + chunk] = z;
}

__device__ __forceinline__ double ordered_total(const double *v, int n)
{
    double s = 0.0;
    for (int c = 0; c < n; ++c) s += v[c];
    return s;
}

// residual (or bonus) mass of one vocabulary entry
__device__ __forceinline__ double mass(float lp, float lq, const RowPick &pk, double inv_t, double inv_zp, double inv_zq)
{
    const double p = exp(((double)lp - (double)pk.m_p) * inv_t) * inv_zp;
    if (pk.q_row < 0) return p;
    const double q = exp(((double)lq - (double)pk.m_q) * inv_t) * inv_zq;
    return p > q ? p - q : 0.0;
}

// ---- pass 2b: residual mass per chunk -------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_mass_kernel(AcceptArgs a, Workspace w)
{
    __shared__ double sh[4];
    const int chunk = blockIdx.x % w.nchunks, b = blockIdx.x / w.nchunks, tid = threadIdx.x;
    const RowPick pk = w.pick[b];
    const double zp = ordered_total(w.zp + (int64_t)b * w.nchunks, w.nchunks);
    if (pk.q_row < 0) {  // bonus distribution: the chunk's share of p
        if (tid == 0) w.sc[(int64_t)b * w.nchunks + chunk] = w.zp[(int64_t)b * w.nchunks + chunk] / zp;
        return;
    }
    const double zq = ordered_total(w.zq + (int64_t)b * w.nchunks, w.nchunks);
    const double inv_t = 1.0 / (double)pk.temperature, inv_zp = 1.0 / zp, inv_zq = 1.0 / zq;
    float xp[kPerThread], xq[kPerThread];
    load_slots<false>(row_ptr(a.target, pk.p_row, a.row_stride, a.logit_dtype), a.vocab, chunk * kChunk, tid,
                      a.logit_dtype, xp);
    load_slots<false>(row_ptr(a.draft, pk.q_row, a.row_stride, a.logit_dtype), a.vocab, chunk * kChunk, tid,
                      a.logit_dtype, xq);
    double s = 0.0;
#pragma unroll 4
    for (int i = 0; i < kPerThread; ++i) s += mass(xp[i], xq[i], pk, inv_t, inv_zp, inv_zq);
    s = block_sum<double>(s, sh);
    if (tid == 0) w.sc[(int64_t)b * w.nchunks + chunk] = s;
}

// ---- pass 2c: inverse-CDF search ------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_pick_kernel(AcceptArgs a, Workspace w)
{
    __shared__ double wave_tot[4];
    __shared__ int sh_first[4], sh_last[4];
    __shared__ float sh_f[4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowPick pk = w.pick[b];
    int32_t *dst = a.out_tokens + (int64_t)b * SS_OUT_WIDTH + pk.n;
    const double *sc = w.sc + (int64_t)b * w.nchunks;

    // chunk that holds u * S (every lane does the same short scan)
    const double S = ordered_total(sc, w.nchunks);
    if (!(S > 0.0)) {
        // p_n == q_n exactly: no residual mass; fall back to the lowest-index argmax of the target row
        const void *row = row_ptr(a.target, pk.p_row, a.row_stride, a.logit_dtype);
        float best = -INFINITY;
        for (int v = tid; v < a.vocab; v += kThreads)
            best = fmaxf(best, load_logit(a.target, pk.p_row, a.row_stride, a.logit_dtype, v));
        best = block_max(best, sh_f);
        int arg = 0x7fffffff;
        for (int v = tid; v < a.vocab; v += kThreads)
            if (load_logit(a.target, pk.p_row, a.row_stride, a.logit_dtype, v) == best) { arg = v; break; }
        for (int off = 32; off; off >>= 1) arg = min(arg, __shfl_xor(arg, off));
        if (lane == 0) sh_first[wave] = arg;
        __syncthreads();
        if (tid == 0) *dst = min(min(sh_first[0], sh_first[1]), min(sh_first[2], sh_first[3]));
        (void)row;
        return;
    }
    const double thr = (double)a.u_sample[b] * S;
    int cstar = -1, last_pos = -1;
    double prefix = 0.0, run = 0.0;
    for (int c = 0; c < w.nchunks; ++c) {
        if (sc[c] > 0.0) {
            last_pos = c;
            if (cstar < 0 && run + sc[c] > thr) {
                cstar = c;
                prefix = run;
            }
            run += sc[c];
        }
    }
    const bool take_last = cstar < 0;  // rounding left u*S at or past the total: last entry with mass
    if (take_last) cstar = last_pos;

    const double zp = ordered_total(w.zp + (int64_t)b * w.nchunks, w.nchunks);
    const double zq = pk.q_row >= 0 ? ordered_total(w.zq + (int64_t)b * w.nchunks, w.nchunks) : 1.0;
    const double inv_t = 1.0 / (double)pk.temperature, inv_zp = 1.0 / zp, inv_zq = 1.0 / zq;
    float xp[kPerThread], xq[kPerThread];
    load_slots<true>(row_ptr(a.target, pk.p_row, a.row_stride, a.logit_dtype), a.vocab, cstar * kChunk, tid,
                     a.logit_dtype, xp);
    if (pk.q_row >= 0)
        load_slots<true>(row_ptr(a.draft, pk.q_row, a.row_stride, a.logit_dtype), a.vocab, cstar * kChunk, tid,
                         a.logit_dtype, xq);
    else {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) xq[i] = 0.f;
    }
    double r[kPerThread];
    double local = 0.0;
    int my_last = -1;
#pragma unroll 4
    for (int i = 0; i < kPerThread; ++i) {
        r[i] = mass(xp[i], xq[i], pk, inv_t, inv_zp, inv_zq);
        local += r[i];
        if (r[i] > 0.0) my_last = cstar * kChunk + tid * kPerThread + i;
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
#pragma unroll 4
        for (int i = 0; i < kPerThread; ++i) {
            if (r[i] > 0.0) {
                c += r[i];
                if (tok < 0 && c > thr) tok = cstar * kChunk + tid * kPerThread + i;
            }
        }
        // the lane total crossed but the element-wise sum may round differently: then its last entry with mass
        *dst = tok >= 0 ? tok : my_last;
    }
}

}  // namespace

size_t accept_workspace_bytes(int batch, int total_rows, int vocab)
{
    const size_t nch = num_chunks(vocab);
    const size_t rows = 2 * (size_t)total_rows - batch;
    size_t n = 3 * align_up(sizeof(float) * rows * nch, 256);
    n += align_up(sizeof(RowPick) * (size_t)batch, 256);
    n += 3 * align_up(sizeof(double) * (size_t)batch * nch, 256);
    return n + 256;
}

int32_t accept_launch(const AcceptArgs &a, hipStream_t stream)
{
    const Workspace w = carve(a.workspace, a.batch, a.total_rows, a.vocab);
    const unsigned rows = a.greedy ? (unsigned)a.total_rows : (unsigned)w.rows;
    hipLaunchKernelGGL(accept_rowstats_kernel, dim3((unsigned)w.nchunks * rows), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_rowstats_kernel");
    hipLaunchKernelGGL(accept_decide_kernel, dim3(a.batch), dim3(64), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_decide_kernel");
    if (a.greedy) return SS_OK;
    hipLaunchKernelGGL(accept_norm_kernel, dim3((unsigned)w.nchunks * (unsigned)a.batch), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_norm_kernel");
    hipLaunchKernelGGL(accept_mass_kernel, dim3((unsigned)w.nchunks * (unsigned)a.batch), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_mass_kernel");
    hipLaunchKernelGGL(accept_pick_kernel, dim3(a.batch), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_pick_kernel");
    return SS_OK;
}

}  // namespace ss
