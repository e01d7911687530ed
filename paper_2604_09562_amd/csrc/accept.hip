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
#include "accept_common.h"

namespace ss {
namespace {

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

// Every logit is read exactly once by this pass: non-temporal loads keep the stream from displacing the one or
// two rows per request that the later passes read again.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const char *p)
{
    const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
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
            raw[v] = stream_load16(static_cast<const char *>(row) + (int64_t)i0 * (DT == SS_BF16 ? 2 : 4));
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
// One 256-lane workgroup per request.  Each quarter of a wavefront merges the chunk statistics of one row
// (16 lanes over the chunks; 16 rows per trip), then lanes 0..k-1 of wave 0 evaluate their draft and a
// ballot finds the first rejection.
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

    // Sixteen rows at a time: every quarter of a wavefront (16 lanes over the chunks) merges one row, so the
    // rows of an ordinary request are done in one trip.
    const int quarter = lane >> 4, ql = lane & 15;
    for (int j0 = 0; j0 < nrows; j0 += 16) {
        const int j = j0 + wave * 4 + quarter;
        const bool live = j < nrows;
        const int64_t ry = !live ? 0 : (j <= k ? (int64_t)t0 + j : (int64_t)a.total_rows + d0 + (j - k - 1));
        float m = -INFINITY;
        if (live)
            for (int c = ql; c < w.nchunks; c += 16) m = fmaxf(m, w.cmax[ry * w.nchunks + c]);
        for (int off = 8; off; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));   // (stays inside the quarter)
        if (a.greedy) {
            int best = 0x7fffffff;
            if (live)
                for (int c = ql; c < w.nchunks; c += 16)
                    if (w.cmax[ry * w.nchunks + c] == m) best = min(best, w.carg[ry * w.nchunks + c]);
            for (int off = 8; off; off >>= 1) best = min(best, __shfl_xor(best, off));
            if (live && ql == 0) row_arg[j] = best;
        } else {
            double z = 0.0;
            if (live)
                for (int c = ql; c < w.nchunks; c += 16) {
                    const float cm = w.cmax[ry * w.nchunks + c];
                    if (cm != -INFINITY)
                        z += (double)w.csum[ry * w.nchunks + c] * exp2(((double)cm - (double)m) * inv_t * kLog2eD);
                }
            for (int off = 8; off; off >>= 1) z += __shfl_xor(z, off);
            if (live && ql == 0) {
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

int32_t accept_rowstats_launch(const AcceptArgs &a, hipStream_t stream)
{
    const Workspace w = carve(a.workspace, a.batch, a.total_rows, a.vocab);
    const unsigned long long g1 =
        (unsigned long long)a.batch * (a.greedy ? a.max_q_len : 2 * a.max_q_len - 1) * ((w.nchunks + 3) / 4);
    if (g1 > 0x7fffffffull) return fail(SS_ERR_UNSUPPORTED, "batch * vocab too large for one launch");
    if (a.logit_dtype == SS_BF16)
        hipLaunchKernelGGL(accept_rowstats_kernel<SS_BF16>, dim3((unsigned)g1), dim3(kThreads), 0, stream, a, w);
    else
        hipLaunchKernelGGL(accept_rowstats_kernel<SS_F32>, dim3((unsigned)g1), dim3(kThreads), 0, stream, a, w);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_rowstats_kernel");
    return SS_OK;
}

}  // namespace ss
