// Sampled acceptance over draft trees (the chain rule and the greedy tree walk are in accept.hip).
#include "accept_common.h"

namespace ss {
namespace {

// ---- sampled acceptance over a draft tree ------------------------------------------------------------------
// The walk of a request is a chain of dependent steps, but only its rejections need the whole vocabulary:
// while the running distribution r is still a node's own target distribution a child is judged from two
// gathered logits and the row statistics of the first pass.  So the work is laid out in rounds, each a
// short sequence of launches over all requests at once (the stream orders them, no kernel waits for
// another workgroup):
//   walk   one wavefront per request: finish the residual of the previous round, then offer children
//          until one is rejected (-> a residual is due) or none is left (-> the draw is due)
//   sums   per 2048-entry block, exact fp64 sums of the proposal's exponentials (and of the target row's,
//          if r has not been written out yet), for the requests that are due
//   resid  the residual max(0, r - q) with the exact normalisers, written to the request's other buffer,
//          and its sum per block; for a request whose draw is due, r itself and its mass per block
// A request needs one round per rejection, at most k; the launcher runs max_q_len - 1 rounds, a last
// walk, sums and resid for the draws, and the pick.  r lives unnormalised in device memory (value / norm),
// two fp64 vocabulary vectors per request.  All reductions have a fixed order.
struct TreeScalars {
    int32_t cur, n, next, phase;       // phase: 0 walking, 1 residual due, 2 draw due
    int32_t pure, degenerate, which, rej;   // which: the buffer that holds r; rej: the child just rejected
    float mp, mq;                      // exact maxima of the current node's target row / the rejected child's draft row
    double zp_stats;                   // normaliser of the target row from the first pass (judging only)
    double norm;                       // exact normaliser of the buffer that holds r
};
struct TreeState {
    TreeScalars s;                     // copied to registers by the kernels
    int32_t tok[SS_OUT_WIDTH];         // accepted tokens and nodes so far: written and read in place (a private copy
    int32_t node[SS_MAX_DEPTH];        // indexed by a run-time value would live in scratch memory)
};

enum { TS_WALK = 0, TS_RESIDUAL = 1, TS_DRAW = 2 };

// maximum and (first-pass) normaliser of a row from its chunk statistics: one wavefront, lanes over chunks
__device__ __forceinline__ void tree_row_stats(const Workspace &w, int64_t ry, double inv_t, float &m, double &z)
{
    const int lane = threadIdx.x & 63;
    m = -INFINITY;
    for (int c = lane; c < w.nchunks; c += 64) m = fmaxf(m, w.cmax[ry * w.nchunks + c]);
    for (int off = 32; off; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    z = 0.0;
    for (int c = lane; c < w.nchunks; c += 64) {
        const float cm = w.cmax[ry * w.nchunks + c];
        if (cm != -INFINITY) z += (double)w.csum[ry * w.nchunks + c] * exp2(((double)cm - (double)m) * inv_t * kLog2eD);
    }
    for (int off = 32; off; off >>= 1) z += __shfl_xor(z, off);   // (xor butterfly: every lane ends with the same bits)
}

__device__ __forceinline__ double tree_exp_at(const void *rows, int64_t row, int64_t stride, int dtype, int v, float m,
                                              double inv_t)
{
    return exp(((double)load_logit(rows, row, stride, dtype, v) - (double)m) * inv_t);
}

template <int DT>
__global__ __launch_bounds__(64) void tree_walk_kernel(AcceptArgs a, Workspace w, TreeState *st, double *arr, int first)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int V = a.vocab;
    const int t0 = a.q_indptr[b], k = a.q_indptr[b + 1] - t0 - 1, d0 = t0 - b;
    const float T = a.temperature ? a.temperature[b] : a.temperature_scalar;
    const double inv_t = 1.0 / (double)T;
    TreeScalars s;
    if (first) {
        s.cur = 0; s.n = 0; s.next = 1; s.phase = TS_WALK; s.pure = 1; s.degenerate = 0; s.which = 0; s.rej = 0;
        s.mq = 0.f; s.norm = 1.0;
        tree_row_stats(w, t0, inv_t, s.mp, s.zp_stats);
        if (lane < k && a.ratio_out) a.ratio_out[d0 + lane] = __builtin_nanf("");
    } else {
        s = st[b].s;   // (every lane reads the same record; only lane 0 writes it back)
        if (s.phase == TS_DRAW) return;
    }
    if (s.phase == TS_RESIDUAL) {   // the residual of the last rejection is in the other buffer: adopt it
        double S = 0.0;
        for (int c = 0; c < w.nsub; ++c) S += w.sc[(int64_t)b * w.nsub + c];
        s.degenerate = !(S > 0.0);
        if (!s.degenerate) {
            s.which ^= 1;
            s.norm = S;
            s.pure = 0;
        }
        s.phase = TS_WALK;
    }
    const double *r_arr = arr + ((int64_t)b * 2 + s.which) * V;
    int c = s.next;
    for (; c <= k; ++c) {
        if (a.tree_parent[t0 + c] != s.cur) continue;
        const int x = a.draft_tokens[d0 + c - 1];
        const double u = (double)a.u_accept[d0 + c - 1];
        float mq;
        double zq;
        tree_row_stats(w, (int64_t)a.total_rows + d0 + c - 1, inv_t, mq, zq);
        const double qx = tree_exp_at(a.draft, d0 + c - 1, a.row_stride, DT, x, mq, inv_t) / zq;
        const double rx = s.pure ? tree_exp_at(a.target, t0 + s.cur, a.row_stride, DT, x, s.mp, inv_t) / s.zp_stats
                                 : r_arr[x] / s.norm;
        if (lane == 0 && a.ratio_out) a.ratio_out[d0 + c - 1] = (float)(rx / qx);
        if (u * qx < rx) {
            if (lane == 0) {
                st[b].tok[s.n] = x;
                st[b].node[s.n] = c;
            }
            ++s.n;
            s.cur = c;
            s.pure = 1;
            s.degenerate = 0;
            tree_row_stats(w, (int64_t)t0 + c, inv_t, s.mp, s.zp_stats);
        } else {
            s.phase = TS_RESIDUAL;
            s.rej = c;
            s.mq = mq;
            break;
        }
    }
    s.next = c + 1;
    if (s.phase == TS_WALK) s.phase = TS_DRAW;   // no child left
    if (lane == 0) st[b].s = s;
}

// Exact block sums of exponentials: of the rejected child's proposal (residual due), of the current
// node's target row (r not written out yet and a residual or the draw is due).  grid: batch * nsub.
template <int DT>
__global__ __launch_bounds__(kThreads) void tree_sums_kernel(AcceptArgs a, Workspace w, const TreeState *st, int final_pass)
{
    __shared__ double sh[4];
    __shared__ ExpTable ex;
    const int sub = blockIdx.x % w.nsub, b = blockIdx.x / w.nsub, tid = threadIdx.x;
    const TreeScalars s = st[b].s;
    const bool want_q = s.phase == TS_RESIDUAL && !final_pass;
    const bool want_p = s.pure && (want_q || (final_pass && s.phase == TS_DRAW && !s.degenerate));
    if (!want_q && !want_p) return;
    ex.init();
    const int t0 = a.q_indptr[b], d0 = t0 - b;
    const float T = a.temperature ? a.temperature[b] : a.temperature_scalar;
    const double inv_t = 1.0 / (double)T;
    const int64_t o = (int64_t)b * w.nsub + sub;
    double zq = 0.0, zp = 0.0;
#pragma unroll
    for (int j = 0; j < kSubPer; ++j) {
        const int v = sub * kSub + j * kThreads + tid;
        if (v < a.vocab) {
            if (want_q) zq += ex(((double)load_logit(a.draft, d0 + s.rej - 1, a.row_stride, DT, v) - (double)s.mq) * inv_t);
            if (want_p) zp += ex(((double)load_logit(a.target, t0 + s.cur, a.row_stride, DT, v) - (double)s.mp) * inv_t);
        }
    }
    if (want_q) {
        zq = block_sum<double>(zq, sh);
        if (tid == 0) w.zq[o] = zq;
    }
    if (want_p) {
        zp = block_sum<double>(zp, sh);
        if (tid == 0) w.zp[o] = zp;
    }
}

// Residual due: other buffer <- max(0, r - q), its block sums.  Draw due (final pass): block masses of r,
// and r written out if it was not yet.  grid: batch * nsub.
template <int DT>
__global__ __launch_bounds__(kThreads) void tree_resid_kernel(AcceptArgs a, Workspace w, const TreeState *st, double *arr,
                                                              int final_pass)
{
    __shared__ double sh[4];
    __shared__ ExpTable ex;
    const int sub = blockIdx.x % w.nsub, b = blockIdx.x / w.nsub, tid = threadIdx.x;
    const TreeScalars s = st[b].s;
    const bool resid = s.phase == TS_RESIDUAL && !final_pass;
    const bool draw = final_pass && s.phase == TS_DRAW && !s.degenerate;
    if (!resid && !draw) return;
    ex.init();
    const int V = a.vocab;
    const int t0 = a.q_indptr[b], d0 = t0 - b;
    const float T = a.temperature ? a.temperature[b] : a.temperature_scalar;
    const double inv_t = 1.0 / (double)T;
    const int64_t ob = (int64_t)b * w.nsub;
    double zq = 1.0, norm = s.norm;
    if (resid) {
        zq = 0.0;
        for (int c = 0; c < w.nsub; ++c) zq += w.zq[ob + c];
    }
    if (s.pure) {
        norm = 0.0;
        for (int c = 0; c < w.nsub; ++c) norm += w.zp[ob + c];
    }
    double *cur_arr = arr + ((int64_t)b * 2 + s.which) * V, *alt = arr + ((int64_t)b * 2 + (s.which ^ 1)) * V;
    const double inv_norm = 1.0 / norm, inv_zq = 1.0 / zq;   // (one division each instead of two per vocabulary entry)
    double sum = 0.0;
#pragma unroll
    for (int j = 0; j < kSubPer; ++j) {
        const int v = sub * kSub + j * kThreads + tid;
        if (v < V) {
            const double e = s.pure ? ex(((double)load_logit(a.target, t0 + s.cur, a.row_stride, DT, v) - (double)s.mp) * inv_t)
                                    : cur_arr[v];
            const double rt = e * inv_norm;
            if (resid) {
                const double qt = ex(((double)load_logit(a.draft, d0 + s.rej - 1, a.row_stride, DT, v) - (double)s.mq) * inv_t) * inv_zq;
                const double res = rt > qt ? rt - qt : 0.0;
                alt[v] = res;
                sum += res;
            } else {
                if (s.pure) cur_arr[v] = e;
                sum += rt;
            }
        }
    }
    sum = block_sum<double>(sum, sh);
    if (tid == 0) w.sc[ob + sub] = sum;
}

// The draw: scan of the block masses, search inside the block that holds u * total.  grid: batch.
template <int DT>
__global__ __launch_bounds__(kThreads) void tree_pick_kernel(AcceptArgs a, Workspace w, const TreeState *st, const double *arr)
{
    __shared__ double sh[4];
    __shared__ int shi[4];
    __shared__ int cstar_sh;
    __shared__ double prefix_sh, total_sh, norm_sh;
    __shared__ double mass_sh[kThreads];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TreeScalars s = st[b].s;
    const int V = a.vocab;
    const int t0 = a.q_indptr[b];
    const int64_t ob = (int64_t)b * w.nsub;
    int y = -1;
    if (s.degenerate) {   // the residual vanished: lowest-index maximum of the current node's target row
        int best = 0x7fffffff;
        for (int v = tid; v < V; v += kThreads)
            if (load_logit(a.target, t0 + s.cur, a.row_stride, DT, v) == s.mp) { best = v; break; }
        for (int off = 32; off; off >>= 1) best = min(best, __shfl_xor(best, off));
        if (lane == 0) shi[wave] = best;
        __syncthreads();
        y = min(min(shi[0], shi[1]), min(shi[2], shi[3]));
    } else {
        // The block masses (and, if r was only just written out, the block sums of its normaliser) are
        // fetched by the lanes at once; lane 0 then adds them in index order, as the other kernels do.
        double total = 0.0, zsum = 0.0;
        for (int base = 0; base < w.nsub; base += kThreads) {
            const int c = base + tid;
            __syncthreads();
            mass_sh[tid] = c < w.nsub ? (s.pure ? w.zp[ob + c] : 0.0) : 0.0;
            __syncthreads();
            if (tid == 0)
                for (int j = 0; j < kThreads && base + j < w.nsub; ++j) zsum += mass_sh[j];
        }
        if (tid == 0) norm_sh = s.pure ? zsum : s.norm;
        const bool one_round = w.nsub <= kThreads;   // vocabularies up to 512k entries: the masses fit the staging array
        __syncthreads();
        mass_sh[tid] = one_round && tid < w.nsub ? w.sc[ob + tid] : 0.0;
        __syncthreads();
        const double norm = norm_sh;
        if (tid == 0) {   // block masses in index order: total, then the first block with mass whose running sum exceeds u * total
            for (int c = 0; c < w.nsub; ++c) total += one_round ? mass_sh[c] : w.sc[ob + c];
            const double thr = (double)a.u_sample[b] * total;
            double cum = 0.0, pre = 0.0, last_pre = 0.0;
            int cstar = -1, last = -1;
            for (int c = 0; c < w.nsub; ++c) {
                const double m = one_round ? mass_sh[c] : w.sc[ob + c];
                if (m > 0.0) {
                    last = c;
                    last_pre = cum;
                    if (cstar < 0 && cum + m > thr) {
                        cstar = c;
                        pre = cum;
                    }
                    cum += m;
                }
            }
            if (cstar < 0) {   // rounding left u * total at or past the sum: the last block with mass
                cstar = last < 0 ? 0 : last;   // (no mass at all cannot happen for a valid batch; stay in bounds anyway)
                pre = last_pre;
            }
            cstar_sh = cstar;
            prefix_sh = pre;
            total_sh = total;
        }
        __syncthreads();
        const int cstar = cstar_sh;
        const double thr = (double)a.u_sample[b] * total_sh;
        const double *r_arr = arr + ((int64_t)b * 2 + s.which) * V;
        // lane t owns the block's entries t*8 .. t*8+7 in token order
        double r[kSubPer], local = 0.0;
        int my_last = -1;
#pragma unroll
        for (int j = 0; j < kSubPer; ++j) {
            const int v = cstar * kSub + tid * kSubPer + j;
            r[j] = v < V ? r_arr[v] / norm : 0.0;
            if (r[j] > 0.0) {
                local += r[j];
                my_last = v;
            }
        }
        double incl = local;
        for (int off = 1; off < 64; off <<= 1) {
            const double t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        if (lane == 63) sh[wave] = incl;
        __syncthreads();
        double before = prefix_sh;
        for (int wv = 0; wv < wave; ++wv) before += sh[wv];
        const double excl = before + (incl - local);
        const unsigned long long bal = __ballot(excl + local > thr);
        if (lane == 0) shi[wave] = bal ? wave * 64 + (__ffsll((long long)bal) - 1) : 0x7fffffff;
        int lw = my_last;
        for (int off = 32; off; off >>= 1) lw = max(lw, __shfl_xor(lw, off));
        __syncthreads();
        const int first = min(min(shi[0], shi[1]), min(shi[2], shi[3]));
        __syncthreads();
        if (lane == 0) shi[wave] = lw;
        __syncthreads();
        const int last_tok = max(max(shi[0], shi[1]), max(shi[2], shi[3]));
        __syncthreads();
        int tok = -1;
        if (tid == first) {
            double c = excl;
#pragma unroll
            for (int j = 0; j < kSubPer; ++j) {
                if (r[j] > 0.0) {
                    c += r[j];
                    if (tok < 0 && c > thr) tok = cstar * kSub + tid * kSubPer + j;
                }
            }
            if (tok < 0) tok = my_last;   // the lane total crossed but the element-wise sum rounds differently
        }
        for (int off = 32; off; off >>= 1) tok = max(tok, __shfl_xor(tok, off));
        if (lane == 0) shi[wave] = tok;
        __syncthreads();
        y = first == 0x7fffffff ? last_tok : max(max(shi[0], shi[1]), max(shi[2], shi[3]));
    }
    if (tid < SS_OUT_WIDTH)
        a.out_tokens[(int64_t)b * SS_OUT_WIDTH + tid] = tid < s.n ? st[b].tok[tid] : (tid == s.n ? y : -1);
    if (tid < SS_MAX_DEPTH) a.accepted_nodes[(int64_t)b * SS_MAX_DEPTH + tid] = tid < s.n ? st[b].node[tid] : -1;
    if (tid == 0) a.accepted_len[b] = s.n;
}

}  // namespace

size_t accept_tree_workspace_bytes(int batch, int total_rows, int vocab)
{
    return accept_workspace_bytes(batch, total_rows, vocab) + align_up(sizeof(TreeState) * (size_t)batch, 256) +
           align_up(sizeof(double) * 2 * (size_t)batch * vocab, 256);
}

template <int DT>
static int32_t tree_sample_rounds(const AcceptArgs &a, const Workspace &w, TreeState *st, double *arr, hipStream_t stream)
{
    const dim3 per_request((unsigned)a.batch), per_block((unsigned)a.batch * w.nsub);
    for (int round = 0; round < a.max_q_len; ++round) {   // a request has at most max_q_len - 1 rejections
        hipLaunchKernelGGL(tree_walk_kernel<DT>, per_request, dim3(64), 0, stream, a, w, st, arr, round == 0 ? 1 : 0);
        const int final_pass = round == a.max_q_len - 1;   // by now every request is waiting for its draw
        hipLaunchKernelGGL(tree_sums_kernel<DT>, per_block, dim3(kThreads), 0, stream, a, w, st, final_pass);
        hipLaunchKernelGGL(tree_resid_kernel<DT>, per_block, dim3(kThreads), 0, stream, a, w, st, arr, final_pass);
    }
    hipLaunchKernelGGL(tree_pick_kernel<DT>, per_request, dim3(kThreads), 0, stream, a, w, st, arr);
    SS_HIP_CHECK(hipGetLastError(), "launch of the sampled tree walk");
    return SS_OK;
}

int32_t accept_tree_sample_launch(const AcceptArgs &a, hipStream_t stream)
{
    const Workspace w = carve(a.workspace, a.batch, a.total_rows, a.vocab);
    char *p = static_cast<char *>(a.workspace) + accept_workspace_bytes(a.batch, a.total_rows, a.vocab);
    TreeState *st = reinterpret_cast<TreeState *>(p);
    double *arr = reinterpret_cast<double *>(p + align_up(sizeof(TreeState) * (size_t)a.batch, 256));
    if ((unsigned long long)a.batch * w.nsub > 0x7fffffffull) return fail(SS_ERR_UNSUPPORTED, "batch * vocab too large for one launch");
    const int32_t rc = accept_rowstats_launch(a, stream);
    if (rc != SS_OK) return rc;
    if (a.logit_dtype == SS_BF16) return tree_sample_rounds<SS_BF16>(a, w, st, arr, stream);
    return tree_sample_rounds<SS_F32>(a, w, st, arr, stream);
}

}  // namespace ss
