// Sampled acceptance over draft trees (the chain rule and the greedy tree walk are in accept.hip).
#include "accept_common.h"

namespace ss {
namespace {

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

size_t accept_tree_workspace_bytes(int batch, int total_rows, int vocab)
{
    return accept_workspace_bytes(batch, total_rows, vocab) + align_up(sizeof(double) * 3 * (size_t)batch * vocab, 256);
}

int32_t accept_tree_sample_launch(const AcceptArgs &a, hipStream_t stream)
{
    const Workspace w = carve(a.workspace, a.batch, a.total_rows, a.vocab);
    double *buf = reinterpret_cast<double *>(static_cast<char *>(a.workspace) +
                                             accept_workspace_bytes(a.batch, a.total_rows, a.vocab));
    const int32_t rc = accept_rowstats_launch(a, stream);
    if (rc != SS_OK) return rc;
    if (a.logit_dtype == SS_BF16)
        hipLaunchKernelGGL(accept_tree_sample_kernel<SS_BF16>, dim3(a.batch), dim3(kTreeThreads), 0, stream, a, w, buf);
    else
        hipLaunchKernelGGL(accept_tree_sample_kernel<SS_F32>, dim3(a.batch), dim3(kTreeThreads), 0, stream, a, w, buf);
    SS_HIP_CHECK(hipGetLastError(), "launch accept_tree_sample_kernel");
    return SS_OK;
}

}  // namespace ss
