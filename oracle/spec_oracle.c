/*
 * CPU oracle for the decode lane's speculative-verification step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the GPU library must compute.  It shares no code, header, table or constant
 * with the HIP path, and only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * What the paper fixes: the decode worker verifies a request's draft tokens in
 * one parallel target-model pass while preserving the target's output
 * distribution (Section 2.2, the speculative-sampling rule of the work cited
 * there), over a paged KV cache (Section 2.4) that holds the prefill KV with
 * every decoded token appended (Section 3.4, Eq. 7); the depth of each request
 * is chosen per request by the controller (Section 3.5, Alg. 4, Eq. 13).  The
 * paper gives no further detail of the verification itself, so the functions
 * below write out the textbook definitions; every reading taken where the
 * paper is silent is listed in the repository's design notes.
 *
 * All floating point is IEEE double.  Inputs arrive in their storage format
 * (float32, bfloat16 bits, OCP e4m3fn bytes) and are decoded here, exactly.
 *
 * Pin status: every function in this file is pinned by tests/test_oracle_*.py
 * (library attention routine, brute force, closed forms, exhaustive
 * enumeration of the sampling identity, library storage casts).  Accepted-length statistics on the
 * five workloads are "parity unpinned" by the paper (it prints none).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { OR_F32 = 0, OR_BF16 = 1, OR_FP8_E4M3 = 2 };

/* ---- exact storage decoders ------------------------------------------------ */

static double decode_bf16(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16; /* bfloat16 is the upper half of a float32 */
    float f;
    memcpy(&f, &w, 4);
    return (double)f;
}

/* OCP 8-bit float, 1 sign / 4 exponent (bias 7) / 3 mantissa bits, "fn" flavour:
 * no infinities, the single NaN pattern is S.1111.111, largest finite is 448. */
static double decode_e4m3fn(uint8_t b)
{
    int sign = b >> 7, e = (b >> 3) & 0xF, m = b & 0x7;
    double v;
    if (e == 0xF && m == 0x7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6); /* subnormal: 2^(1-7) * m/8 */
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

static double load_elem(const void *base, int64_t idx, int dtype)
{
    switch (dtype) {
    case OR_F32:
        return (double)((const float *)base)[idx];
    case OR_BF16:
        return decode_bf16(((const uint16_t *)base)[idx]);
    default:
        return decode_e4m3fn(((const uint8_t *)base)[idx]);
    }
}

/* for tests: decode n elements of a storage array */
void oracle_decode(const void *src, int64_t n, int dtype, double *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = load_elem(src, i, dtype);
}

/* ---- verify attention -------------------------------------------------------
 *
 * Request b brings q_len = q_indptr[b+1]-q_indptr[b] = k_b+1 query tokens: the
 * last accepted token followed by its k_b draft tokens.  Their keys/values are
 * already the last q_len of the kv_len[b] valid cache positions, so query
 * token i sits at absolute position pos_i = kv_len - q_len + i and attends to
 * cache positions 0..pos_i (causal among the new tokens, everything older is
 * visible).  Query head h reads KV head h / (Hq/Hkv).
 *
 * With tree_mask != NULL the new tokens form a draft tree instead of a chain
 * (node 0 is the last accepted token, node j's parent has a smaller index): bit
 * j of tree_mask[row] says that the row attends new token j, i.e. that j is the
 * row's own node or one of its ancestors; the older context stays fully visible.
 * The chain is the special case tree_mask[row i] = 2^(i+1) - 1.
 *
 *     s_t = sm_scale * <Q[row,h,:], K[t,:]>        t = 0..pos_i
 *     out = sum_t softmax(s)_t * V[t,:]            lse = ln sum_t exp(s_t)
 *
 * Cache position t of request b lives in physical block block_table[b][t/bs],
 * slot t%bs; element (block, kv head, slot, d) of the dense cache array.  For
 * e4m3 caches the real value is decode(byte) * scale[block][kv head].
 *
 * part_tokens > 0 computes the same thing the split way: the visible range is
 * cut into pieces of part_tokens positions, each piece yields its own
 * softmax-weighted value sum and log-sum-exp, and the pieces are merged with
 *     lse = ln sum_p exp(lse_p),   out = sum_p exp(lse_p - lse) * out_p.
 * Both ways must agree to rounding; a test checks that.
 *
 * req_list (may be NULL = all) selects which requests to compute; rows of the
 * other requests are left untouched.  Returns 0, or a negative code on bad
 * arguments (checked before any work).
 */
static void attend_range(const double *qrow, int D, int dtype, const void *kc, const void *vc,
                         const float *k_scale, const float *v_scale, const int32_t *bt_row,
                         int Hkv, int g, int bs, const int *pos, int t0, int t1, double sm_scale,
                         double *s /*scratch t1-t0*/, double *out /*D*/, double *lse)
{
    /* attends the cache positions pos[t0..t1) */
    double m = -INFINITY;
    for (int t = t0; t < t1; ++t) {
        int64_t phys = bt_row[pos[t] / bs];
        int64_t base = ((phys * Hkv + g) * bs + (pos[t] % bs)) * (int64_t)D;
        double acc = 0.0;
        for (int d = 0; d < D; ++d)
            acc += qrow[d] * load_elem(kc, base + d, dtype);
        if (k_scale)
            acc *= (double)k_scale[phys * Hkv + g];
        s[t - t0] = sm_scale * acc;
        if (s[t - t0] > m)
            m = s[t - t0];
    }
    double l = 0.0;
    for (int t = t0; t < t1; ++t) {
        s[t - t0] = exp(s[t - t0] - m);
        l += s[t - t0];
    }
    for (int d = 0; d < D; ++d)
        out[d] = 0.0;
    for (int t = t0; t < t1; ++t) {
        int64_t phys = bt_row[pos[t] / bs];
        int64_t base = ((phys * Hkv + g) * bs + (pos[t] % bs)) * (int64_t)D;
        double w = s[t - t0] / l;
        if (v_scale)
            w *= (double)v_scale[phys * Hkv + g];
        for (int d = 0; d < D; ++d)
            out[d] += w * load_elem(vc, base + d, dtype);
    }
    *lse = m + log(l);
}

int oracle_verify_attn(int B, int Hq, int Hkv, int D, int bs, int max_blocks, int kv_dtype,
                       const void *k_cache, const void *v_cache, const float *k_scale,
                       const float *v_scale, const int32_t *block_table, const int32_t *kv_len,
                       const int32_t *q_indptr, const uint32_t *tree_mask, int q_dtype, const void *q,
                       double sm_scale, int part_tokens, const int32_t *req_list, int n_req, double *out,
                       double *lse, int num_threads)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || D <= 0 || bs <= 0 || part_tokens < 0)
        return -1;
    if (kv_dtype < 0 || kv_dtype > 2 || q_dtype < 0 || q_dtype > 1)
        return -2;
    if ((kv_dtype == OR_FP8_E4M3) != (k_scale != NULL) || (k_scale == NULL) != (v_scale == NULL))
        return -3;
    for (int b = 0; b < B; ++b) {
        int ql = q_indptr[b + 1] - q_indptr[b];
        if (ql < 1 || kv_len[b] < ql || (kv_len[b] + bs - 1) / bs > max_blocks)
            return -4;
        /* a row of a draft tree sees itself and only new tokens of its own request */
        for (int i = 0; tree_mask && i < ql; ++i) {
            uint32_t mk = tree_mask[q_indptr[b] + i];
            if (ql > 32 || !((mk >> i) & 1u) || (ql < 32 && (mk >> ql)))
                return -6;
        }
    }
    int G = Hq / Hkv;
    int n = req_list ? n_req : B;
    int fail = 0;
#ifdef _OPENMP
    if (num_threads > 0)
        omp_set_num_threads(num_threads);
#endif
    (void)num_threads;
    /* one unit of parallel work = (request, query head); the arithmetic inside is sequential */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int ib = 0; ib < n; ++ib) {
        for (int h = 0; h < Hq; ++h) {
            int b = req_list ? req_list[ib] : ib;
            int ql = q_indptr[b + 1] - q_indptr[b];
            int L = kv_len[b];
            int g = h / G;
            const int32_t *bt_row = block_table + (int64_t)b * max_blocks;
            double *s = (double *)malloc(sizeof(double) * (size_t)L);
            double *qrow = (double *)malloc(sizeof(double) * (size_t)D * 3);
            int *pos = (int *)malloc(sizeof(int) * (size_t)L);
            if (!s || !qrow || !pos) {
                fail = 1;
                free(s);
                free(qrow);
                free(pos);
                continue;
            }
            double *o_part = qrow + D, *o_sum = qrow + 2 * D;
            for (int i = 0; i < ql; ++i) {
                int64_t row = q_indptr[b] + i;
                /* Visible positions, ascending: the whole context before this step's tokens, then
                 * new token j (at position L-ql+j) if it is an ancestor of row i or row i itself.
                 * In a chain that is every j <= i; in a tree the mask's bit j says so. */
                int vis = 0;
                for (int t = 0; t < L; ++t) {
                    int j = t - (L - ql);
                    if (j < 0 || (tree_mask ? (int)((tree_mask[row] >> j) & 1u) : j <= i))
                        pos[vis++] = t;
                }
                double *o = out + (row * Hq + h) * (int64_t)D;
                for (int d = 0; d < D; ++d)
                    qrow[d] = load_elem(q, (row * Hq + h) * (int64_t)D + d, q_dtype);
                if (part_tokens == 0) {
                    attend_range(qrow, D, kv_dtype, k_cache, v_cache, k_scale, v_scale, bt_row,
                                 Hkv, g, bs, pos, 0, vis, sm_scale, s, o, &lse[row * Hq + h]);
                } else {
                    /* split into pieces, then merge the pieces by their log-sum-exp */
                    int np = (vis + part_tokens - 1) / part_tokens;
                    double *pl = (double *)malloc(sizeof(double) * (size_t)np);
                    double *po = (double *)malloc(sizeof(double) * (size_t)np * D);
                    double mx = -INFINITY, tot = 0.0;
                    for (int p = 0; p < np; ++p) {
                        int t0 = p * part_tokens;
                        int t1 = t0 + part_tokens < vis ? t0 + part_tokens : vis;
                        attend_range(qrow, D, kv_dtype, k_cache, v_cache, k_scale, v_scale,
                                     bt_row, Hkv, g, bs, pos, t0, t1, sm_scale, s, o_part, &pl[p]);
                        memcpy(po + (size_t)p * D, o_part, sizeof(double) * D);
                        if (pl[p] > mx)
                            mx = pl[p];
                    }
                    for (int p = 0; p < np; ++p)
                        tot += exp(pl[p] - mx);
                    double L_all = mx + log(tot);
                    for (int d = 0; d < D; ++d)
                        o_sum[d] = 0.0;
                    for (int p = 0; p < np; ++p) {
                        double w = exp(pl[p] - L_all);
                        for (int d = 0; d < D; ++d)
                            o_sum[d] += w * po[(size_t)p * D + d];
                    }
                    memcpy(o, o_sum, sizeof(double) * D);
                    lse[row * Hq + h] = L_all;
                    free(pl);
                    free(po);
                }
            }
            free(s);
            free(qrow);
            free(pos);
        }
    }
    return fail ? -5 : 0;
}

/* ---- acceptance / resampling -------------------------------------------------
 *
 * Per request b with depth k (k+1 target rows lp_0..lp_k, k draft rows
 * lq_0..lq_{k-1}, draft tokens x_0..x_{k-1}, uniforms u_0..u_{k-1} and u_s,
 * temperature T > 0):
 *
 *     p_i = softmax(lp_i / T),  q_i = softmax(lq_i / T)
 *     walk i = 0,1,..: accept draft i iff  u_i * q_i[x_i] < p_i[x_i]
 *                      (that is u_i < min(1, p/q)); stop at the first rejection
 *     n = number accepted
 *     n < k : r = max(0, p_n - q_n)   (residual of the rejected position)
 *     n = k : r = p_k                 (bonus distribution)
 *     S = sum_v r_v,  c_v = r_0 + .. + r_v in token order,
 *     y = the first v with c_v > u_s * S   (never a zero-mass token);
 *         if rounding leaves none, the last v with r_v > 0;
 *         if S == 0 (p_n == q_n exactly), the lowest-index argmax of lp_n
 *     emit x_0..x_{n-1}, y;  accepted_len = n
 *
 * Greedy mode ignores T and the uniforms: accept while the lowest-index argmax
 * of lp_i equals x_i; y is the lowest-index argmax of lp_n.
 *
 * Row placement: target rows of request b are q_indptr[b] .. q_indptr[b+1]-1 of
 * a [rows][row_stride] array; its draft rows, tokens and u_i start at
 * q_indptr[b] - b of the draft-side arrays.
 *
 * Diagnostics for the comparison harness (none feeds back into the result):
 *   ratio[j]     p/q of every draft position j (also those after the rejection)
 *   near_tie[j]  1 where |u_j - min(1,p/q)| < tie_eps: the one place where the
 *                test statement allows a GPU result to differ
 *   y_lo/y_hi[b] the tokens whose CDF interval [c_{v-1}, c_v]/S comes within
 *                tie_eps of u_s (zero-mass tokens skipped); y_lo <= y <= y_hi
 *   resid_sum[b] S
 */
static void softmax_row(const void *logits, int64_t off, int V, int dtype, double T, double *p)
{
    double m = -INFINITY, z = 0.0;
    for (int v = 0; v < V; ++v) {
        p[v] = load_elem(logits, off + v, dtype) / T;
        if (p[v] > m)
            m = p[v];
    }
    for (int v = 0; v < V; ++v) {
        p[v] = exp(p[v] - m);
        z += p[v];
    }
    for (int v = 0; v < V; ++v)
        p[v] /= z;
}

static int argmax_row(const void *logits, int64_t off, int V, int dtype)
{
    int best = 0;
    double bv = load_elem(logits, off, dtype);
    for (int v = 1; v < V; ++v) {
        double x = load_elem(logits, off + v, dtype);
        if (x > bv) { /* strict: ties keep the lowest index */
            bv = x;
            best = v;
        }
    }
    return best;
}

int oracle_spec_accept(int B, int V, int64_t row_stride, int logit_dtype, const int32_t *q_indptr,
                       const void *target_logits, const void *draft_logits,
                       const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                       const float *temperature, int greedy, int width, double tie_eps,
                       int32_t *accepted_len, int32_t *out_tokens, double *ratio,
                       int32_t *near_tie, int32_t *y_lo, int32_t *y_hi, double *resid_sum,
                       int num_threads)
{
    if (B < 0 || V <= 0 || row_stride < V || logit_dtype < 0 || logit_dtype > 1 || width < 1)
        return -1;
    for (int b = 0; b < B; ++b) {
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        if (k < 0 || k + 1 > width)
            return -4;
        if (!greedy && !(temperature[b] > 0.0f))
            return -6;
        for (int i = 0; i < k; ++i) {
            int x = draft_tokens[q_indptr[b] - b + i];
            if (x < 0 || x >= V)
                return -7;
        }
    }
    int fail = 0;
#ifdef _OPENMP
    if (num_threads > 0)
        omp_set_num_threads(num_threads);
#endif
    (void)num_threads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        int64_t trow0 = q_indptr[b], drow0 = q_indptr[b] - b;
        int32_t *toks = out_tokens + (int64_t)b * width;
        for (int j = 0; j < width; ++j)
            toks[j] = -1;
        if (greedy) {
            int n = 0;
            while (n < k &&
                   argmax_row(target_logits, (trow0 + n) * row_stride, V, logit_dtype) ==
                       draft_tokens[drow0 + n])
                ++n;
            for (int j = 0; j < n; ++j)
                toks[j] = draft_tokens[drow0 + j];
            toks[n] = argmax_row(target_logits, (trow0 + n) * row_stride, V, logit_dtype);
            accepted_len[b] = n;
            for (int j = 0; j < k; ++j) {
                if (ratio) ratio[drow0 + j] = NAN;
                if (near_tie) near_tie[drow0 + j] = 0;
            }
            if (y_lo) y_lo[b] = toks[n];
            if (y_hi) y_hi[b] = toks[n];
            if (resid_sum) resid_sum[b] = NAN;
            continue;
        }
        double T = (double)temperature[b];
        double *p = (double *)malloc(sizeof(double) * (size_t)V * 2);
        if (!p) {
            fail = 1;
            continue;
        }
        double *q = p + V;
        int n = k; /* becomes the index of the first rejection */
        for (int i = 0; i < k; ++i) {
            softmax_row(target_logits, (trow0 + i) * row_stride, V, logit_dtype, T, p);
            softmax_row(draft_logits, (drow0 + i) * row_stride, V, logit_dtype, T, q);
            int x = draft_tokens[drow0 + i];
            double u = (double)u_accept[drow0 + i];
            int accept = u * q[x] < p[x];
            if (!accept && n == k)
                n = i;
            double rho = p[x] / q[x]; /* inf if q underflowed to 0 < p; nan if 0/0 */
            if (ratio) ratio[drow0 + i] = rho;
            if (near_tie) {
                double capped = rho < 1.0 ? rho : 1.0;
                near_tie[drow0 + i] = (rho == rho) && fabs(u - capped) < tie_eps && rho < 1.0 + tie_eps;
            }
        }
        /* distribution to draw the one new token from */
        softmax_row(target_logits, (trow0 + n) * row_stride, V, logit_dtype, T, p);
        if (n < k) {
            softmax_row(draft_logits, (drow0 + n) * row_stride, V, logit_dtype, T, q);
            for (int v = 0; v < V; ++v)
                p[v] = p[v] > q[v] ? p[v] - q[v] : 0.0;
        }
        double S = 0.0;
        for (int v = 0; v < V; ++v)
            S += p[v];
        int y = -1, lo = -1, hi = -1;
        if (S > 0.0) {
            double thr = (double)u_sample[b] * S, c = 0.0, us = (double)u_sample[b];
            int last_pos = -1;
            for (int v = 0; v < V; ++v) {
                if (!(p[v] > 0.0))
                    continue;
                double c_prev = c;
                c += p[v];
                last_pos = v;
                if (y < 0 && c > thr)
                    y = v;
                /* does [c_prev, c]/S come within tie_eps of u_s ? */
                if (c_prev / S - tie_eps <= us && us <= c / S + tie_eps) {
                    if (lo < 0) lo = v;
                    hi = v;
                }
            }
            if (y < 0)
                y = last_pos;
            if (lo < 0) lo = hi = y;
            if (y < lo) lo = y;
            if (y > hi) hi = y;
        } else {
            y = lo = hi = argmax_row(target_logits, (trow0 + n) * row_stride, V, logit_dtype);
        }
        for (int j = 0; j < n; ++j)
            toks[j] = draft_tokens[drow0 + j];
        toks[n] = y;
        accepted_len[b] = n;
        if (y_lo) y_lo[b] = lo;
        if (y_hi) y_hi[b] = hi;
        if (resid_sum) resid_sum[b] = S;
        free(p);
    }
    return fail ? -5 : 0;
}

/* ---- greedy acceptance over a draft tree --------------------------------------
 *
 * The new tokens of request b form a tree: node 0 is the last accepted token,
 * node i >= 1 carries draft token x_i (entry q_indptr[b]-b+i-1 of draft_tokens)
 * and has parent tree_parent[q_indptr[b]+i] < i (-1 for node 0).  Target row i
 * holds the logits that follow node i.  Greedy decoding emits, after any node,
 * the lowest-index argmax of that node's row, so the walk is
 *
 *     cur = 0
 *     repeat: t = argmax(row cur); c = the lowest-numbered child of cur with
 *             x_c == t; if there is none stop, else accept c and set cur = c
 *     emit the accepted tokens, then t (the argmax at the node where it stopped)
 *
 * and the output is exactly what plain greedy decoding of the target model
 * would have produced.  accepted_nodes lists the accepted node numbers in path
 * order (they are increasing), -1 beyond accepted_len.  A chain
 * (tree_parent[i] = i-1) gives the greedy mode of oracle_spec_accept.
 */
int oracle_tree_accept_greedy(int B, int V, int64_t row_stride, int logit_dtype, const int32_t *q_indptr,
                              const int32_t *tree_parent, const void *target_logits,
                              const int32_t *draft_tokens, int out_width, int32_t *accepted_len,
                              int32_t *out_tokens, int32_t *accepted_nodes)
{
    if (B < 0 || V <= 0 || row_stride < V || out_width < 1)
        return -1;
    for (int b = 0; b < B; ++b) {
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        if (k < 0 || k + 1 > out_width || tree_parent[q_indptr[b]] != -1)
            return -4;
        for (int i = 1; i <= k; ++i)
            if (tree_parent[q_indptr[b] + i] < 0 || tree_parent[q_indptr[b] + i] >= i)
                return -6;
    }
    for (int b = 0; b < B; ++b) {
        int64_t row0 = q_indptr[b];
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        const int32_t *x = draft_tokens + (row0 - b) - 1; /* x[i] = token of node i, i = 1..k */
        int32_t *toks = out_tokens + (int64_t)b * out_width;
        int32_t *nodes = accepted_nodes + (int64_t)b * (out_width - 1);
        for (int j = 0; j < out_width; ++j)
            toks[j] = -1;
        for (int j = 0; j < out_width - 1; ++j)
            nodes[j] = -1;
        int cur = 0, n = 0;
        for (;;) {
            int t = argmax_row(target_logits, (row0 + cur) * row_stride, V, logit_dtype);
            int child = -1;
            for (int i = cur + 1; i <= k && child < 0; ++i)
                if (tree_parent[row0 + i] == cur && x[i] == t)
                    child = i;
            if (child < 0) {
                toks[n] = t;
                break;
            }
            toks[n] = t;
            nodes[n] = child;
            ++n;
            cur = child;
        }
        accepted_len[b] = n;
    }
    return 0;
}

/* ---- sampled acceptance over a draft tree --------------------------------------
 *
 * Tree layout as for the greedy walk.  Draft row c-1 of the request (row q_indptr[b]-b+c-1 of
 * draft_logits) is the distribution node c's token x_c was drawn from, u_c = u_accept at the same
 * index its uniform.  The walk keeps a current node and a current distribution r, starting at node 0
 * with r = p_0 = softmax(target row 0 / T), and offers r the children of the current node one after
 * the other, in node order, each as one step of speculative sampling against its own proposal
 * q_c = softmax(draft row of c / T):
 *
 *     accept c  iff  u_c * q_c[x_c] < r[x_c]      (u_c < min(1, r/q))
 *     accepted: c becomes the current node, r = p_c, and its children are offered next
 *     rejected: r <- max(0, r - q_c) / S,  S = sum_v max(0, r_v - q_c,v)   (unchanged if S == 0),
 *               and the next sibling is offered
 *     no child left: draw y from r by the inverse CDF in token order with u_s (first v whose
 *               running sum exceeds u_s * sum(r); if rounding leaves none, the last v with mass);
 *               if the last rejection found S == 0 (r equal to the proposal), y is the
 *               lowest-index argmax of the current node's target row, as in the chain rule.
 *
 * Every step is the accept/residual step of speculative sampling applied to the distribution the
 * previous step left, so the emitted tokens are distributed as plain sampling from the target; a
 * chain reduces to oracle_spec_accept.  Outputs as for the greedy walk, plus per draft node the
 * ratio r[x]/q[x] it was offered at (NaN for nodes the walk never offered) and the near-tie flag.
 */
int oracle_tree_accept_sample(int B, int V, int64_t row_stride, int logit_dtype, const int32_t *q_indptr,
                              const int32_t *tree_parent, const void *target_logits, const void *draft_logits,
                              const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                              const float *temperature, int out_width, double tie_eps, int32_t *accepted_len,
                              int32_t *out_tokens, int32_t *accepted_nodes, double *ratio, int32_t *near_tie)
{
    if (B < 0 || V <= 0 || row_stride < V || out_width < 1)
        return -1;
    for (int b = 0; b < B; ++b) {
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        if (k < 0 || k + 1 > out_width || tree_parent[q_indptr[b]] != -1 || !(temperature[b] > 0.0f))
            return -4;
        for (int i = 1; i <= k; ++i) {
            int par = tree_parent[q_indptr[b] + i], x = draft_tokens[q_indptr[b] - b + i - 1];
            if (par < 0 || par >= i || x < 0 || x >= V)
                return -6;
        }
    }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int64_t row0 = q_indptr[b], d0 = q_indptr[b] - b;
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        double T = (double)temperature[b];
        int32_t *toks = out_tokens + (int64_t)b * out_width;
        int32_t *nodes = accepted_nodes + (int64_t)b * (out_width - 1);
        for (int j = 0; j < out_width; ++j)
            toks[j] = -1;
        for (int j = 0; j < out_width - 1; ++j)
            nodes[j] = -1;
        for (int i = 0; i < k; ++i) {
            if (ratio) ratio[d0 + i] = NAN;
            if (near_tie) near_tie[d0 + i] = 0;
        }
        double *r = (double *)malloc(sizeof(double) * (size_t)V * 2);
        if (!r) {
            fail = 1;
            continue;
        }
        double *q = r + V;
        int cur = 0, n = 0, degenerate = 0;
        softmax_row(target_logits, row0 * row_stride, V, logit_dtype, T, r);
        for (;;) {
            int moved = 0;
            for (int c = cur + 1; c <= k && !moved; ++c) {
                if (tree_parent[row0 + c] != cur)
                    continue;
                int x = draft_tokens[d0 + c - 1];
                double u = (double)u_accept[d0 + c - 1];
                softmax_row(draft_logits, (d0 + c - 1) * row_stride, V, logit_dtype, T, q);
                double rho = r[x] / q[x];
                if (ratio) ratio[d0 + c - 1] = rho;
                if (near_tie) {
                    double capped = rho < 1.0 ? rho : 1.0;
                    near_tie[d0 + c - 1] = (rho == rho) && fabs(u - capped) < tie_eps && rho < 1.0 + tie_eps;
                }
                if (u * q[x] < r[x]) {
                    toks[n] = x;
                    nodes[n] = c;
                    ++n;
                    cur = c;
                    degenerate = 0;
                    softmax_row(target_logits, (row0 + c) * row_stride, V, logit_dtype, T, r);
                    moved = 1;
                } else {
                    double S = 0.0;
                    for (int v = 0; v < V; ++v)
                        S += r[v] > q[v] ? r[v] - q[v] : 0.0;
                    degenerate = !(S > 0.0);
                    if (!degenerate)
                        for (int v = 0; v < V; ++v)
                            r[v] = (r[v] > q[v] ? r[v] - q[v] : 0.0) / S;
                }
            }
            if (!moved)
                break;
        }
        int y = -1;
        if (degenerate) {
            y = argmax_row(target_logits, (row0 + cur) * row_stride, V, logit_dtype);
        } else {
            double S = 0.0, c = 0.0;
            for (int v = 0; v < V; ++v)
                S += r[v];
            double thr = (double)u_sample[b] * S;
            int last_pos = -1;
            for (int v = 0; v < V; ++v) {
                if (!(r[v] > 0.0))
                    continue;
                c += r[v];
                last_pos = v;
                if (y < 0 && c > thr)
                    y = v;
            }
            if (y < 0)
                y = last_pos;
        }
        toks[n] = y;
        accepted_len[b] = n;
        free(r);
    }
    return fail ? -5 : 0;
}

/* ---- KV append and commit (the steps around verification) --------------------
 *
 * Section 3.4, Eq. 7: the decode worker's KV is the prefill KV with every new
 * token's key/value appended.  Before a verification step the k_b+1 new tokens
 * of request b (last accepted token + drafts) are written to the last q_len of
 * the kv_len[b] cache positions: row i of the request goes to position
 * pos = kv_len - q_len + i, i.e. physical block block_table[b][pos/bs], slot
 * pos%bs, for every KV head.  New keys/values arrive as [row][kv head][d] in
 * float32 or bfloat16 and are stored in the cache's format:
 *   float32 cache   the value itself;
 *   bfloat16 cache  the nearest bfloat16, ties to the even mantissa;
 *   e4m3 cache      byte = nearest e4m3fn to clamp(x / scale, +-448), ties to
 *                   even, with x / scale taken in float32 (one IEEE division);
 *                   scale is one float32 per (block, kv head).  A block whose
 *                   slot 0 is written by this call gets a new scale = amax / 448
 *                   (float32 division; 1.0 if amax == 0), amax over this call's
 *                   values for that block and head, keys and values separately;
 *                   a block that already held older tokens keeps its scale.
 *
 * After acceptance, request b keeps its n_b accepted drafts: the valid length
 * becomes kv_len - k_b + n_b (the token drawn by the acceptance step is the
 * first query token of the next step and is appended then).  Rejected slots
 * simply fall beyond the valid length.
 *
 * Pins: tests/test_oracle_kv.py (round trip through an independently built
 * cache, library bfloat16/e4m3 casts, a hand-worked scale example, a token-list
 * simulation of commit).
 */
static uint16_t encode_bf16(float f)
{
    uint32_t w;
    memcpy(&w, &f, 4);
    if (isnan(f))
        return (uint16_t)((w >> 16) | 0x40);
    uint16_t lo = (uint16_t)(w >> 16);   /* towards zero */
    uint16_t hi = (uint16_t)(lo + 1);    /* next one away from zero */
    double x = fabs((double)f), a = fabs(decode_bf16(lo));
    double b = ((hi & 0x7F80) == 0x7F80) ? ldexp(1.0, 128) : fabs(decode_bf16(hi)); /* infinity stands for 2^128 */
    double da = x - a, db = b - x;
    if (da < db) return lo;
    if (db < da) return hi;
    return (lo & 1) ? hi : lo;
}

static uint8_t encode_e4m3fn(float q) /* q finite, |q| <= 448 */
{
    int neg = signbit(q) ? 1 : 0, best = -1;
    double x = fabs((double)q), bd = 0.0;
    for (int c = 0; c < 0x7F; ++c) { /* all finite magnitudes */
        double d = fabs(decode_e4m3fn((uint8_t)c) - x);
        if (best < 0 || d < bd || (d == bd && (c & 1) == 0 && (best & 1) == 1)) {
            best = c;
            bd = d;
        }
    }
    return (uint8_t)(best | (neg << 7));
}

static float new_value(const void *src, int64_t idx, int dtype)
{
    if (dtype == OR_F32) return ((const float *)src)[idx];
    return (float)decode_bf16(((const uint16_t *)src)[idx]);
}

int oracle_kv_append(int B, int Hkv, int D, int bs, int max_blocks, int kv_dtype, void *k_cache, void *v_cache,
                     float *k_scale, float *v_scale, const int32_t *block_table, const int32_t *kv_len,
                     const int32_t *q_indptr, int new_dtype, const void *k_new, const void *v_new)
{
    if (B < 0 || Hkv <= 0 || D <= 0 || bs <= 0 || (new_dtype != OR_F32 && new_dtype != OR_BF16)) return -1;
    if (kv_dtype == OR_FP8_E4M3 && (!k_scale || !v_scale)) return -2;
    for (int b = 0; b < B; ++b) {
        int q_len = q_indptr[b + 1] - q_indptr[b], L = kv_len[b];
        if (q_len < 1 || L < q_len || (L + bs - 1) / bs > max_blocks) return -3;
    }
    for (int side = 0; side < 2; ++side) {
        void *cache = side ? v_cache : k_cache;
        float *scale = side ? v_scale : k_scale;
        const void *src = side ? v_new : k_new;
        for (int b = 0; b < B; ++b) {
            int r0 = q_indptr[b], q_len = q_indptr[b + 1] - r0, P = kv_len[b] - q_len;
            for (int h = 0; h < Hkv; ++h) {
                if (kv_dtype == OR_FP8_E4M3) { /* scales of the blocks this call starts */
                    for (int blk = P / bs; blk <= (kv_len[b] - 1) / bs; ++blk) {
                        if (blk * bs < P) continue; /* holds older tokens: scale stays */
                        float amax = 0.f;
                        for (int i = 0; i < q_len; ++i)
                            if ((P + i) / bs == blk)
                                for (int d = 0; d < D; ++d) {
                                    float a = fabsf(new_value(src, ((int64_t)(r0 + i) * Hkv + h) * D + d, new_dtype));
                                    if (a > amax) amax = a;
                                }
                        int phys = block_table[(int64_t)b * max_blocks + blk];
                        scale[(int64_t)phys * Hkv + h] = amax > 0.f ? amax / 448.0f : 1.0f;
                    }
                }
                for (int i = 0; i < q_len; ++i) {
                    int pos = P + i, phys = block_table[(int64_t)b * max_blocks + pos / bs];
                    int64_t dst = (((int64_t)phys * Hkv + h) * bs + pos % bs) * D;
                    for (int d = 0; d < D; ++d) {
                        float x = new_value(src, ((int64_t)(r0 + i) * Hkv + h) * D + d, new_dtype);
                        if (kv_dtype == OR_F32) {
                            ((float *)cache)[dst + d] = x;
                        } else if (kv_dtype == OR_BF16) {
                            ((uint16_t *)cache)[dst + d] = encode_bf16(x);
                        } else {
                            float q = x / scale[(int64_t)phys * Hkv + h];
                            if (q > 448.0f) q = 448.0f;
                            if (q < -448.0f) q = -448.0f;
                            ((uint8_t *)cache)[dst + d] = isnan(q) ? 0x7F : encode_e4m3fn(q);
                        }
                    }
                }
            }
        }
    }
    return 0;
}

int oracle_kv_commit(int B, const int32_t *q_indptr, const int32_t *accepted_len, int32_t *kv_len)
{
    for (int b = 0; b < B; ++b) {
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        if (accepted_len[b] < 0 || accepted_len[b] > k) return -1;
    }
    for (int b = 0; b < B; ++b) {
        int k = q_indptr[b + 1] - q_indptr[b] - 1;
        kv_len[b] = kv_len[b] - k + accepted_len[b];
    }
    return 0;
}

/* Compaction after acceptance over a draft tree.  The q_len new tokens of request b sit at
 * positions P+i (P = kv_len - q_len, i = node number).  The accepted path a_1 < a_2 < .. < a_n
 * (accepted_nodes, row width nodes_width) must end up at positions P+1 .. P+n, where a chain would
 * have put it, so that oracle_kv_commit's length rule applies unchanged: for j = 1..n in this order,
 * if a_j != j the key/value of every head moves from position P+a_j to position P+j (a_j >= j, and a
 * later move never reads a slot an earlier one wrote).  Storage is copied as it is, except in e4m3
 * caches when source and destination lie in different blocks, whose scales differ: then
 *     byte' = nearest e4m3fn (ties to even) of clamp((decode(byte) * s_src) / s_dst, +-448),
 * product and quotient each one float32 operation.  No scale changes.  Everything else in the cache,
 * the rejected slots included, is left as it was.
 */
int oracle_kv_compact(int B, int Hkv, int D, int bs, int max_blocks, int kv_dtype, void *k_cache, void *v_cache,
                      const float *k_scale, const float *v_scale, const int32_t *block_table, const int32_t *kv_len,
                      const int32_t *q_indptr, const int32_t *accepted_nodes, int nodes_width,
                      const int32_t *accepted_len)
{
    if (B < 0 || Hkv <= 0 || D <= 0 || bs <= 0 || nodes_width < 0) return -1;
    if (kv_dtype == OR_FP8_E4M3 && (!k_scale || !v_scale)) return -2;
    for (int b = 0; b < B; ++b) {
        int q_len = q_indptr[b + 1] - q_indptr[b], L = kv_len[b], n = accepted_len[b];
        if (q_len < 1 || L < q_len || (L + bs - 1) / bs > max_blocks) return -3;
        if (n < 0 || n > q_len - 1 || n > nodes_width) return -4;
        for (int j = 1; j <= n; ++j) {
            int a = accepted_nodes[(int64_t)b * nodes_width + j - 1];
            int prev = j > 1 ? accepted_nodes[(int64_t)b * nodes_width + j - 2] : 0;
            if (a <= prev || a > q_len - 1) return -6;
        }
    }
    size_t esz = kv_dtype == OR_F32 ? 4 : kv_dtype == OR_BF16 ? 2 : 1;
    for (int side = 0; side < 2; ++side) {
        char *cache = (char *)(side ? v_cache : k_cache);
        const float *scale = side ? v_scale : k_scale;
        for (int b = 0; b < B; ++b) {
            int q_len = q_indptr[b + 1] - q_indptr[b], P = kv_len[b] - q_len;
            for (int j = 1; j <= accepted_len[b]; ++j) {
                int a = accepted_nodes[(int64_t)b * nodes_width + j - 1];
                if (a == j) continue;
                int ps = P + a, pd = P + j;
                int64_t bs_src = block_table[(int64_t)b * max_blocks + ps / bs];
                int64_t bs_dst = block_table[(int64_t)b * max_blocks + pd / bs];
                for (int h = 0; h < Hkv; ++h) {
                    int64_t src = ((bs_src * Hkv + h) * bs + ps % bs) * (int64_t)D;
                    int64_t dst = ((bs_dst * Hkv + h) * bs + pd % bs) * (int64_t)D;
                    if (kv_dtype != OR_FP8_E4M3 || bs_src == bs_dst) {
                        memmove(cache + dst * esz, cache + src * esz, esz * (size_t)D);
                        continue;
                    }
                    float s_src = scale[bs_src * Hkv + h], s_dst = scale[bs_dst * Hkv + h];
                    for (int d = 0; d < D; ++d) {
                        float x = (float)decode_e4m3fn(((uint8_t *)cache)[src + d]);
                        float y = x * s_src;
                        float q = y / s_dst;
                        if (q > 448.0f) q = 448.0f;
                        if (q < -448.0f) q = -448.0f;
                        ((uint8_t *)cache)[dst + d] = isnan(q) ? 0x7F : encode_e4m3fn(q);
                    }
                }
            }
        }
    }
    return 0;
}

/* for tests: the two storage encoders on arrays */
void oracle_encode(const float *src, int64_t n, int dtype, void *dst)
{
    for (int64_t i = 0; i < n; ++i) {
        if (dtype == OR_BF16) ((uint16_t *)dst)[i] = encode_bf16(src[i]);
        else ((uint8_t *)dst)[i] = isnan(src[i]) ? 0x7F : encode_e4m3fn(src[i]);
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
