/*
 * specverify: the decode lane's speculative-verification step on one MI355X.
 *
 * Two operations, both defined by the method the paper builds on (Section 2.2:
 * draft tokens are verified by the target model in one parallel pass while the
 * target's output distribution is preserved), with the per-request draft depth
 * k chosen by the paper's controller (Section 3.5, Alg. 4, Eq. 13) and handed
 * in as a ragged row count:
 *
 *   ss_spec_verify_attn  attention of each request's k+1 new tokens (causal
 *                        among themselves) over its paged KV cache
 *                        (Section 2.4; the cache holds prefill KV with decoded
 *                        tokens appended, Section 3.4 Eq. 7)
 *   ss_spec_accept       accept/reject walk over the k drafts and the draw of
 *                        the one new token (residual or bonus distribution)
 *
 * Around them, the other steps of a decode loop: ss_kv_append (write the new
 * tokens' K/V before verification), ss_kv_commit (valid lengths after
 * acceptance), for tree-shaped drafts ss_batch.tree_mask,
 * ss_spec_accept_tree_greedy and ss_kv_compact, and as host arithmetic the
 * paper's depth controller (ss_depth_update, Section 3.5) and router
 * (ss_route_select, Section 3.2).
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory on the current device, "host"
 *     pointers ordinary host memory.  The caller owns every buffer, including
 *     the workspace; the library allocates no device memory, frees nothing and
 *     keeps no state between calls (except the optional profiling events).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.
 *   - Return value: SS_OK or an ss_status error; ss_last_error() gives the
 *     thread's last message.  Host-visible arguments are validated before
 *     anything is launched; on error nothing has been enqueued.  Contents of
 *     device arrays (block ids inside the pool, kv_len >= q_len, draft tokens
 *     inside the vocabulary) are the caller's responsibility.
 *   - There is no CPU fallback: without a usable GPU the calls fail with
 *     SS_ERR_DEVICE.
 */
#ifndef SPECVERIFY_H
#define SPECVERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SS_OK = 0,
    SS_ERR_INVALID_ARG = 1, /* null pointer, bad size, bad dtype, misaligned buffer */
    SS_ERR_UNSUPPORTED = 2, /* valid, but no kernel is built for this combination */
    SS_ERR_WORKSPACE = 3,   /* workspace smaller than the *_workspace() query */
    SS_ERR_DEVICE = 4       /* HIP reported an error (message has the HIP text) */
} ss_status;

typedef enum {
    SS_F32 = 0,
    SS_BF16 = 1,     /* bfloat16: upper 16 bits of an IEEE float32 */
    SS_FP8_E4M3 = 2  /* OCP e4m3fn byte (bias 7, max 448, no inf, NaN = S.1111.111); KV cache only */
} ss_dtype;

#define SS_BLOCK_SIZE 16 /* tokens per KV block */
#define SS_MAX_DEPTH 20  /* largest k (the controller's d_max, Section 3.5); a request brings 1..21 query rows */
#define SS_OUT_WIDTH 21  /* out_tokens row width = SS_MAX_DEPTH + 1 */

/*
 * Paged KV cache of one layer (Section 2.4).
 *   k, v     device, dense [num_blocks][num_kv_heads][block_size][head_dim] in `dtype`,
 *            16-byte aligned.  Slots past a request's kv_len and blocks no request
 *            references may hold anything (NaN included); they are never used.
 *   k_scale, v_scale  device float [num_blocks][num_kv_heads]; required iff dtype is
 *            SS_FP8_E4M3 (value = decode(byte) * scale), must be NULL otherwise.
 */
typedef struct ss_paged_kv {
    int32_t num_blocks;
    int32_t block_size; /* must be SS_BLOCK_SIZE */
    int32_t num_kv_heads;
    int32_t head_dim;   /* 64 or 128 */
    int32_t dtype;      /* ss_dtype */
    const void *k;
    const void *v;
    const float *k_scale;
    const float *v_scale;
} ss_paged_kv;

/*
 * One decode-lane batch.
 *   block_table  device int32 [batch][max_blocks_per_seq]: logical block j of request b
 *                is physical block block_table[b][j]; entries past ceil(kv_len/16) are ignored.
 *   kv_len       device int32 [batch]: valid cache positions of each request, INCLUDING the
 *                q_len new tokens of this step, whose K/V the caller has already appended.
 *   q_indptr     device int32 [batch+1]: request b owns query rows q_indptr[b]..q_indptr[b+1]-1
 *                (q_len = k_b + 1 in 1..SS_OUT_WIDTH, row i = the i-th new token, at position kv_len-q_len+i).
 *   max_q_len    host value: an upper bound of q_len over the batch (the controller's largest depth
 *                this step, plus one), or 0 if unknown (SS_OUT_WIDTH is assumed).  A tight bound lets the
 *                library pick a kernel with fewer padded query rows; a bound that some request
 *                exceeds is a caller error (rows beyond it are not computed).
 *   flags        SS_BATCH_REUSE_PLAN tells ss_spec_verify_attn that its workspace still holds the plan an
 *                earlier call built for exactly this batch (same block_table, kv_len, q_indptr contents,
 *                same max_q_len, head counts and workspace; only q, the cache contents and the outputs
 *                may differ): the layers of one decode step share their batch, so all but the first
 *                can skip the plan kernel.  Ignored where no stored plan can serve (the vector kernel,
 *                or a row bound that takes several passes).  Other calls ignore the field.
 *   tree_mask    NULL: the new tokens of a request form a chain (row i attends new tokens 0..i).
 *                Otherwise device uint32 [total rows]: the new tokens form a draft tree (the dynamic
 *                draft trees of the speculative systems the paper builds on, Section 2.2) with row 0
 *                the root; bit j of a row's word says that the row attends new token j of its own request
 *                (position kv_len-q_len+j), i.e. that node j is the row's own node or an ancestor of it.
 *                Every row's own bit must be set and no bit at or above q_len; the context before the new
 *                tokens is always visible.  Read by ss_spec_verify_attn only.
 */
#define SS_BATCH_REUSE_PLAN 1

typedef struct ss_batch {
    int32_t batch;
    int32_t max_blocks_per_seq;
    int32_t max_q_len;
    int32_t flags;    /* 0 or SS_BATCH_REUSE_PLAN */
    const int32_t *block_table;
    const int32_t *kv_len;
    const int32_t *q_indptr;
    const uint32_t *tree_mask;
} ss_batch;

/* Library version (major*10000 + minor*100 + patch). */
int32_t ss_version(void);

/* Message of the calling thread's most recent failing call ("" if none). Never NULL. */
const char *ss_last_error(void);

/*
 * Bytes of device workspace ss_spec_verify_attn needs for this shape (256-byte aligned
 * buffer).  Depends only on the host-visible fields, not on device contents (batch->max_q_len
 * included: a workspace sized for a larger bound, or for 0, also serves calls with a smaller one).
 * Returns 0 and sets the error message if the arguments are invalid.
 */
size_t ss_spec_verify_attn_workspace(const ss_paged_kv *kv, const ss_batch *batch, int32_t num_q_heads,
                                     int32_t total_rows);

/*
 * Verify attention (Section 2.2 "parallel verification", over the cache of Sections 2.4/3.4).
 * For request b, new token i, query head h (KV head h / (num_q_heads/num_kv_heads)):
 *     s_t = sm_scale * <q[row,h,:], K_b[t,:]>   for cache positions t = 0 .. kv_len_b - q_len_b + i
 *     out[row,h,:] = sum_t softmax(s)_t * V_b[t,:],      lse[row,h] = ln sum_t exp(s_t)
 *
 *   q      device [total_rows][num_q_heads][head_dim], q_dtype SS_F32 or SS_BF16, 16-byte aligned
 *   out    device, same shape and dtype as q (rounded to nearest even from fp32 accumulators)
 *   lse    device float [total_rows][num_q_heads], or NULL
 *   total_rows  must equal q_indptr[batch] (host copy of that value)
 *   workspace   device, >= ss_spec_verify_attn_workspace(...) bytes; contents are scratch
 *
 * Internally the KV stream is cut into partitions that are reduced independently and merged
 * by their log-sum-exp; the result does not depend on the partitioning beyond fp32 rounding.
 * The matrix-core kernel covers head_dim 128, bf16 queries, bf16 or e4m3 caches and 1/2/4/8 query heads per
 * KV head.  One pass over the cache serves up to 80 query rows per KV head (max_q_len * heads per KV head:
 * depth 9 for groups of 8, depth 19 for groups of 4, any depth for smaller groups); a larger bound is
 * served in two or three passes over equal windows of query tokens, each reading the cache again.
 * Everything else takes a plain fp32 vector kernel that has no shape limits and is far slower.
 * batch == 0 or total_rows == 0 is a no-op returning SS_OK.
 */
int32_t ss_spec_verify_attn(const ss_paged_kv *kv, const ss_batch *batch, const void *q, int32_t q_dtype,
                            int32_t num_q_heads, int32_t total_rows, float sm_scale, void *out, float *lse,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device workspace ss_spec_accept needs (0 + error message on invalid arguments). */
size_t ss_spec_accept_workspace(int32_t batch, int32_t total_rows, int32_t vocab);

/*
 * Acceptance walk and resampling (the speculative-sampling rule behind Section 2.2's
 * "preserving output distribution").  Request b has k = q_len-1 drafts x_0..x_{k-1}; its
 * target rows are rows q_indptr[b].. of target_logits (row i judges draft i, row k is the
 * bonus distribution); its draft rows / tokens / u_accept entries start at q_indptr[b]-b.
 *
 *     p_i = softmax(target_i / T_b),  q_i = softmax(draft_i / T_b)
 *     accept draft i iff u_accept_i < p_i[x_i] / q_i[x_i]; n = index of the first rejection (k if none)
 *     r = max(0, p_n - q_n) if n < k, else p_k;  y = first token whose running sum of r (token
 *     order) exceeds u_sample_b * sum(r)
 *     out_tokens[b] = x_0..x_{n-1}, y, then -1 up to SS_OUT_WIDTH;  accepted_len[b] = n
 *   greedy != 0: accept while the lowest-index argmax of target_i equals x_i; y = that argmax of
 *   target_n; temperatures and uniforms are not read (their pointers may be NULL).
 *
 *   vocab, row_stride   logits rows hold `vocab` entries, `row_stride` elements apart (>= vocab)
 *   logit_dtype         SS_F32 or SS_BF16; rows must start 16-byte aligned
 *   total_rows          host copy of q_indptr[batch]; the draft-side arrays have total_rows-batch entries
 *   max_q_len           host value: an upper bound of k_b+1 over the batch, or 0 if unknown (SS_OUT_WIDTH is
 *                       assumed); as for ss_batch.max_q_len a tight bound only saves idle workgroups, and a bound
 *                       that some request exceeds is a caller error
 *   temperature         device float [batch] (> 0), or NULL to use temperature_scalar for all
 *   ratio_out           device float [total_rows-batch] or NULL: p/q of every draft (diagnostic)
 *   Row statistics are accumulated in fp32/fp64; the resampling pass runs in fp64 so that the
 *   drawn token is reproducible against an fp64 reference.
 */
int32_t ss_spec_accept(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype, int32_t total_rows,
                       int32_t max_q_len, const int32_t *q_indptr, const void *target_logits, const void *draft_logits,
                       const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                       const float *temperature, float temperature_scalar, int32_t greedy, int32_t *accepted_len,
                       int32_t *out_tokens, float *ratio_out, void *workspace, size_t workspace_bytes,
                       void *stream);

/*
 * ss_spec_accept for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * ss_spec_accept minus the workspace: the partial results live in a static array of
 * SS_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU the library is used on, held
 * until the process ends).  The call allocates and frees nothing, on the device or the host, and
 * never synchronises; option "validate" does not apply to it.
 *   - A shape whose scratch need (ss_spec_accept_workspace) exceeds SS_STATIC_SCRATCH_BYTES is rejected with
 *     SS_ERR_WORKSPACE before anything is launched (16 MiB serves e.g. 128 requests at depth 8 with a
 *     152 064-entry vocabulary, or 200 requests at depth 20).
 *   - All calls on one GPU share that GPU's array: calls that can overlap on one GPU (different streams,
 *     different threads) race on it and must be serialised by the caller; calls on one stream are ordered.
 *     The array keeps what the last call left; the kernels initialise whatever they read.
 * ss_spec_accept_static_capacity returns SS_STATIC_SCRATCH_BYTES as the library was built.
 */
#define SS_STATIC_SCRATCH_BYTES (16u << 20)
size_t ss_spec_accept_static_capacity(void);
int32_t ss_spec_accept_static(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype, int32_t total_rows,
                              int32_t max_q_len, const int32_t *q_indptr, const void *target_logits,
                              const void *draft_logits, const int32_t *draft_tokens, const float *u_accept,
                              const float *u_sample, const float *temperature, float temperature_scalar, int32_t greedy,
                              int32_t *accepted_len, int32_t *out_tokens, float *ratio_out, void *stream);

/*
 * Greedy acceptance over draft trees (Section 2.2: dynamic draft trees, verified in one parallel
 * pass with the target's output preserved; here at temperature 0).  The new tokens of
 * request b form a tree: node 0 is the last accepted token, node i in 1..k carries draft token
 * draft_tokens[q_indptr[b]-b+i-1] and hangs under node tree_parent[q_indptr[b]+i] < i; target row i
 * holds the logits that follow node i (computed by ss_spec_verify_attn with the matching tree_mask).
 *     cur = 0; repeat: t = lowest-index argmax of target row cur; c = lowest-numbered child of cur
 *     whose token is t; none: stop; else accept c, cur = c
 *   out_tokens[b]      the accepted tokens, then t of the node where the walk stopped, then -1
 *                      (SS_OUT_WIDTH entries): exactly what greedy decoding of the target emits
 *   accepted_len[b]    number of accepted nodes n
 *   accepted_nodes[b]  device int32 [batch][SS_MAX_DEPTH]: the accepted node numbers in path order,
 *                      -1 beyond n (what a cache compaction needs)
 *   tree_parent        device int32 [total_rows]; -1 for every request's node 0
 * Other arguments, the workspace (ss_spec_accept_workspace) and errors as for ss_spec_accept.
 */
int32_t ss_spec_accept_tree_greedy(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype,
                                   int32_t total_rows, int32_t max_q_len, const int32_t *q_indptr, const int32_t *tree_parent,
                                   const void *target_logits, const int32_t *draft_tokens, int32_t *accepted_len,
                                   int32_t *out_tokens, int32_t *accepted_nodes, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * Sampled acceptance over draft trees (Section 2.2, as above, at temperature > 0).  Tree layout as for
 * ss_spec_accept_tree_greedy; draft row i-1 of the request (row q_indptr[b]-b+i-1 of draft_logits) is the
 * distribution node i's token was drawn from (siblings drawn from one proposal carry equal rows), and
 * u_accept at the same index is its uniform.  The walk starts at node 0 with r = softmax(target row 0 / T)
 * and offers r the children of the current node in node order, each as one step of speculative sampling
 * against its own proposal q_c = softmax(draft row of c / T):
 *     accept c iff u_c * q_c[x_c] < r[x_c]; then c is the current node, r = softmax(target row c / T)
 *     rejected: r <- max(0, r - q_c) / sum(max(0, r - q_c))  (unchanged if that sum is 0); next sibling
 *     no child left: y = first token whose running sum of r (token order) exceeds u_sample_b * sum(r); if the
 *     last rejection left no residual mass, y = lowest-index argmax of the current node's target row
 * Every step leaves the distribution that plain sampling from the target would have at that point, so the
 * emitted tokens are distributed as the target's own; a chain gives the result of ss_spec_accept.
 *   out_tokens, accepted_len, accepted_nodes   as for ss_spec_accept_tree_greedy
 *   ratio_out   device float [total_rows-batch] or NULL: r[x]/q[x] of every node that was offered, NaN elsewhere
 *   workspace   >= ss_spec_accept_tree_sample_workspace(...) bytes (it holds two fp64 vocabulary vectors
 *               per request besides the row statistics)
 *   max_q_len   also bounds the number of rejections a request can have, hence the number of rounds the
 *               call enqueues (a walk, block sums and a residual pass per round): a tight bound saves launches
 * Children are judged from two gathered logits and the row statistics (fp32 chunk sums, relative error
 * below 1e-6, as in ss_spec_accept); residuals, their normalisers and the draw are fp64 with fixed reduction
 * orders.  Other arguments and errors as for ss_spec_accept.
 */
size_t ss_spec_accept_tree_sample_workspace(int32_t batch, int32_t total_rows, int32_t vocab);
int32_t ss_spec_accept_tree_sample(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype,
                                   int32_t total_rows, int32_t max_q_len, const int32_t *q_indptr,
                                   const int32_t *tree_parent, const void *target_logits, const void *draft_logits,
                                   const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                                   const float *temperature, float temperature_scalar, int32_t *accepted_len,
                                   int32_t *out_tokens, int32_t *accepted_nodes, float *ratio_out, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * KV append, the step before verification (paper Section 3.4, Eq. 7: the decode KV is the prefill KV
 * with the new tokens' keys/values appended; Section 2.4: paged layout).  Request b's
 * q_len = q_indptr[b+1]-q_indptr[b] new tokens are written to the last q_len of its kv_len[b] cache
 * positions (kv_len already counts them): row i goes to position kv_len[b]-q_len+i, i.e. block
 * block_table[b][pos/16], slot pos%16, for every KV head.
 *   kv            the cache to write.  Its k, v (and for SS_FP8_E4M3 k_scale, v_scale) buffers are
 *                 WRITTEN through although the struct declares them const for the read-only calls.
 *   batch         block_table, kv_len, q_indptr, max_q_len as for ss_spec_verify_attn (tree_mask is not read).
 *   k_new, v_new  device, [total_rows][num_kv_heads][head_dim], dense, new_dtype = SS_F32 or SS_BF16.
 * Stored as: SS_F32 cache the value; SS_BF16 cache nearest bfloat16, ties to even; SS_FP8_E4M3 cache
 * byte = nearest e4m3fn (ties to even) of clamp(x / scale, +-448) with x / scale one float32
 * division.  A block whose slot 0 is written by this call gets scale = amax / 448 (1.0 if amax is 0)
 * over this call's values for that block and KV head, keys and values separately; a block that already
 * holds older tokens keeps its scale.  NaN inputs give unspecified NaN payloads.
 * The caller owns all buffers; nothing is allocated; the kernel is enqueued on `stream`.
 * Errors: SS_ERR_INVALID_ARG (NULL pointers, bad dtypes or sizes), SS_ERR_DEVICE (launch failure).
 * Device-side contents (block ids in range, kv_len >= q_len, q_len <= SS_OUT_WIDTH) are the caller's contract.
 */
int32_t ss_kv_append(const ss_paged_kv *kv, const ss_batch *batch, const void *k_new, const void *v_new,
                     int32_t new_dtype, int32_t total_rows, void *stream);

/*
 * Compaction after acceptance over a draft tree (between ss_spec_accept_tree_greedy and ss_kv_commit).
 * The q_len new tokens of request b sit at cache positions P+i, P = kv_len[b]-q_len, i = node number.
 * Its accepted path accepted_nodes[b][0..n-1] = a_1 < .. < a_n (n = accepted_len[b]) is moved to
 * positions P+1 .. P+n, where a chain would have put it, so that ss_kv_commit's length rule applies
 * unchanged: in path order, if a_j != j the key and value of every KV head move from position P+a_j to
 * P+j.  Storage is copied as it is, except e4m3 bytes whose source and destination lie in different
 * blocks: byte' = nearest e4m3fn (ties to even) of clamp((decode(byte) * scale_src) / scale_dst, +-448),
 * product and quotient one float32 operation each.  No scale changes; all other slots, the rejected
 * ones included, keep their contents.  For a chain (a_j = j) nothing moves.
 *   kv, batch       as for ss_kv_append (kv_len still counts all q_len new tokens; the cache is WRITTEN)
 *   accepted_nodes  device int32 [batch][SS_MAX_DEPTH], as written by ss_spec_accept_tree_greedy
 *   accepted_len    device int32 [batch]
 * A row of accepted_nodes that is not increasing within 1..q_len-1 ends that request's moves at the
 * offending entry (nothing outside the request's new slots is ever touched).
 * Errors: SS_ERR_INVALID_ARG (NULL pointers, bad dtypes or sizes), SS_ERR_DEVICE (launch failure).
 */
int32_t ss_kv_compact(const ss_paged_kv *kv, const ss_batch *batch, const int32_t *accepted_nodes,
                      const int32_t *accepted_len, int32_t total_rows, void *stream);

/*
 * Commit after acceptance (same passage): request b keeps its accepted_len[b] accepted drafts, so its
 * valid cache length becomes kv_len[b] - k_b + accepted_len[b] with k_b = q_indptr[b+1]-q_indptr[b]-1;
 * the rejected slots fall past the end (no data moves), and the token the acceptance step drew is
 * appended by the next step.  All arrays are device arrays; kv_len [batch] is updated in place.
 * Errors: SS_ERR_INVALID_ARG (NULL pointers, negative batch), SS_ERR_DEVICE.
 */
int32_t ss_kv_commit(int32_t batch, const int32_t *q_indptr, const int32_t *accepted_len, int32_t *kv_len,
                     void *stream);

/*
 * Speculation-depth controller (paper Section 3.5, Eq. 8-16, Algorithm 4): host arithmetic only, no
 * device work.  One ss_depth_state is the state of one stream of updates (the flow vector of the last h
 * acceptance gradients, its write index, the smoothed throughput).  ss_depth_init fills a state with the
 * paper's typical parameters (h 10, d_base 5, gamma 5, d_min 2, d_max 20, tau_target 400, tau_recent 0);
 * the caller may then change the parameter fields.  ss_depth_update takes the metrics of the step just
 * finished (accept_rate = accepted drafts / drafts in [0,1], load, throughput in tokens/s) and returns
 * the clipped real depth d_star, the micro-batch size, the projected throughput, and k = the integer
 * depth for the next verify step: floor(d_star + 1/2), at most SS_MAX_DEPTH.  Arithmetic is IEEE double.
 * Where Algorithm 4 and the equations differ (which throughput scales and projects) the algorithm is
 * followed: the `throughput` argument in both places.
 * Errors: SS_ERR_INVALID_ARG (NULL state or output, h outside [1, SS_FLOW_MAX], NaN metrics).
 */
#define SS_FLOW_MAX 64
typedef struct {
    int32_t h;   /* history length */
    int32_t idx; /* next slot of f to overwrite */
    double f[SS_FLOW_MAX];
    double d_base, gamma, d_min, d_max, tau_target, tau_recent;
} ss_depth_state;

int32_t ss_depth_init(ss_depth_state *state);
int32_t ss_depth_update(ss_depth_state *state, double accept_rate, double load, double throughput, double *d_star,
                        int32_t *b_micro, double *t_proj, int32_t *k);

/*
 * Router worker selection (paper Section 3.2, Eq. 1-4, Algorithm 2): host arithmetic only.  Worker i
 * reports cache hit rate, memory utilisation and active load in [0,1], its queue depth, and whether its
 * metrics are stale.  A worker is eligible if it is not stale and its overload score
 * mem + 2 * depth / q_max does not exceed tau (Eq. 2, 3; the memory term of Eq. 3 is the paper's
 * "per cent / 100", i.e. the same number in [0,1]).  Among the eligible workers the one with the highest
 * score alpha[0]*cache + alpha[1]*(1-mem) + alpha[2]*(1-min(depth/q_max,1)) + alpha[3]*(1-load) is chosen
 * (Eq. 1); if none is eligible, the worker with the smallest queue depth among all (Eq. 4).  Ties go to
 * the lowest index.  alpha == NULL takes the paper's weights (0.4, 0.1, 0.3, 0.2); tau <= 0 takes 0.85.
 * Arithmetic is IEEE double.  Errors: SS_ERR_INVALID_ARG (n <= 0, NULL workers/chosen, q_max <= 0).
 */
typedef struct {
    double cache_hit, mem, load;
    int32_t queue_depth;
    int32_t stale;
} ss_worker_metrics;

int32_t ss_route_select(const ss_worker_metrics *workers, int32_t n, const double *alpha, double tau, double q_max,
                        int32_t *chosen);

/*
 * Options (process-wide, not thread-safe; meant for tests and measurement).
 *   "attn_path"     0 = automatic, 1 = force the plain fp32 vector kernel, 2 = require the MFMA kernel
 *   "attn_waves"    number of KV stream partitions (wavefronts) of the MFMA kernel, 0 = automatic
 *   "attn_unit_weight"  what opening a (request, KV head) unit is taken to cost a wavefront, in KV tiles, when the
 *                   KV stream is cut into partitions (default 3; 0 = partitions of equal tile counts)
 *   "validate"      1 = before launching, ss_spec_verify_attn, ss_kv_append and ss_spec_accept check the
 *                   device-resident metadata with a small kernel (row offsets, lengths against block counts,
 *                   block ids, draft tokens, temperatures, uniforms), synchronise the stream and return
 *                   SS_ERR_INVALID_ARG naming the first inconsistency; 0 (default) = contents are trusted
 * Returns SS_ERR_INVALID_ARG for an unknown name or value.
 */
int32_t ss_set_option(const char *name, int64_t value);

/*
 * Kernel timing for the benchmark.  After ss_profile_begin(n) the next n calls of
 * ss_spec_verify_attn record a HIP event pair around their KV-streaming kernel (the dominant
 * one) on the caller's stream.  ss_profile_collect synchronises on those events, writes up to
 * `cap` durations in milliseconds to the host array `ms`, returns how many were written and
 * ends profiling.  Events are the only objects the library creates; they are destroyed here.
 */
int32_t ss_profile_begin(int32_t max_calls);
int32_t ss_profile_collect(float *ms, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* SPECVERIFY_H */
