// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "specverify.h"

namespace ss {

// ---- error reporting ---------------------------------------------------------------------
int32_t fail(int32_t code, const char *fmt, ...);   // stores the thread's message, returns code
int32_t hip_fail(hipError_t e, const char *what);   // SS_ERR_DEVICE with the HIP text

#define SS_HIP_CHECK(expr, what)                      \
    do {                                              \
        hipError_t e__ = (expr);                      \
        if (e__ != hipSuccess) return ss::hip_fail(e__, what); \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- attention -----------------------------------------------------------------------------
constexpr int kTile = SS_BLOCK_SIZE;     // tokens per KV tile = tokens per cache block
constexpr int kWavesPerWg = 4;
constexpr int kMinTilesPerWave = 8;      // below this a KV partition is not worth its partial write
constexpr int kDescInts = 16;            // ints per wave descriptor
constexpr int kDescAddrs = 4;            // tile addresses a descriptor carries for the span's first tiles
constexpr int kMfmaHeadDim = 128;        // head_dim the matrix-core kernel is written for
constexpr int kMaxRowBlocks = 5;         // 16-row blocks of query rows one wavefront can keep accumulators for
constexpr int kUnitWeight = 3;           // default cost of opening a unit, in tiles, for the span cuts

// Query tokens of a request that fall into the pass's window, and the KV tiles its units stream in this
// pass: a request without rows in the window keeps one tile so that no unit of the flat tile space is empty.
__host__ __device__ inline int window_q_len(int q_len, int q_lo, int q_win)
{
    const int n = q_len - q_lo;
    return n < 0 ? 0 : (n > q_win ? q_win : n);
}
// Query rows per (request, KV head) that the partial slots are sized for: the hinted bound, or one pass's window.
inline int attn_rows_pad(int max_q_len, int G)
{
    const int cap = 16 * kMaxRowBlocks, rows = max_q_len * G;
    if (rows <= cap || cap / G == 0) return (int)align_up((size_t)rows, 16);
    const int win_max = cap / G, passes = (max_q_len + win_max - 1) / win_max;
    return (int)align_up((size_t)((max_q_len + passes - 1) / passes) * G, 16);
}
__host__ __device__ inline int window_tiles(int kv_len, int q_len, int q_lo)
{
    return q_len > q_lo ? (kv_len + kTile - 1) / kTile : 1;
}

// Written by the plan kernel, read by the streaming and merge kernels.
struct AttnPlan {
    int32_t total_tiles;   // sum over requests of ceil(kv_len/16) * num_kv_heads
    int32_t num_waves;     // partitions actually used (<= launched wavefronts)
    int32_t unit_weight;   // virtual tiles per unit in the coordinate the spans were cut in (0: plain tile counts)
    int32_t pad;
};

struct AttnArgs {
    // cache
    const void *k, *v;
    const float *k_scale, *v_scale;
    int32_t num_kv_heads, head_dim, kv_dtype;
    // batch
    int32_t batch, max_blocks;
    const int32_t *block_table, *kv_len, *q_indptr;
    const uint32_t *tree_mask;   // per query row, or nullptr for chains: which new tokens of its request the row attends
    // query / output
    const void *q;
    void *out;
    float *lse;
    int32_t q_dtype, num_q_heads, total_rows, max_q_len;
    // Query-token window of this pass: the kernels compute query tokens q_lo .. q_lo+q_win-1 of every
    // request (those it has).  One pass covers everything unless a request can bring more rows per KV
    // head than a wavefront holds; then the launcher walks the windows one after the other.
    int32_t q_lo, q_win;
    int32_t reuse_plan;    // the workspace already holds this batch's plan (single-pass launches only)
    float sm_scale;
    // workspace carve-up
    AttnPlan *plan;
    int32_t *tile_prefix;  // [batch+1] exclusive prefix of ceil(kv_len/16)
    int32_t *tile_addr;    // [batch*max_blocks*kv_heads] flat tile list: physical block * kv_heads + kv head
    int32_t *wave_desc;    // [launch_waves][kDescInts]: where each wave's span starts and what its first loads need
    float *part_o;         // [slots][rows_pad][head_dim]
    float *part_ml;        // [slots][rows_pad][2]  (log2-domain max, sum)
    int32_t rows_pad;      // query rows per (request, kv head), padded to 16
    int32_t launch_waves;  // upper bound of streaming wavefronts (sizes the partial slots)
    int32_t unit_weight;   // what opening a unit costs a wave, in tiles (weights the span cuts; 0 = equal tile counts)
    int32_t chain;         // set by the launcher: partials are per (workgroup, unit), units inside one workgroup are final
};

size_t attn_workspace_bytes(int batch, int max_blocks, int num_q_heads, int num_kv_heads, int head_dim,
                            int launch_waves, int max_q_len);
bool attn_mfma_supported(const AttnArgs &a);
int32_t attn_mfma_launch(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);
int32_t attn_mfma_launch_g1(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);   // per head grouping,
int32_t attn_mfma_launch_g2(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);   // after the plan kernel
int32_t attn_mfma_launch_g4(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);
int32_t attn_mfma_launch_g8(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);
int32_t attn_generic_launch(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1);
int attn_default_waves();

// ---- accept --------------------------------------------------------------------------------
constexpr int kChunk = 8192;  // vocabulary entries per workgroup in the streaming passes

struct AcceptArgs {
    int32_t batch, vocab, logit_dtype, total_rows, greedy;
    int32_t max_q_len;   // bound of k_b + 1 over the batch (sizes the row-statistics grid)
    int64_t row_stride;
    const int32_t *q_indptr;
    const void *target, *draft;
    const int32_t *draft_tokens;
    const float *u_accept, *u_sample, *temperature;
    float temperature_scalar;
    int32_t *accepted_len, *out_tokens;
    float *ratio_out;
    void *workspace;
    // greedy walk over draft trees (both NULL for chains)
    const int32_t *tree_parent;   // per target row: parent node within the request, -1 for node 0
    int32_t *accepted_nodes;      // [batch][SS_MAX_DEPTH]
};
size_t accept_workspace_bytes(int batch, int total_rows, int vocab);
int32_t accept_launch(const AcceptArgs &a, hipStream_t stream);
int32_t accept_rowstats_launch(const AcceptArgs &a, hipStream_t stream);   // the first pass alone (row maxima and sums)
int32_t spec_accept_call(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype, int32_t total_rows,
                         int32_t max_q_len, const int32_t *q_indptr, const void *target_logits, const void *draft_logits,
                         const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                         const float *temperature, float temperature_scalar, int32_t greedy, int32_t *accepted_len,
                         int32_t *out_tokens, float *ratio_out, void *workspace, size_t workspace_bytes, void *stream,
                         bool apply_validate);   // argument checks + launch of ss_spec_accept
size_t accept_tree_workspace_bytes(int batch, int total_rows, int vocab);
int32_t accept_tree_sample_launch(const AcceptArgs &a, hipStream_t stream);

// ---- KV append / commit ----------------------------------------------------------------------
struct KvAppendArgs {
    void *k, *v;
    float *k_scale, *v_scale;
    int32_t num_kv_heads, head_dim, kv_dtype;
    int32_t batch, max_blocks;
    const int32_t *block_table, *kv_len, *q_indptr;
    const void *k_new, *v_new;
    int32_t new_dtype;
    int32_t max_q_len;   // bound of the new tokens per request (sizes the append grid)
};
int32_t kv_append_launch(const KvAppendArgs &a, hipStream_t stream);
int32_t kv_compact_launch(const KvAppendArgs &a, const int32_t *accepted_nodes, const int32_t *accepted_len,
                          hipStream_t stream);   // k_new/v_new/new_dtype of the arguments are not used
int32_t kv_commit_launch(int batch, const int32_t *q_indptr, const int32_t *accepted_len, int32_t *kv_len,
                         hipStream_t stream);

// ---- optional checks of device-resident metadata (option "validate") ---------------------------------
int32_t validate_batch(const int32_t *block_table, const int32_t *kv_len, const int32_t *q_indptr,
                       const uint32_t *tree_mask, int batch, int max_blocks, int num_blocks, int total_rows, int max_q_len, hipStream_t stream, const char *what);
int32_t validate_accept(const int32_t *draft_tokens, const float *u_accept, const float *u_sample, const float *temperature,
                        int batch, int n_draft, int vocab, int greedy, hipStream_t stream, const char *what);

}  // namespace ss
