// C-ABI entry points: argument validation, workspace sizing, dispatch.  No arithmetic here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "common.h"

namespace ss {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int32_t hip_fail(hipError_t e, const char *what)
{
    return fail(SS_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

// process-wide options and profiling state
static int64_t g_attn_path = 0;
static int64_t g_attn_waves = 0;
static int64_t g_validate = 0;
static int64_t g_unit_weight = kUnitWeight;
static std::vector<hipEvent_t> g_events;  // pairs
static int g_prof_cap = 0, g_prof_used = 0;

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int32_t check_attn_shape(const ss_paged_kv *kv, const ss_batch *b, int32_t num_q_heads, int32_t total_rows)
{
    if (!kv || !b) return fail(SS_ERR_INVALID_ARG, "kv and batch descriptors must not be NULL");
    if (kv->block_size != SS_BLOCK_SIZE)
        return fail(SS_ERR_INVALID_ARG, "block_size must be %d, got %d", SS_BLOCK_SIZE, kv->block_size);
    if (kv->head_dim != 64 && kv->head_dim != 128)
        return fail(SS_ERR_INVALID_ARG, "head_dim must be 64 or 128, got %d", kv->head_dim);
    if (kv->num_kv_heads <= 0 || num_q_heads <= 0 || num_q_heads % kv->num_kv_heads)
        return fail(SS_ERR_INVALID_ARG, "num_q_heads (%d) must be a positive multiple of num_kv_heads (%d)",
                    num_q_heads, kv->num_kv_heads);
    if (num_q_heads / kv->num_kv_heads > 16)
        return fail(SS_ERR_UNSUPPORTED, "more than 16 query heads per KV head is not built");
    if (kv->dtype < SS_F32 || kv->dtype > SS_FP8_E4M3)
        return fail(SS_ERR_INVALID_ARG, "unknown KV dtype %d", kv->dtype);
    if (b->batch < 0 || total_rows < 0) return fail(SS_ERR_INVALID_ARG, "negative batch or total_rows");
    if (total_rows < b->batch || (int64_t)total_rows > (int64_t)b->batch * SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "total_rows (%d) must lie in [batch, %d*batch] for batch %d", total_rows,
                    SS_OUT_WIDTH, b->batch);
    if (b->batch > 0 && b->max_blocks_per_seq <= 0)
        return fail(SS_ERR_INVALID_ARG, "max_blocks_per_seq must be positive");
    if (kv->num_blocks < 0) return fail(SS_ERR_INVALID_ARG, "negative num_blocks");
    if ((int64_t)kv->num_blocks * kv->num_kv_heads > 0x7fffffffll ||
        (int64_t)b->batch * b->max_blocks_per_seq * kv->num_kv_heads > 0x7fffffffll)
        return fail(SS_ERR_UNSUPPORTED, "num_blocks * num_kv_heads and batch * max_blocks * num_kv_heads must fit 31 bits");
    if (b->max_q_len < 0 || b->max_q_len > SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "max_q_len must be 0 (unknown) or in [1, %d]", SS_OUT_WIDTH);
    if (b->flags & ~SS_BATCH_REUSE_PLAN) return fail(SS_ERR_INVALID_ARG, "unknown bits in ss_batch.flags (%d)", b->flags);
    return SS_OK;
}

int attn_default_waves()
{
    if (g_attn_waves > 0) return (int)g_attn_waves;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    } else {
        (void)hipGetLastError();
    }
    return cus * 4;  // one wavefront per SIMD
}

// The checks and the launch behind ss_spec_accept; ss_spec_accept_static calls it with its own buffer and
// without the optional metadata check (which synchronises and owns a pinned host record).
int32_t spec_accept_call(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype, int32_t total_rows,
                         int32_t max_q_len, const int32_t *q_indptr, const void *target_logits, const void *draft_logits,
                         const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                         const float *temperature, float temperature_scalar, int32_t greedy, int32_t *accepted_len,
                         int32_t *out_tokens, float *ratio_out, void *workspace, size_t workspace_bytes, void *stream,
                         bool apply_validate)
{
    if (batch < 0 || vocab <= 0 || total_rows < batch || (int64_t)total_rows > (int64_t)batch * SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "bad batch/total_rows/vocab (%d, %d, %d)", batch, total_rows, vocab);
    if (batch == 0) return SS_OK;
    if (max_q_len < 0 || max_q_len > SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "max_q_len must be 0 (unknown) or in [1, %d]", SS_OUT_WIDTH);
    if (row_stride < vocab) return fail(SS_ERR_INVALID_ARG, "row_stride (%lld) < vocab (%d)", (long long)row_stride, vocab);
    if (logit_dtype != SS_F32 && logit_dtype != SS_BF16)
        return fail(SS_ERR_INVALID_ARG, "logit_dtype must be SS_F32 or SS_BF16");
    const int64_t esz = logit_dtype == SS_F32 ? 4 : 2;
    const int n_draft = total_rows - batch;
    if (!q_indptr || !target_logits || !accepted_len || !out_tokens)
        return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if (n_draft > 0 && (!draft_tokens || (!greedy && (!draft_logits || !u_accept))))
        return fail(SS_ERR_INVALID_ARG, "draft-side arrays must be given when any request has drafts");
    if (!greedy && !u_sample) return fail(SS_ERR_INVALID_ARG, "u_sample is required unless greedy");
    if (!greedy && !temperature && !(temperature_scalar > 0.0f))
        return fail(SS_ERR_INVALID_ARG, "temperature must be positive unless greedy");
    if (!aligned16(target_logits) || (draft_logits && !aligned16(draft_logits)) || (row_stride * esz) % 16)
        return fail(SS_ERR_INVALID_ARG, "logits rows must start 16-byte aligned (base and row_stride)");
    const size_t need = accept_workspace_bytes(batch, total_rows, vocab);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(SS_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device buffer");
    if (workspace_bytes < need)
        return fail(SS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    if (apply_validate && g_validate) {
        int32_t rc = validate_batch(nullptr, nullptr, q_indptr, nullptr, batch, 0, 0, total_rows, max_q_len, static_cast<hipStream_t>(stream),
                                    "ss_spec_accept");
        if (rc == SS_OK)
            rc = validate_accept(draft_tokens, u_accept, u_sample, temperature, batch, n_draft, vocab, greedy ? 1 : 0,
                                 static_cast<hipStream_t>(stream), "ss_spec_accept");
        if (rc != SS_OK) return rc;
    }
    AcceptArgs a{};
    a.batch = batch; a.vocab = vocab; a.logit_dtype = logit_dtype; a.total_rows = total_rows; a.greedy = greedy ? 1 : 0;
    a.row_stride = row_stride; a.q_indptr = q_indptr; a.target = target_logits; a.draft = draft_logits;
    a.draft_tokens = draft_tokens; a.u_accept = u_accept; a.u_sample = u_sample; a.temperature = temperature;
    a.temperature_scalar = temperature_scalar; a.accepted_len = accepted_len; a.out_tokens = out_tokens;
    a.ratio_out = ratio_out; a.workspace = workspace;
    a.max_q_len = max_q_len ? max_q_len : SS_OUT_WIDTH;
    return accept_launch(a, static_cast<hipStream_t>(stream));
}

}  // namespace ss

using namespace ss;

extern "C" {

int32_t ss_version(void) { return 100; }

const char *ss_last_error(void) { return g_err; }

int32_t ss_set_option(const char *name, int64_t value)
{
    if (!name) return fail(SS_ERR_INVALID_ARG, "option name is NULL");
    if (!strcmp(name, "attn_path")) {
        if (value < 0 || value > 2) return fail(SS_ERR_INVALID_ARG, "attn_path must be 0, 1 or 2");
        g_attn_path = value;
        return SS_OK;
    }
    if (!strcmp(name, "attn_waves")) {
        if (value < 0 || value > 65536 || value % kWavesPerWg)
            return fail(SS_ERR_INVALID_ARG, "attn_waves must be a multiple of %d in [0, 65536]", kWavesPerWg);
        g_attn_waves = value;
        return SS_OK;
    }
    if (!strcmp(name, "attn_unit_weight")) {
        if (value < 0 || value > 64) return fail(SS_ERR_INVALID_ARG, "attn_unit_weight must be in [0, 64]");
        g_unit_weight = value;
        return SS_OK;
    }
    if (!strcmp(name, "validate")) {
        if (value < 0 || value > 1) return fail(SS_ERR_INVALID_ARG, "validate must be 0 or 1");
        g_validate = value;
        return SS_OK;
    }
    return fail(SS_ERR_INVALID_ARG, "unknown option '%s'", name);
}

size_t ss_spec_verify_attn_workspace(const ss_paged_kv *kv, const ss_batch *batch, int32_t num_q_heads,
                                     int32_t total_rows)
{
    if (check_attn_shape(kv, batch, num_q_heads, total_rows) != SS_OK) return 0;
    return attn_workspace_bytes(batch->batch, batch->max_blocks_per_seq, num_q_heads, kv->num_kv_heads, kv->head_dim,
                                attn_default_waves(), batch->max_q_len ? batch->max_q_len : SS_OUT_WIDTH);
}

int32_t ss_spec_verify_attn(const ss_paged_kv *kv, const ss_batch *batch, const void *q, int32_t q_dtype,
                            int32_t num_q_heads, int32_t total_rows, float sm_scale, void *out, float *lse,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    int32_t rc = check_attn_shape(kv, batch, num_q_heads, total_rows);
    if (rc != SS_OK) return rc;
    if (batch->batch == 0 || total_rows == 0) return SS_OK;
    if (q_dtype != SS_F32 && q_dtype != SS_BF16) return fail(SS_ERR_INVALID_ARG, "q_dtype must be SS_F32 or SS_BF16");
    if (!kv->k || !kv->v || !batch->block_table || !batch->kv_len || !batch->q_indptr || !q || !out)
        return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if ((kv->dtype == SS_FP8_E4M3) != (kv->k_scale != nullptr) || (kv->k_scale == nullptr) != (kv->v_scale == nullptr))
        return fail(SS_ERR_INVALID_ARG, "k_scale/v_scale must both be given for fp8 caches and be NULL otherwise");
    if (!aligned16(kv->k) || !aligned16(kv->v) || !aligned16(q) || !aligned16(out))
        return fail(SS_ERR_INVALID_ARG, "k, v, q and out must be 16-byte aligned");
    if (!(sm_scale == sm_scale) || sm_scale <= 0.0f) return fail(SS_ERR_INVALID_ARG, "sm_scale must be positive");
    const int launch_waves = attn_default_waves();
    const int max_q_len = batch->max_q_len ? batch->max_q_len : SS_OUT_WIDTH;
    const size_t need = attn_workspace_bytes(batch->batch, batch->max_blocks_per_seq, num_q_heads, kv->num_kv_heads,
                                             kv->head_dim, launch_waves, max_q_len);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(SS_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device buffer");
    if (workspace_bytes < need)
        return fail(SS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    if (g_validate) {
        rc = validate_batch(batch->block_table, batch->kv_len, batch->q_indptr, batch->tree_mask, batch->batch, batch->max_blocks_per_seq,
                            kv->num_blocks, total_rows, batch->max_q_len, static_cast<hipStream_t>(stream),
                            "ss_spec_verify_attn");
        if (rc != SS_OK) return rc;
    }

    AttnArgs a{};
    a.k = kv->k; a.v = kv->v; a.k_scale = kv->k_scale; a.v_scale = kv->v_scale;
    a.num_kv_heads = kv->num_kv_heads; a.head_dim = kv->head_dim; a.kv_dtype = kv->dtype;
    a.batch = batch->batch; a.max_blocks = batch->max_blocks_per_seq;
    a.block_table = batch->block_table; a.kv_len = batch->kv_len; a.q_indptr = batch->q_indptr;
    a.tree_mask = batch->tree_mask;
    a.q = q; a.out = out; a.lse = lse; a.q_dtype = q_dtype; a.num_q_heads = num_q_heads; a.total_rows = total_rows;
    a.sm_scale = sm_scale;
    a.launch_waves = launch_waves;
    const int G = num_q_heads / kv->num_kv_heads;
    a.rows_pad = attn_rows_pad(max_q_len, G);
    a.max_q_len = max_q_len;
    a.q_lo = 0;
    a.q_win = max_q_len;
    a.reuse_plan = (batch->flags & SS_BATCH_REUSE_PLAN) ? 1 : 0;
    a.unit_weight = (int32_t)g_unit_weight;
    // carve the workspace
    char *w = static_cast<char *>(workspace);
    a.plan = reinterpret_cast<AttnPlan *>(w);
    w += 256;
    a.tile_prefix = reinterpret_cast<int32_t *>(w);
    w += align_up(sizeof(int32_t) * ((size_t)batch->batch + 1), 256);
    a.wave_desc = reinterpret_cast<int32_t *>(w);
    w += align_up(sizeof(int32_t) * kDescInts * (size_t)launch_waves, 256);
    a.tile_addr = reinterpret_cast<int32_t *>(w);
    w += align_up(sizeof(int32_t) * (size_t)batch->batch * batch->max_blocks_per_seq * kv->num_kv_heads, 256);
    const size_t slots = (size_t)launch_waves + (size_t)batch->batch * kv->num_kv_heads;
    a.part_ml = reinterpret_cast<float *>(w);
    w += align_up(slots * a.rows_pad * 2 * sizeof(float), 256);
    a.part_o = reinterpret_cast<float *>(w);

    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (g_prof_used < g_prof_cap) {
        ev0 = g_events[2 * g_prof_used];
        ev1 = g_events[2 * g_prof_used + 1];
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mfma_ok = attn_mfma_supported(a);
    if (g_attn_path == 2 && !mfma_ok)
        return fail(SS_ERR_UNSUPPORTED, "attn_path=2 but the MFMA kernel does not cover this shape/dtype");
    if (mfma_ok && g_attn_path != 1)
        rc = attn_mfma_launch(a, s, ev0, ev1);
    else
        rc = attn_generic_launch(a, s, ev0, ev1);
    if (rc == SS_OK && ev0) ++g_prof_used;
    return rc;
}

size_t ss_spec_accept_workspace(int32_t batch, int32_t total_rows, int32_t vocab)
{
    if (batch < 0 || vocab <= 0 || total_rows < batch || (int64_t)total_rows > (int64_t)batch * SS_OUT_WIDTH) {
        fail(SS_ERR_INVALID_ARG, "bad batch/total_rows/vocab (%d, %d, %d)", batch, total_rows, vocab);
        return 0;
    }
    return accept_workspace_bytes(batch, total_rows, vocab);
}

int32_t ss_spec_accept_tree_greedy(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype,
                                   int32_t total_rows, int32_t max_q_len, const int32_t *q_indptr, const int32_t *tree_parent,
                                   const void *target_logits, const int32_t *draft_tokens, int32_t *accepted_len,
                                   int32_t *out_tokens, int32_t *accepted_nodes, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    if (batch < 0 || vocab <= 0 || total_rows < batch || (int64_t)total_rows > (int64_t)batch * SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "bad batch/total_rows/vocab (%d, %d, %d)", batch, total_rows, vocab);
    if (batch == 0) return SS_OK;
    if (max_q_len < 0 || max_q_len > SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "max_q_len must be 0 (unknown) or in [1, %d]", SS_OUT_WIDTH);
    if (row_stride < vocab) return fail(SS_ERR_INVALID_ARG, "row_stride (%lld) < vocab (%d)", (long long)row_stride, vocab);
    if (logit_dtype != SS_F32 && logit_dtype != SS_BF16)
        return fail(SS_ERR_INVALID_ARG, "logit_dtype must be SS_F32 or SS_BF16");
    const int64_t esz = logit_dtype == SS_F32 ? 4 : 2;
    if (!q_indptr || !tree_parent || !target_logits || !accepted_len || !out_tokens || !accepted_nodes)
        return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if (total_rows > batch && !draft_tokens)
        return fail(SS_ERR_INVALID_ARG, "draft_tokens must be given when any request has drafts");
    if (!aligned16(target_logits) || (row_stride * esz) % 16)
        return fail(SS_ERR_INVALID_ARG, "logits rows must start 16-byte aligned (base and row_stride)");
    const size_t need = accept_workspace_bytes(batch, total_rows, vocab);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(SS_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device buffer");
    if (workspace_bytes < need)
        return fail(SS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    if (g_validate) {
        int32_t rc = validate_batch(nullptr, nullptr, q_indptr, nullptr, batch, 0, 0, total_rows, max_q_len,
                                    static_cast<hipStream_t>(stream), "ss_spec_accept_tree_greedy");
        if (rc == SS_OK)
            rc = validate_accept(draft_tokens, nullptr, nullptr, nullptr, batch, total_rows - batch, vocab, 1,
                                 static_cast<hipStream_t>(stream), "ss_spec_accept_tree_greedy");
        if (rc != SS_OK) return rc;
    }
    AcceptArgs a{};
    a.batch = batch; a.vocab = vocab; a.logit_dtype = logit_dtype; a.total_rows = total_rows; a.greedy = 1;
    a.row_stride = row_stride; a.q_indptr = q_indptr; a.target = target_logits; a.draft_tokens = draft_tokens;
    a.accepted_len = accepted_len; a.out_tokens = out_tokens; a.workspace = workspace;
    a.tree_parent = tree_parent; a.accepted_nodes = accepted_nodes;
    a.max_q_len = max_q_len ? max_q_len : SS_OUT_WIDTH;
    return accept_launch(a, static_cast<hipStream_t>(stream));
}

size_t ss_spec_accept_tree_sample_workspace(int32_t batch, int32_t total_rows, int32_t vocab)
{
    if (batch < 0 || vocab <= 0 || total_rows < batch || (int64_t)total_rows > (int64_t)batch * SS_OUT_WIDTH) {
        fail(SS_ERR_INVALID_ARG, "bad batch/total_rows/vocab (%d, %d, %d)", batch, total_rows, vocab);
        return 0;
    }
    return accept_tree_workspace_bytes(batch, total_rows, vocab);
}

int32_t ss_spec_accept_tree_sample(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype,
                                   int32_t total_rows, int32_t max_q_len, const int32_t *q_indptr,
                                   const int32_t *tree_parent, const void *target_logits, const void *draft_logits,
                                   const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                                   const float *temperature, float temperature_scalar, int32_t *accepted_len,
                                   int32_t *out_tokens, int32_t *accepted_nodes, float *ratio_out, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    if (batch < 0 || vocab <= 0 || total_rows < batch || (int64_t)total_rows > (int64_t)batch * SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "bad batch/total_rows/vocab (%d, %d, %d)", batch, total_rows, vocab);
    if (batch == 0) return SS_OK;
    if (max_q_len < 0 || max_q_len > SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "max_q_len must be 0 (unknown) or in [1, %d]", SS_OUT_WIDTH);
    if (row_stride < vocab) return fail(SS_ERR_INVALID_ARG, "row_stride (%lld) < vocab (%d)", (long long)row_stride, vocab);
    if (logit_dtype != SS_F32 && logit_dtype != SS_BF16)
        return fail(SS_ERR_INVALID_ARG, "logit_dtype must be SS_F32 or SS_BF16");
    const int64_t esz = logit_dtype == SS_F32 ? 4 : 2;
    const int n_draft = total_rows - batch;
    if (!q_indptr || !tree_parent || !target_logits || !accepted_len || !out_tokens || !accepted_nodes || !u_sample)
        return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if (n_draft > 0 && (!draft_tokens || !draft_logits || !u_accept))
        return fail(SS_ERR_INVALID_ARG, "draft-side arrays must be given when any request has drafts");
    if (!temperature && !(temperature_scalar > 0.0f)) return fail(SS_ERR_INVALID_ARG, "temperature must be positive");
    if (!aligned16(target_logits) || (draft_logits && !aligned16(draft_logits)) || (row_stride * esz) % 16)
        return fail(SS_ERR_INVALID_ARG, "logits rows must start 16-byte aligned (base and row_stride)");
    const size_t need = accept_tree_workspace_bytes(batch, total_rows, vocab);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(SS_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device buffer");
    if (workspace_bytes < need)
        return fail(SS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    if (g_validate) {
        int32_t rc = validate_batch(nullptr, nullptr, q_indptr, nullptr, batch, 0, 0, total_rows, max_q_len,
                                    static_cast<hipStream_t>(stream), "ss_spec_accept_tree_sample");
        if (rc == SS_OK)
            rc = validate_accept(draft_tokens, u_accept, u_sample, temperature, batch, n_draft, vocab, 0,
                                 static_cast<hipStream_t>(stream), "ss_spec_accept_tree_sample");
        if (rc != SS_OK) return rc;
    }
    AcceptArgs a{};
    a.batch = batch; a.vocab = vocab; a.logit_dtype = logit_dtype; a.total_rows = total_rows; a.greedy = 0;
    a.row_stride = row_stride; a.q_indptr = q_indptr; a.target = target_logits; a.draft = draft_logits;
    a.draft_tokens = draft_tokens; a.u_accept = u_accept; a.u_sample = u_sample; a.temperature = temperature;
    a.temperature_scalar = temperature_scalar; a.accepted_len = accepted_len; a.out_tokens = out_tokens;
    a.ratio_out = ratio_out; a.workspace = workspace;
    a.tree_parent = tree_parent; a.accepted_nodes = accepted_nodes;
    a.max_q_len = max_q_len ? max_q_len : SS_OUT_WIDTH;
    return accept_tree_sample_launch(a, static_cast<hipStream_t>(stream));
}

int32_t ss_spec_accept(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype, int32_t total_rows,
                       int32_t max_q_len, const int32_t *q_indptr, const void *target_logits, const void *draft_logits,
                       const int32_t *draft_tokens, const float *u_accept, const float *u_sample,
                       const float *temperature, float temperature_scalar, int32_t greedy, int32_t *accepted_len,
                       int32_t *out_tokens, float *ratio_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return spec_accept_call(batch, vocab, row_stride, logit_dtype, total_rows, max_q_len, q_indptr, target_logits,
                            draft_logits, draft_tokens, u_accept, u_sample, temperature, temperature_scalar, greedy,
                            accepted_len, out_tokens, ratio_out, workspace, workspace_bytes, stream, true);
}

// Host-visible checks shared by the calls that write the cache; *empty is set for a batch of zero requests.
static int32_t check_kv_write(const ss_paged_kv *kv, const ss_batch *batch, int32_t total_rows, bool *empty)
{
    *empty = false;
    if (!kv || !batch) return fail(SS_ERR_INVALID_ARG, "kv and batch descriptors must not be NULL");
    if (kv->block_size != SS_BLOCK_SIZE)
        return fail(SS_ERR_INVALID_ARG, "block_size must be %d, got %d", SS_BLOCK_SIZE, kv->block_size);
    if (kv->head_dim != 64 && kv->head_dim != 128)
        return fail(SS_ERR_INVALID_ARG, "head_dim must be 64 or 128, got %d", kv->head_dim);
    if (kv->num_kv_heads <= 0 || kv->num_blocks < 0) return fail(SS_ERR_INVALID_ARG, "bad num_kv_heads or num_blocks");
    if (kv->dtype < SS_F32 || kv->dtype > SS_FP8_E4M3) return fail(SS_ERR_INVALID_ARG, "unknown KV dtype %d", kv->dtype);
    if (batch->batch < 0 || total_rows < batch->batch || (int64_t)total_rows > (int64_t)batch->batch * SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "total_rows (%d) must lie in [batch, %d*batch] for batch %d", total_rows,
                    SS_OUT_WIDTH, batch->batch);
    if (batch->batch == 0) {
        *empty = true;
        return SS_OK;
    }
    if (batch->max_blocks_per_seq <= 0) return fail(SS_ERR_INVALID_ARG, "max_blocks_per_seq must be positive");
    if (batch->max_q_len < 0 || batch->max_q_len > SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "max_q_len must be 0 (unknown) or in [1, %d]", SS_OUT_WIDTH);
    if ((int64_t)batch->batch * SS_OUT_WIDTH * kv->num_kv_heads > 0x7fffffffll)
        return fail(SS_ERR_UNSUPPORTED, "batch * kv heads too large for one launch");
    if (!kv->k || !kv->v || !batch->block_table || !batch->kv_len || !batch->q_indptr)
        return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if ((kv->dtype == SS_FP8_E4M3) != (kv->k_scale != nullptr) || (kv->k_scale != nullptr) != (kv->v_scale != nullptr))
        return fail(SS_ERR_INVALID_ARG, "k_scale/v_scale must both be given for fp8 caches and be NULL otherwise");
    return SS_OK;
}

static KvAppendArgs kv_write_args(const ss_paged_kv *kv, const ss_batch *batch)
{
    KvAppendArgs a{};
    a.k = const_cast<void *>(kv->k); a.v = const_cast<void *>(kv->v);
    a.k_scale = const_cast<float *>(kv->k_scale); a.v_scale = const_cast<float *>(kv->v_scale);
    a.num_kv_heads = kv->num_kv_heads; a.head_dim = kv->head_dim; a.kv_dtype = kv->dtype;
    a.batch = batch->batch; a.max_blocks = batch->max_blocks_per_seq;
    a.block_table = batch->block_table; a.kv_len = batch->kv_len; a.q_indptr = batch->q_indptr;
    a.max_q_len = batch->max_q_len ? batch->max_q_len : SS_OUT_WIDTH;
    return a;
}

int32_t ss_kv_append(const ss_paged_kv *kv, const ss_batch *batch, const void *k_new, const void *v_new,
                     int32_t new_dtype, int32_t total_rows, void *stream)
{
    bool empty;
    const int32_t rc0 = check_kv_write(kv, batch, total_rows, &empty);
    if (rc0 != SS_OK || empty) return rc0;
    if (new_dtype != SS_F32 && new_dtype != SS_BF16) return fail(SS_ERR_INVALID_ARG, "new_dtype must be SS_F32 or SS_BF16");
    if (!k_new || !v_new) return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if (g_validate) {
        const int32_t rc = validate_batch(batch->block_table, batch->kv_len, batch->q_indptr, nullptr, batch->batch,
                                          batch->max_blocks_per_seq, kv->num_blocks, total_rows, batch->max_q_len,
                                          static_cast<hipStream_t>(stream), "ss_kv_append");
        if (rc != SS_OK) return rc;
    }
    KvAppendArgs a = kv_write_args(kv, batch);
    a.k_new = k_new; a.v_new = v_new; a.new_dtype = new_dtype;
    return kv_append_launch(a, static_cast<hipStream_t>(stream));
}

int32_t ss_kv_compact(const ss_paged_kv *kv, const ss_batch *batch, const int32_t *accepted_nodes,
                      const int32_t *accepted_len, int32_t total_rows, void *stream)
{
    bool empty;
    const int32_t rc0 = check_kv_write(kv, batch, total_rows, &empty);
    if (rc0 != SS_OK || empty) return rc0;
    if (!accepted_nodes || !accepted_len) return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    if (g_validate) {
        const int32_t rc = validate_batch(batch->block_table, batch->kv_len, batch->q_indptr, nullptr, batch->batch,
                                          batch->max_blocks_per_seq, kv->num_blocks, total_rows, batch->max_q_len,
                                          static_cast<hipStream_t>(stream), "ss_kv_compact");
        if (rc != SS_OK) return rc;
    }
    return kv_compact_launch(kv_write_args(kv, batch), accepted_nodes, accepted_len, static_cast<hipStream_t>(stream));
}

int32_t ss_kv_commit(int32_t batch, const int32_t *q_indptr, const int32_t *accepted_len, int32_t *kv_len, void *stream)
{
    if (batch < 0) return fail(SS_ERR_INVALID_ARG, "negative batch");
    if (batch == 0) return SS_OK;
    if (!q_indptr || !accepted_len || !kv_len) return fail(SS_ERR_INVALID_ARG, "a required device pointer is NULL");
    return kv_commit_launch(batch, q_indptr, accepted_len, kv_len, static_cast<hipStream_t>(stream));
}

int32_t ss_profile_begin(int32_t max_calls)
{
    if (max_calls < 0 || max_calls > 100000) return fail(SS_ERR_INVALID_ARG, "max_calls out of range");
    for (hipEvent_t e : g_events) (void)hipEventDestroy(e);
    g_events.clear();
    g_prof_cap = g_prof_used = 0;
    for (int i = 0; i < 2 * max_calls; ++i) {
        hipEvent_t e;
        SS_HIP_CHECK(hipEventCreate(&e), "hipEventCreate");
        g_events.push_back(e);
    }
    g_prof_cap = max_calls;
    return SS_OK;
}

int32_t ss_profile_collect(float *ms, int32_t cap)
{
    int n = 0;
    for (int i = 0; i < g_prof_used; ++i) {
        float t = 0.f;
        if (hipEventSynchronize(g_events[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&t, g_events[2 * i], g_events[2 * i + 1]) != hipSuccess) {
            (void)hipGetLastError();
            break;
        }
        if (ms && n < cap) ms[n++] = t;
    }
    for (hipEvent_t e : g_events) (void)hipEventDestroy(e);
    g_events.clear();
    g_prof_cap = g_prof_used = 0;
    return n;
}

}  // extern "C"
