// Optional checks of device-resident metadata (option "validate").  The entry points normally trust
// what the caller's device arrays hold (block ids in range, lengths consistent): checking them costs a
// kernel and a stream synchronisation.  With the option on, a single workgroup walks the metadata first,
// reading nothing beyond the sizes the arguments declare, and reports the first inconsistency through a
// small pinned host record, so that a bad batch becomes an error code instead of a wild read.
#include "common.h"

namespace ss {
namespace {

struct CheckRecord {
    int32_t code;    // 0 = consistent
    int32_t where;   // request (or row) index
    int32_t value;   // offending value
    int32_t aux;
};

enum { CK_QLEN = 1, CK_QSTART, CK_QTOTAL, CK_KVLEN, CK_BLOCKS, CK_BLOCK_ID, CK_TOKEN, CK_TEMP, CK_UNIFORM, CK_TREE };

__global__ __launch_bounds__(256) void validate_batch_kernel(const int32_t *block_table, const int32_t *kv_len,
                                                             const int32_t *q_indptr, const uint32_t *tree_mask, int batch,
                                                             int max_blocks, int num_blocks, int total_rows, int max_q_len,
                                                             CheckRecord *out)
{
    __shared__ int bad_req;     // lowest request index with a problem
    const int tid = threadIdx.x;
    if (tid == 0) bad_req = 0x7fffffff;
    __syncthreads();
    // pass 1: find the first bad request (any kind of problem)
    for (int b = 0; b < batch; ++b) {
        const int q0 = q_indptr[b], q1 = q_indptr[b + 1], q_len = q1 - q0;
        bool bad = q_len < 1 || q_len > max_q_len || (b == 0 && q0 != 0) || (b == batch - 1 && q1 != total_rows);
        if (block_table) {
            const int L = kv_len[b];
            const long long nblk = ((long long)L + kTile - 1) / kTile;
            bad = bad || L < q_len || L < 1 || nblk > max_blocks;
            const int n = (int)(nblk < max_blocks ? (nblk > 0 ? nblk : 0) : max_blocks);
            for (int t = tid; t < n; t += 256) {
                const int id = block_table[(long long)b * max_blocks + t];
                if (id < 0 || id >= num_blocks) bad = true;
            }
        }
        // a tree row attends itself and only new tokens of its own request
        if (tree_mask && q_len >= 1 && q_len <= max_q_len && q0 >= 0 && q1 <= total_rows && tid < q_len) {
            const uint32_t w = tree_mask[q0 + tid];
            if (!((w >> tid) & 1u) || (w >> q_len)) bad = true;
        }
        if (bad) atomicMin(&bad_req, b);
        __syncthreads();
        if (bad_req != 0x7fffffff) break;   // uniform: read after the barrier
    }
    __syncthreads();
    if (tid != 0) return;
    CheckRecord r = {0, 0, 0, 0};
    if (bad_req != 0x7fffffff) {   // pass 2 (one lane): name the problem of that request
        const int b = bad_req;
        const int q0 = q_indptr[b], q1 = q_indptr[b + 1], q_len = q1 - q0;
        r.where = b;
        if (b == 0 && q0 != 0) { r.code = CK_QSTART; r.value = q0; }
        else if (q_len < 1 || q_len > max_q_len) { r.code = CK_QLEN; r.value = q_len; r.aux = max_q_len; }
        else if (b == batch - 1 && q1 != total_rows) { r.code = CK_QTOTAL; r.value = q1; }
        else if (block_table) {
            const int L = kv_len[b];
            const long long nblk = ((long long)L + kTile - 1) / kTile;
            if (L < q_len || L < 1) { r.code = CK_KVLEN; r.value = L; r.aux = q_len; }
            else if (nblk > max_blocks) { r.code = CK_BLOCKS; r.value = L; r.aux = max_blocks; }
            else {
                for (int t = 0; t < (int)nblk; ++t) {
                    const int id = block_table[(long long)b * max_blocks + t];
                    if (id < 0 || id >= num_blocks) { r.code = CK_BLOCK_ID; r.value = id; r.aux = t; break; }
                }
            }
        }
        if (r.code == 0 && tree_mask) {
            for (int i = 0; i < q_len; ++i) {
                const uint32_t w = tree_mask[q0 + i];
                if (!((w >> i) & 1u) || (w >> q_len)) { r.code = CK_TREE; r.value = i; r.aux = (int32_t)w; break; }
            }
        }
    }
    *out = r;
    __threadfence_system();
}

__global__ __launch_bounds__(256) void validate_accept_kernel(const int32_t *draft_tokens, const float *u_accept,
                                                              const float *u_sample, const float *temperature, int batch,
                                                              int n_draft, int vocab, int greedy, CheckRecord *out)
{
    const int tid = threadIdx.x;
    // lowest offending index per kind; kinds are reported in a fixed order of precedence
    int tok_bad = 0x7fffffff, u_bad = 0x7fffffff, t_bad = 0x7fffffff;
    for (int i = tid; i < n_draft; i += 256) {
        if (draft_tokens && (draft_tokens[i] < 0 || draft_tokens[i] >= vocab)) tok_bad = min(tok_bad, i);
        if (!greedy && u_accept && !(u_accept[i] >= 0.f && u_accept[i] < 1.f)) u_bad = min(u_bad, i);
    }
    for (int b = tid; b < batch; b += 256) {
        if (!greedy && u_sample && !(u_sample[b] >= 0.f && u_sample[b] < 1.f)) u_bad = min(u_bad, n_draft + b);
        if (!greedy && temperature && !(temperature[b] > 0.f)) t_bad = min(t_bad, b);
    }
    __shared__ int s_tok, s_u, s_t;
    if (tid == 0) { s_tok = s_u = s_t = 0x7fffffff; }
    __syncthreads();
    atomicMin(&s_tok, tok_bad);
    atomicMin(&s_u, u_bad);
    atomicMin(&s_t, t_bad);
    __syncthreads();
    if (tid != 0) return;
    CheckRecord r = {0, 0, 0, 0};
    if (s_tok != 0x7fffffff) { r.code = CK_TOKEN; r.where = s_tok; r.value = draft_tokens[s_tok]; }
    else if (s_t != 0x7fffffff) { r.code = CK_TEMP; r.where = s_t; }
    else if (s_u != 0x7fffffff) { r.code = CK_UNIFORM; r.where = s_u; }
    *out = r;
    __threadfence_system();
}

CheckRecord *g_record = nullptr;   // pinned host memory, mapped into the device's address space

int32_t record(CheckRecord **host, CheckRecord **dev)
{
    if (!g_record) SS_HIP_CHECK(hipHostMalloc(reinterpret_cast<void **>(&g_record), sizeof(CheckRecord), hipHostMallocMapped),
                                "hipHostMalloc (validation record)");
    *host = g_record;
    SS_HIP_CHECK(hipHostGetDevicePointer(reinterpret_cast<void **>(dev), g_record, 0), "hipHostGetDevicePointer");
    return SS_OK;
}

int32_t report(const CheckRecord &r, const char *what)
{
    switch (r.code) {
    case 0: return SS_OK;
    case CK_QLEN: return fail(SS_ERR_INVALID_ARG, "%s: request %d has %d query rows (must be 1..%d)", what, r.where, r.value, r.aux);
    case CK_QSTART: return fail(SS_ERR_INVALID_ARG, "%s: q_indptr[0] is %d, not 0", what, r.value);
    case CK_QTOTAL: return fail(SS_ERR_INVALID_ARG, "%s: q_indptr[batch] is %d, not total_rows", what, r.value);
    case CK_KVLEN: return fail(SS_ERR_INVALID_ARG, "%s: request %d has kv_len %d but %d query rows", what, r.where, r.value, r.aux);
    case CK_BLOCKS: return fail(SS_ERR_INVALID_ARG, "%s: request %d with kv_len %d needs more than max_blocks_per_seq = %d blocks", what, r.where, r.value, r.aux);
    case CK_BLOCK_ID: return fail(SS_ERR_INVALID_ARG, "%s: request %d, logical block %d maps to physical block %d (out of range)", what, r.where, r.aux, r.value);
    case CK_TOKEN: return fail(SS_ERR_INVALID_ARG, "%s: draft token %d at draft row %d is outside the vocabulary", what, r.value, r.where);
    case CK_TEMP: return fail(SS_ERR_INVALID_ARG, "%s: request %d has a non-positive temperature", what, r.where);
    case CK_TREE: return fail(SS_ERR_INVALID_ARG, "%s: request %d, row %d has tree mask 0x%x (own bit missing or a bit past its query rows)", what, r.where, r.value, (unsigned)r.aux);
    default: return fail(SS_ERR_INVALID_ARG, "%s: uniform %d is outside [0, 1)", what, r.where);
    }
}

}  // namespace

int32_t validate_batch(const int32_t *block_table, const int32_t *kv_len, const int32_t *q_indptr,
                       const uint32_t *tree_mask, int batch, int max_blocks, int num_blocks, int total_rows, int max_q_len, hipStream_t stream, const char *what)
{
    CheckRecord *host = nullptr, *dev = nullptr;
    const int32_t rc = record(&host, &dev);
    if (rc != SS_OK) return rc;
    hipLaunchKernelGGL(validate_batch_kernel, dim3(1), dim3(256), 0, stream, block_table, kv_len, q_indptr, tree_mask, batch, max_blocks,
                       num_blocks, total_rows, max_q_len > 0 ? max_q_len : SS_OUT_WIDTH, dev);
    SS_HIP_CHECK(hipGetLastError(), "launch validate_batch_kernel");
    SS_HIP_CHECK(hipStreamSynchronize(stream), "hipStreamSynchronize (validation)");
    return report(*host, what);
}

int32_t validate_accept(const int32_t *draft_tokens, const float *u_accept, const float *u_sample, const float *temperature,
                        int batch, int n_draft, int vocab, int greedy, hipStream_t stream, const char *what)
{
    CheckRecord *host = nullptr, *dev = nullptr;
    const int32_t rc = record(&host, &dev);
    if (rc != SS_OK) return rc;
    hipLaunchKernelGGL(validate_accept_kernel, dim3(1), dim3(256), 0, stream, draft_tokens, u_accept, u_sample, temperature,
                       batch, n_draft, vocab, greedy, dev);
    SS_HIP_CHECK(hipGetLastError(), "launch validate_accept_kernel");
    SS_HIP_CHECK(hipStreamSynchronize(stream), "hipStreamSynchronize (validation)");
    return report(*host, what);
}

}  // namespace ss
