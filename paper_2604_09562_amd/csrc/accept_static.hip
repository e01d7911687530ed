// ss_spec_accept_static: ss_spec_accept for callers that cannot allocate device memory.
//
// The acceptance kernels keep their partial results (chunk statistics, block sums, the list of
// boundary entries, per-request counters) in a workspace the caller of ss_spec_accept brings.  Here
// that workspace is a fixed array in the library's own device image, so the call needs nothing but its
// inputs and outputs and performs no allocation of any kind.  Every GPU the library's code object is
// loaded on holds its own copy of the array at its own address, until the process ends.
#include <mutex>

#include "common.h"

namespace ss {
namespace {

// Partial results of one acceptance call.  In host code the name is only a handle for
// hipGetSymbolAddress: the device address it yields, per device, is what kernels and copies receive.
static __device__ __align__(256) unsigned char scratch[SS_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once looked up

// Address of the current device's copy of the array (looked up once per device, with that device current).
int32_t scratch_of_current_device(void **out)
{
    int dev = -1;
    SS_HIP_CHECK(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(SS_ERR_UNSUPPORTED, "device ordinal %d is beyond the %d supported", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        SS_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress (static scratch)");
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return fail(SS_ERR_DEVICE, "static scratch has no usable device address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SS_OK;
}

}  // namespace
}  // namespace ss

using namespace ss;

extern "C" {

size_t ss_spec_accept_static_capacity(void) { return SS_STATIC_SCRATCH_BYTES; }

int32_t ss_spec_accept_static(int32_t batch, int32_t vocab, int64_t row_stride, int32_t logit_dtype, int32_t total_rows,
                              int32_t max_q_len, const int32_t *q_indptr, const void *target_logits,
                              const void *draft_logits, const int32_t *draft_tokens, const float *u_accept,
                              const float *u_sample, const float *temperature, float temperature_scalar, int32_t greedy,
                              int32_t *accepted_len, int32_t *out_tokens, float *ratio_out, void *stream)
{
    if (batch < 0 || vocab <= 0 || total_rows < batch || (int64_t)total_rows > (int64_t)batch * SS_OUT_WIDTH)
        return fail(SS_ERR_INVALID_ARG, "bad batch/total_rows/vocab (%d, %d, %d)", batch, total_rows, vocab);
    if (batch == 0) return SS_OK;
    const size_t need = accept_workspace_bytes(batch, total_rows, vocab);
    if (need > (size_t)SS_STATIC_SCRATCH_BYTES)
        return fail(SS_ERR_WORKSPACE,
                    "ss_spec_accept_static: batch %d, %d rows, vocabulary %d need %zu bytes of scratch, the static buffer "
                    "holds %zu; use ss_spec_accept with a workspace of the caller's", batch, total_rows, vocab, need,
                    (size_t)SS_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    const int32_t rc = scratch_of_current_device(&ws);
    if (rc != SS_OK) return rc;
    // The kernels initialise every counter and slot they read (nothing has to start at zero), so the
    // contents the previous call left behind are harmless.
    return spec_accept_call(batch, vocab, row_stride, logit_dtype, total_rows, max_q_len, q_indptr, target_logits,
                            draft_logits, draft_tokens, u_accept, u_sample, temperature, temperature_scalar, greedy,
                            accepted_len, out_tokens, ratio_out, ws, (size_t)SS_STATIC_SCRATCH_BYTES, stream, false);
}

}  // extern "C"
