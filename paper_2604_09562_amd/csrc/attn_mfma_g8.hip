// Matrix-core verify attention: the streaming and merge kernel instances for 8 query heads per KV head.
#include "attn_mfma_kernels.h"

namespace ss {

int32_t attn_mfma_launch_g8(const AttnArgs &a, hipStream_t stream, hipEvent_t ev0, hipEvent_t ev1)
{
    return launch_for_group<8>(a, stream, ev0, ev1);
}

}  // namespace ss
