// MFMA tree attention (bf16, head_dim 128) -- placeholder until the kernel lands.
#include "cb_internal.h"
namespace cb {
hipError_t launch_attn_mfma(hipStream_t, const AttnParams&, const SeqMeta&, int, int) { return hipErrorNotSupported; }
}  // namespace cb
