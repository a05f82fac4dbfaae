// bf16 MFMA paged attention (placeholder: routed to the plain kernel until the MFMA path lands).
#include "common.h"
namespace sv {
hipError_t launch_attention_mfma_bf16(const AttnArgs& a, hipStream_t st) { return launch_attention_simple(a, SPEC_BF16, st); }
}  // namespace sv
