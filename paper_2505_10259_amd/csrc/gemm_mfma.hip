// bf16 MFMA GEMM kernels (placeholder: routed to the plain kernel until the MFMA path lands).
#include "common.h"
namespace sv {
hipError_t launch_gemm_mfma_bf16(const GemmArgs& a, hipStream_t st) { return launch_gemm_simple(a, SPEC_BF16, st); }
}  // namespace sv
