// bf16 MFMA GEMM family (placeholder until the kernels land: reports "not supported").
#include "hr_kernels.h"
namespace hr {
bool gemm_mfma_supported(const hr_model_cfg&) { return false; }
hipError_t launch_gemm_mfma(GemmEpilogue, const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace hr
