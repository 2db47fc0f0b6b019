// Paged GQA prefix attention on MFMA (placeholder until the kernel lands: reports "not supported").
#include "hr_kernels.h"
namespace hr {
bool attn_mfma_supported(const hr_model_cfg&, int, int) { return false; }
hipError_t launch_attn_mfma(const void*, const void*, const void*, void*, const MetaView&, const PoolView&, int, int, int,
                            hipStream_t) { return hipErrorNotSupported; }
}  // namespace hr
