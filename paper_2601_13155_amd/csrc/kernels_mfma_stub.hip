#include "spts_internal.h"
namespace spts {
bool gemm_mfma_supported(const GemmArgs&) { return false; }
hipError_t launch_gemm_mfma(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
bool attention_mfma_supported(const AttnArgs&) { return false; }
hipError_t launch_attention_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
bool probe_mfma_supported(const ProbeArgs&) { return false; }
hipError_t launch_probe_mfma(const ProbeArgs&, hipStream_t) { return hipErrorNotSupported; }
}
