#include "d2ft_common.h"
namespace d2ft {
bool gemm_mfma_supported(const GemmArgs&) { return false; }
hipError_t launch_gemm_mfma(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace d2ft
