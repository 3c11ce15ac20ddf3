#include "kernels.hpp"
namespace qasr {
bool gemm_mfma_supported(const ConvParams&) { return false; }
hipError_t launch_gemm_mfma(const ConvParams&, hipStream_t) { return hipErrorNotSupported; }
}
