// placeholder until the MFMA grouped GEMM lands
#include "common.h"
namespace moepp {
bool ffn_mfma_supported(const Dims &) { return false; }
hipError_t launch_ffn_mfma(const FfnArgs &, int, hipStream_t) { return hipErrorNotSupported; }
}  // namespace moepp
