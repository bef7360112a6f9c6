// placeholder until the MFMA router lands
#include "common.h"
namespace moepp {
bool router_mfma_supported(const Dims &) { return false; }
hipError_t launch_router_mfma(const RouterArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace moepp
