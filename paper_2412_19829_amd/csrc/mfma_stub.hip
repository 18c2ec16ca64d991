#include "common.hpp"
namespace gformer {
hipError_t launch_windowed_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_linear_state_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_linear_main_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
}
