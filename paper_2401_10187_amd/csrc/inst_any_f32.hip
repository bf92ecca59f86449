// Compiled instances: the MFMA kernel with run-time factor shapes, fp32.
#include "launch_any.hpp"

namespace km {
template hipError_t launch_mfma_any<float>(const LaunchArgs&);
}  // namespace km
