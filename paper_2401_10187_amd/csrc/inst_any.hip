// Compiled instances: the MFMA kernel with run-time factor shapes (fp32 and fp64).
#include "launch_any.hpp"

namespace km {
template hipError_t launch_mfma_any<float>(const LaunchArgs&);
template hipError_t launch_mfma_any<double>(const LaunchArgs&);
}  // namespace km
