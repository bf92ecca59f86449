// Compiled instances: the MFMA kernel with run-time factor shapes, fp64.
#include "launch_any.hpp"

namespace km {
template hipError_t launch_mfma_any<double>(const LaunchArgs&);
}  // namespace km
