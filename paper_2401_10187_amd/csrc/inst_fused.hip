// Compiled instances: the dedicated small-factor kernel (fp32 and fp64) and the lane-exchange kernel.
#include "launch_fused.hpp"
#include "instances.hpp"

namespace km {
#define KM_X(T, DT, P, Q, NF, ST, NT) template hipError_t launch_fused<T, P, Q, NF, ST, NT>(const LaunchArgs&);
#define KM_NONE(...)
KM_INSTANCES(KM_X, KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_NONE)
hipError_t launch_shuffle(const LaunchArgs& a) { return launch_shuffle_impl(a); }
}  // namespace km
