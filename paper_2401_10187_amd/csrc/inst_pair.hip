// Compiled instances: register-chained MFMA pairs (fp32).
#include "launch_pair.hpp"
#include "instances.hpp"

namespace km {
#define KM_Z(P, ST, NW, PD, NPASS) template hipError_t launch_mfma_pair<P, ST, NW, PD, NPASS>(const LaunchArgs&);
#define KM_R(P, ST, NW) template hipError_t launch_mfma_pair_rows<P, ST, NW>(const LaunchArgs&);
#define KM_NONE(...)
KM_INSTANCES(KM_NONE, KM_NONE, KM_Z, KM_NONE, KM_R, KM_NONE, KM_NONE)
}  // namespace km
