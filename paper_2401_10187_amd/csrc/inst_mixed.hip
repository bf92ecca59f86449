// Compiled instances: several small factors per LDS pass with a factor shape per stage, fp32 and fp64.
#include "launch_multi.hpp"
#include "instances.hpp"

namespace km {
#define KM_V(T, DT, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT) \
    template hipError_t launch_multi<MixedShape<T, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, ST, NT>>(const LaunchArgs&);
#define KM_NONE(...)
KM_INSTANCES(KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_V, KM_NONE)
}  // namespace km
