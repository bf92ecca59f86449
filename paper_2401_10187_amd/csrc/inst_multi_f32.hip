// Compiled instances: several small factors per LDS pass, fp32.
#include "launch_multi.hpp"
#include "instances.hpp"

namespace km {
#define KM_W_KM_F32(T, P, Q, G0, G1, G2, ST, NT) template hipError_t launch_multi<MultiShape<T, P, Q, G0, G1, G2, ST, NT>>(const LaunchArgs&);
#define KM_W_KM_F64(...)
#define KM_W(T, DT, P, Q, G0, G1, G2, ST, NT) KM_W_##DT(T, P, Q, G0, G1, G2, ST, NT)
#define KM_NONE(...)
KM_INSTANCES(KM_NONE, KM_NONE, KM_NONE, KM_W, KM_NONE, KM_NONE)
}  // namespace km
