// Compiled instances: small factors in four super-stages (whole short rows in one launch), fp64.
#include "launch_multi.hpp"
#include "instances.hpp"

namespace km {
#define KM_U_KM_F64(T, P, Q, G0, G1, G2, G3, ST, NT) template hipError_t launch_multi<MultiShape<T, P, Q, G0, G1, G2, ST, NT, G3>>(const LaunchArgs&);
#define KM_U_KM_F32(...)
#define KM_U(T, DT, P, Q, G0, G1, G2, G3, ST, NT) KM_U_##DT(T, P, Q, G0, G1, G2, G3, ST, NT)
#define KM_NONE(...)
KM_INSTANCES(KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_U)
}  // namespace km
