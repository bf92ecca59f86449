// Compiled instances: LDS-staged MFMA kernels, fp64.
#include "launch_mfma.hpp"
#include "instances.hpp"

namespace km {
#define KM_Y_KM_F64(OP, P, Q, NF, ST, NW, QS) template hipError_t launch_mfma<OP, P, Q, NF, ST, NW, QS>(const LaunchArgs&);
#define KM_Y_KM_F32(...)
#define KM_Y(OP, DT, P, Q, NF, ST, NW, QS) KM_Y_##DT(OP, P, Q, NF, ST, NW, QS)
#define KM_NONE(...)
KM_INSTANCES(KM_NONE, KM_Y, KM_NONE, KM_NONE, KM_NONE, KM_NONE, KM_NONE)
}  // namespace km
