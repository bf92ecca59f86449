// Compiled instances: several small factors per LDS pass, fp32, factors with P of 2 and 4.
#include "launch_multi.hpp"
#include "instances.hpp"

namespace km {
#define KM_INST(T, P, Q, G0, G1, G2, ST, NT) template hipError_t launch_multi<MultiShape<T, P, Q, G0, G1, G2, ST, NT>>(const LaunchArgs&);
#define KM_SKIP(...)
#define KM_W_F32_P2 KM_INST
#define KM_W_F32_P3 KM_SKIP
#define KM_W_F32_P4 KM_INST
#define KM_W_F32_P5 KM_SKIP
#define KM_W_F32_P6 KM_SKIP
#define KM_W_F32_P7 KM_SKIP
#define KM_W_F32_P8 KM_SKIP
#define KM_W_F32_P9 KM_SKIP
#define KM_W_F32_P10 KM_SKIP
#define KM_W_F32_P12 KM_SKIP
#define KM_W_F32_P11 KM_SKIP
#define KM_W_F32_P13 KM_SKIP
#define KM_W_F32_P14 KM_SKIP
#define KM_W_F32_P15 KM_SKIP
#define KM_W_KM_F32(T, P, Q, G0, G1, G2, ST, NT) KM_W_F32_P##P(T, P, Q, G0, G1, G2, ST, NT)
#define KM_W_KM_F64(...)
#define KM_W(T, DT, P, Q, G0, G1, G2, ST, NT) KM_W_##DT(T, P, Q, G0, G1, G2, ST, NT)
#define KM_NONE(...)
KM_INSTANCES(KM_NONE, KM_NONE, KM_NONE, KM_W, KM_NONE, KM_NONE, KM_NONE)
}  // namespace km
