// The compiled kernel instances, in the planner's order of preference among instances that fit a
// shape.  Each translation unit of the library expands the list with the macros of its own family.
#pragma once

// Fused FMA instances: X(type, dtype code, P, Q, factors per launch, tile_slices, threads).
// Register-resident MFMA pairs: Z(P, tile_slices, wavefronts, units fetched ahead, output passes) (fp32, Q = 32, two factors).
// Small-factor instances with several factors per LDS pass and a run-time tile length:
// W(type, dtype code, P, Q, G0, G1, G2, largest tile_slices, threads).
// The same with a fourth super-stage (whole rows of P^4 elements in one launch):
// U(type, dtype code, P, Q, G0, G1, G2, G3, largest tile_slices, threads).
// The same for rows of exactly P*P elements, ST rows per tile: R(P, rows per tile, wavefronts).
// MFMA instances: Y(op, dtype code, P, Q, factors per launch, tile_slices, wavefronts, q split).
// The same with a factor shape per stage, for neighbouring runs of different small shapes, stages in
// order of application (the group's last factors first):
// V(type, dtype code, P0, Q0, G0, P1, Q1, G1, P2, Q2, G2, largest tile_slices, threads); the comment
// behind a row gives the factors in the order of the Kronecker product.  A curated list (neighbouring
// runs of 2x2, 4x4 and 8x8, 5x5 beside 2x2, 3x3 beside 2x2): a further combination is one more row.
// Order = preference among instances that fit a shape.
#define KM_INSTANCES(X, Y, Z, W, R, V, U)                    \
    X(float, KM_F32, 8, 8, 3, 32, 1024)                 \
    X(float, KM_F32, 8, 8, 3, 32, 256)                  \
    X(float, KM_F32, 8, 8, 3, 16, 256)                  \
    X(float, KM_F32, 8, 8, 3, 8, 128)                   \
    X(float, KM_F32, 8, 8, 3, 1, 64)                    \
    X(float, KM_F32, 8, 8, 2, 256, 256)                 \
    X(float, KM_F32, 8, 8, 2, 64, 256)                  \
    X(float, KM_F32, 8, 8, 2, 8, 64)                    \
    X(float, KM_F32, 8, 8, 2, 1, 64)                    \
    X(float, KM_F32, 8, 8, 1, 2048, 256)                \
    X(float, KM_F32, 8, 8, 1, 64, 64)                   \
    X(float, KM_F32, 8, 8, 1, 8, 64)                    \
    X(float, KM_F32, 8, 8, 1, 1, 64)                    \
    X(float, KM_F32, 6, 6, 3, 48, 256)                  \
    X(float, KM_F32, 6, 6, 2, 288, 256)                 \
    X(double, KM_F64, 6, 6, 3, 16, 256)                 \
    R(32, 32, 4)                                        \
    Z(32, 32, 16, 1, 1)                                 \
    Z(32, 32, 4, 1, 2)                                  \
    Y(MfmaF32x32, KM_F32, 32, 32, 2, 32, 8, 1)          \
    Y(MfmaF32x32, KM_F32, 32, 32, 2, 32, 16, 1)         \
    Y(MfmaF32x32, KM_F32, 32, 32, 2, 16, 4, 1)          \
    Y(MfmaF32x32, KM_F32, 32, 32, 1, 256, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 32, 32, 1, 128, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 32, 32, 1, 32, 1, 1)          \
    R(16, 32, 4)                                        \
    Z(16, 32, 8, 1, 1)                                  \
    Z(16, 32, 4, 1, 2)                                  \
    Y(MfmaF32x32, KM_F32, 16, 32, 2, 32, 4, 1)          \
    Y(MfmaF32x32, KM_F32, 16, 32, 2, 16, 4, 1)          \
    Y(MfmaF32x32, KM_F32, 16, 32, 1, 256, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 16, 32, 1, 128, 4, 1)         \
    Y(MfmaF64x16, KM_F64, 128, 128, 1, 32, 8, 8)         \
    Y(MfmaF64x16, KM_F64, 128, 128, 1, 16, 4, 4)         \
    Y(MfmaF64x16, KM_F64, 128, 128, 1, 32, 4, 4)         \
    Y(MfmaF32x16, KM_F32, 16, 16, 2, 32, 4, 1)          \
    Y(MfmaF32x16, KM_F32, 16, 16, 1, 256, 4, 1)         \
    Y(MfmaF32x16, KM_F32, 16, 16, 1, 64, 4, 1)          \
    Y(MfmaF32x16, KM_F32, 16, 16, 1, 16, 1, 1)          \
    Y(MfmaF32x32, KM_F32, 64, 64, 1, 128, 8, 2)         \
    Y(MfmaF32x32, KM_F32, 64, 64, 1, 128, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 64, 64, 1, 64, 2, 1)          \
    Y(MfmaF32x32, KM_F32, 128, 128, 1, 32, 4, 4)        \
    Y(MfmaF32x16, KM_F32, 32, 16, 1, 256, 4, 1)         \
    Y(MfmaF32x16, KM_F32, 64, 16, 1, 128, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 64, 32, 1, 128, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 32, 64, 1, 256, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 16, 64, 1, 256, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 128, 64, 1, 64, 4, 2)         \
    Y(MfmaF32x32, KM_F32, 64, 128, 1, 128, 8, 2)        \
    Y(MfmaF32x32, KM_F32, 128, 32, 1, 64, 2, 1)         \
    Y(MfmaF32x32, KM_F32, 32, 128, 1, 256, 4, 2)        \
    Y(MfmaF32x16, KM_F32, 48, 48, 1, 128, 4, 1)         \
    Y(MfmaF32x32, KM_F32, 96, 96, 1, 64, 6, 3)          \
    Y(MfmaF32x16, KM_F32, 80, 80, 1, 128, 10, 5)        \
    Y(MfmaF32x16, KM_F32, 80, 80, 1, 64, 10, 5)         \
    Y(MfmaF32x16, KM_F32, 112, 112, 1, 64, 7, 7)        \
    Y(MfmaF32x16, KM_F32, 144, 144, 1, 64, 9, 9)        \
    Y(MfmaF32x16, KM_F32, 160, 160, 1, 64, 10, 10)      \
    Y(MfmaF32x16, KM_F32, 192, 192, 1, 64, 12, 12)      \
    Y(MfmaF32x16, KM_F32, 256, 256, 1, 64, 16, 16)      \
    Y(MfmaF64x16, KM_F64, 48, 48, 1, 64, 4, 1)          \
    Y(MfmaF64x16, KM_F64, 80, 80, 1, 64, 10, 5)         \
    Y(MfmaF64x16, KM_F64, 96, 96, 1, 64, 6, 6)          \
    Y(MfmaF64x16, KM_F64, 112, 112, 1, 64, 7, 7)        \
    Y(MfmaF64x16, KM_F64, 144, 144, 1, 64, 9, 9)        \
    Y(MfmaF64x16, KM_F64, 160, 160, 1, 64, 10, 10)      \
    Y(MfmaF64x16, KM_F64, 192, 192, 1, 64, 12, 12)      \
    Y(MfmaF64x16, KM_F64, 32, 16, 1, 128, 4, 1)         \
    Y(MfmaF64x16, KM_F64, 16, 32, 1, 128, 4, 1)         \
    Y(MfmaF64x16, KM_F64, 64, 32, 1, 64, 4, 1)          \
    Y(MfmaF64x16, KM_F64, 32, 64, 1, 128, 4, 1)         \
    Y(MfmaF64x16, KM_F64, 16, 16, 2, 32, 8, 1)          \
    Y(MfmaF64x16, KM_F64, 16, 16, 2, 16, 4, 1)          \
    Y(MfmaF64x16, KM_F64, 16, 16, 1, 256, 4, 1)         \
    Y(MfmaF64x16, KM_F64, 16, 16, 1, 64, 4, 1)          \
    Y(MfmaF64x16, KM_F64, 16, 16, 1, 16, 1, 1)          \
    Y(MfmaF64x16, KM_F64, 32, 32, 2, 16, 8, 1)          \
    Y(MfmaF64x16, KM_F64, 32, 32, 1, 128, 4, 1)         \
    Y(MfmaF64x16, KM_F64, 32, 32, 1, 32, 2, 1)          \
    Y(MfmaF64x16, KM_F64, 64, 64, 1, 64, 8, 2)          \
    Y(MfmaF64x16, KM_F64, 64, 64, 1, 64, 4, 1)          \
    W(float, KM_F32, 2, 2, 4, 4, 4, 4, 256)             \
    W(float, KM_F32, 2, 2, 4, 4, 3, 8, 256)             \
    W(float, KM_F32, 2, 2, 4, 3, 3, 16, 256)            \
    W(float, KM_F32, 2, 2, 3, 3, 3, 32, 256)            \
    W(float, KM_F32, 2, 2, 4, 4, 0, 64, 256)            \
    W(float, KM_F32, 2, 2, 4, 3, 0, 128, 256)           \
    W(float, KM_F32, 2, 2, 3, 3, 0, 256, 256)           \
    W(float, KM_F32, 2, 2, 3, 2, 0, 512, 256)           \
    W(float, KM_F32, 2, 2, 4, 0, 0, 1024, 256)          \
    W(float, KM_F32, 2, 2, 3, 0, 0, 2048, 256)          \
    W(float, KM_F32, 2, 2, 2, 0, 0, 4096, 256)          \
    W(float, KM_F32, 2, 2, 1, 0, 0, 8192, 256)          \
    W(float, KM_F32, 4, 4, 3, 2, 2, 1, 256)             \
    W(float, KM_F32, 4, 4, 2, 2, 2, 4, 256)             \
    W(float, KM_F32, 4, 4, 2, 2, 1, 16, 256)            \
    W(float, KM_F32, 4, 4, 2, 2, 0, 64, 256)            \
    W(float, KM_F32, 4, 4, 2, 1, 0, 256, 256)           \
    W(float, KM_F32, 4, 4, 2, 0, 0, 1024, 256)          \
    W(float, KM_F32, 4, 4, 1, 0, 0, 4096, 256)          \
    W(float, KM_F32, 3, 3, 3, 2, 2, 9, 256)             \
    W(float, KM_F32, 3, 3, 2, 2, 2, 27, 256)            \
    W(float, KM_F32, 3, 3, 2, 2, 1, 81, 256)            \
    W(float, KM_F32, 3, 3, 2, 2, 0, 81, 256)            \
    W(float, KM_F32, 3, 3, 2, 1, 0, 243, 256)           \
    W(float, KM_F32, 3, 3, 2, 0, 0, 729, 256)           \
    W(float, KM_F32, 3, 3, 1, 0, 0, 2187, 256)          \
    W(float, KM_F32, 5, 5, 2, 2, 0, 25, 256)            \
    W(float, KM_F32, 5, 5, 2, 1, 0, 125, 256)           \
    W(float, KM_F32, 5, 5, 2, 0, 0, 625, 256)           \
    W(float, KM_F32, 5, 5, 1, 0, 0, 3125, 256)          \
    W(float, KM_F32, 6, 6, 2, 1, 0, 72, 256)            \
    W(float, KM_F32, 6, 6, 1, 1, 1, 72, 256)            \
    W(float, KM_F32, 6, 6, 2, 0, 0, 432, 256)           \
    W(float, KM_F32, 6, 6, 1, 0, 0, 2592, 256)          \
    W(double, KM_F64, 2, 2, 4, 4, 4, 2, 256)            \
    W(double, KM_F64, 2, 2, 4, 4, 3, 4, 256)            \
    W(double, KM_F64, 2, 2, 4, 3, 3, 8, 256)            \
    W(double, KM_F64, 2, 2, 3, 3, 3, 16, 256)           \
    W(double, KM_F64, 2, 2, 4, 4, 0, 32, 256)           \
    W(double, KM_F64, 2, 2, 4, 3, 0, 64, 256)           \
    W(double, KM_F64, 2, 2, 3, 3, 0, 128, 256)          \
    W(double, KM_F64, 2, 2, 3, 2, 0, 256, 256)          \
    W(double, KM_F64, 2, 2, 4, 0, 0, 512, 256)          \
    W(double, KM_F64, 2, 2, 3, 0, 0, 1024, 256)         \
    W(double, KM_F64, 2, 2, 1, 0, 0, 4096, 256)         \
    W(double, KM_F64, 4, 4, 3, 2, 2, 1, 512)            \
    W(double, KM_F64, 4, 4, 2, 2, 2, 2, 256)            \
    W(double, KM_F64, 4, 4, 2, 2, 1, 8, 256)            \
    W(double, KM_F64, 4, 4, 2, 2, 0, 32, 256)           \
    W(double, KM_F64, 4, 4, 2, 0, 0, 512, 256)          \
    W(double, KM_F64, 4, 4, 1, 0, 0, 2048, 256)         \
    X(double, KM_F64, 8, 8, 3, 16, 256)                 \
    W(double, KM_F64, 8, 8, 1, 1, 1, 16, 256)           \
    W(double, KM_F64, 8, 8, 1, 1, 0, 128, 256)          \
    W(double, KM_F64, 8, 8, 1, 0, 0, 1024, 256)         \
    W(double, KM_F64, 3, 3, 3, 2, 2, 3, 256)            \
    W(double, KM_F64, 3, 3, 2, 2, 2, 9, 256)            \
    W(double, KM_F64, 3, 3, 2, 2, 1, 27, 256)           \
    W(double, KM_F64, 3, 3, 2, 2, 0, 81, 256)           \
    W(double, KM_F64, 3, 3, 2, 1, 0, 243, 256)          \
    W(double, KM_F64, 3, 3, 2, 0, 0, 729, 256)          \
    W(double, KM_F64, 3, 3, 1, 0, 0, 2187, 256)         \
    W(double, KM_F64, 5, 5, 2, 1, 0, 25, 256)           \
    W(double, KM_F64, 5, 5, 2, 0, 0, 125, 256)          \
    W(double, KM_F64, 5, 5, 1, 0, 0, 625, 256)          \
    W(double, KM_F64, 6, 6, 1, 1, 1, 36, 256)           \
    W(double, KM_F64, 6, 6, 1, 1, 0, 216, 256)          \
    W(double, KM_F64, 6, 6, 1, 0, 0, 1296, 256)         \
    W(float, KM_F32, 8, 8, 1, 1, 1, 16, 256)            \
    W(float, KM_F32, 8, 8, 1, 1, 0, 128, 256)           \
    W(float, KM_F32, 8, 8, 1, 0, 0, 1024, 256)          \
    W(float, KM_F32, 7, 7, 2, 1, 0, 32, 256)            \
    W(float, KM_F32, 7, 7, 2, 0, 0, 256, 256)           \
    W(float, KM_F32, 7, 7, 1, 0, 0, 2048, 256)          \
    W(float, KM_F32, 9, 9, 1, 1, 1, 16, 256)            \
    W(float, KM_F32, 9, 9, 1, 1, 0, 128, 256)           \
    W(float, KM_F32, 9, 9, 1, 0, 0, 1024, 256)          \
    W(float, KM_F32, 10, 10, 1, 1, 1, 12, 256)          \
    W(float, KM_F32, 10, 10, 1, 1, 0, 100, 256)         \
    W(float, KM_F32, 10, 10, 1, 0, 0, 1000, 256)        \
    W(float, KM_F32, 12, 12, 1, 1, 0, 72, 256)          \
    W(float, KM_F32, 12, 12, 1, 0, 0, 864, 256)         \
    W(float, KM_F32, 11, 11, 1, 1, 0, 100, 256)         \
    W(float, KM_F32, 11, 11, 1, 0, 0, 1000, 256)        \
    W(float, KM_F32, 13, 13, 1, 1, 0, 64, 256)          \
    W(float, KM_F32, 13, 13, 1, 0, 0, 832, 256)         \
    W(float, KM_F32, 14, 14, 1, 1, 0, 64, 256)          \
    W(float, KM_F32, 14, 14, 1, 0, 0, 832, 256)         \
    W(float, KM_F32, 15, 15, 1, 1, 0, 64, 256)          \
    W(float, KM_F32, 15, 15, 1, 0, 0, 800, 256)         \
    W(double, KM_F64, 11, 11, 1, 1, 0, 50, 256)         \
    W(double, KM_F64, 11, 11, 1, 0, 0, 500, 256)        \
    W(double, KM_F64, 13, 13, 1, 1, 0, 32, 256)         \
    W(double, KM_F64, 13, 13, 1, 0, 0, 416, 256)        \
    W(double, KM_F64, 14, 14, 1, 1, 0, 32, 256)         \
    W(double, KM_F64, 14, 14, 1, 0, 0, 416, 256)        \
    W(double, KM_F64, 15, 15, 1, 1, 0, 32, 256)         \
    W(double, KM_F64, 15, 15, 1, 0, 0, 400, 256)        \
    W(double, KM_F64, 7, 7, 2, 1, 0, 16, 256)           \
    W(double, KM_F64, 7, 7, 2, 0, 0, 128, 256)          \
    W(double, KM_F64, 7, 7, 1, 0, 0, 1024, 256)         \
    W(double, KM_F64, 9, 9, 1, 1, 1, 8, 256)            \
    W(double, KM_F64, 9, 9, 1, 1, 0, 64, 256)           \
    W(double, KM_F64, 9, 9, 1, 0, 0, 512, 256)          \
    W(double, KM_F64, 10, 10, 1, 1, 1, 6, 256)          \
    W(double, KM_F64, 10, 10, 1, 1, 0, 50, 256)         \
    W(double, KM_F64, 10, 10, 1, 0, 0, 500, 256)        \
    W(double, KM_F64, 12, 12, 1, 1, 0, 36, 256)         \
    W(double, KM_F64, 12, 12, 1, 0, 0, 432, 256)        \
    W(float, KM_F32, 2, 4, 2, 2, 0, 16, 256)            \
    W(float, KM_F32, 2, 4, 2, 0, 0, 512, 256)           \
    W(float, KM_F32, 2, 4, 1, 0, 0, 2048, 256)          \
    W(float, KM_F32, 4, 2, 2, 2, 0, 32, 256)            \
    W(float, KM_F32, 4, 2, 2, 0, 0, 512, 256)           \
    W(float, KM_F32, 4, 2, 1, 0, 0, 2048, 256)          \
    W(float, KM_F32, 4, 8, 2, 1, 0, 16, 256)            \
    W(float, KM_F32, 4, 8, 2, 0, 0, 128, 256)           \
    W(float, KM_F32, 4, 8, 1, 0, 0, 1024, 256)          \
    W(float, KM_F32, 8, 4, 1, 1, 1, 16, 256)            \
    W(float, KM_F32, 8, 4, 1, 1, 0, 128, 256)           \
    W(float, KM_F32, 8, 4, 1, 0, 0, 1024, 256)          \
    W(double, KM_F64, 2, 4, 2, 2, 0, 8, 256)            \
    W(double, KM_F64, 2, 4, 2, 0, 0, 256, 256)          \
    W(double, KM_F64, 2, 4, 1, 0, 0, 1024, 256)         \
    W(double, KM_F64, 4, 2, 2, 2, 0, 16, 256)           \
    W(double, KM_F64, 4, 2, 2, 0, 0, 256, 256)          \
    W(double, KM_F64, 4, 2, 1, 0, 0, 1024, 256)         \
    W(double, KM_F64, 4, 8, 2, 1, 0, 8, 256)            \
    W(double, KM_F64, 4, 8, 2, 0, 0, 64, 256)           \
    W(double, KM_F64, 4, 8, 1, 0, 0, 512, 256)          \
    W(double, KM_F64, 8, 4, 1, 1, 1, 8, 256)            \
    W(double, KM_F64, 8, 4, 1, 1, 0, 64, 256)           \
    W(double, KM_F64, 8, 4, 1, 0, 0, 512, 256)          \
    V(float, KM_F32, 2, 2, 4, 4, 4, 3, 4, 4, 2, 1, 256)    /* 4x4^5, 2x2^4 */ \
    V(float, KM_F32, 2, 2, 4, 4, 4, 2, 4, 4, 2, 4, 256)    /* 4x4^4, 2x2^4 */ \
    V(float, KM_F32, 2, 2, 4, 4, 4, 2, 0, 0, 0, 64, 256)   /* 4x4^2, 2x2^4 */ \
    V(float, KM_F32, 2, 2, 3, 4, 4, 2, 0, 0, 0, 128, 256)  /* 4x4^2, 2x2^3 */ \
    V(float, KM_F32, 4, 4, 2, 2, 2, 4, 2, 2, 4, 4, 256)    /* 2x2^8, 4x4^2 */ \
    V(float, KM_F32, 4, 4, 2, 2, 2, 4, 0, 0, 0, 64, 256)   /* 2x2^4, 4x4^2 */ \
    V(float, KM_F32, 4, 4, 2, 8, 8, 1, 8, 8, 1, 16, 256)   /* 8x8^2, 4x4^2 */ \
    V(float, KM_F32, 8, 8, 1, 8, 8, 1, 4, 4, 2, 16, 256)   /* 4x4^2, 8x8^2 */ \
    V(float, KM_F32, 2, 2, 3, 8, 8, 1, 8, 8, 1, 32, 256)   /* 8x8^2, 2x2^3 */ \
    V(float, KM_F32, 8, 8, 1, 8, 8, 1, 2, 2, 3, 32, 256)   /* 2x2^3, 8x8^2 */ \
    V(float, KM_F32, 2, 2, 1, 5, 5, 2, 0, 0, 0, 256, 256)  /* 5x5^2, 2x2 */ \
    V(float, KM_F32, 5, 5, 2, 2, 2, 1, 0, 0, 0, 256, 256)  /* 2x2, 5x5^2 */ \
    V(float, KM_F32, 2, 2, 2, 3, 3, 2, 0, 0, 0, 432, 256)  /* 3x3^2, 2x2^2 */ \
    V(double, KM_F64, 2, 2, 4, 4, 4, 2, 4, 4, 2, 2, 256)   /* 4x4^4, 2x2^4 */ \
    V(double, KM_F64, 2, 2, 4, 4, 4, 2, 0, 0, 0, 32, 256)  /* 4x4^2, 2x2^4 */ \
    V(double, KM_F64, 4, 4, 2, 2, 2, 4, 0, 0, 0, 32, 256)  /* 2x2^4, 4x4^2 */ \
    V(double, KM_F64, 4, 4, 2, 8, 8, 1, 8, 8, 1, 8, 256)   /* 8x8^2, 4x4^2 */ \
    V(double, KM_F64, 2, 2, 1, 5, 5, 2, 0, 0, 0, 128, 256) /* 5x5^2, 2x2 */ \
    U(float, KM_F32, 13, 13, 1, 1, 1, 1, 1, 1024)       \
    U(float, KM_F32, 12, 12, 1, 1, 1, 1, 1, 1024)       \
    U(float, KM_F32, 14, 14, 1, 1, 1, 1, 1, 1024)       \
    U(float, KM_F32, 11, 11, 1, 1, 1, 1, 1, 512)        \
    U(float, KM_F32, 10, 10, 1, 1, 1, 1, 1, 512)        \
    U(float, KM_F32, 9, 9, 1, 1, 1, 1, 1, 256)          \
    U(double, KM_F64, 11, 11, 1, 1, 1, 1, 1, 1024)      \
    U(double, KM_F64, 10, 10, 1, 1, 1, 1, 1, 512)       \
    U(double, KM_F64, 9, 9, 1, 1, 1, 1, 1, 512)         \
    U(float, KM_F32, 8, 8, 1, 1, 1, 1, 2, 512)          \
    U(float, KM_F32, 7, 7, 2, 1, 1, 1, 1, 512)          \
    U(float, KM_F32, 7, 7, 1, 1, 1, 1, 4, 256)          \
    U(float, KM_F32, 6, 6, 2, 1, 1, 1, 1, 512)          \
    U(float, KM_F32, 5, 5, 2, 2, 1, 1, 1, 512)          \
    U(float, KM_F32, 5, 5, 2, 1, 1, 1, 2, 256)          \
    U(float, KM_F32, 3, 3, 3, 2, 2, 2, 1, 512)          \
    U(float, KM_F32, 3, 3, 2, 2, 2, 2, 1, 256)          \
    U(float, KM_F32, 2, 2, 4, 4, 4, 3, 1, 1024)         \
    U(float, KM_F32, 2, 2, 4, 4, 3, 3, 1, 1024)         \
    U(float, KM_F32, 2, 2, 4, 3, 3, 3, 1, 512)          \
    U(double, KM_F64, 8, 8, 1, 1, 1, 1, 1, 512)         \
    U(double, KM_F64, 7, 7, 2, 1, 1, 1, 1, 512)         \
    U(double, KM_F64, 7, 7, 1, 1, 1, 1, 2, 256)         \
    U(double, KM_F64, 6, 6, 2, 1, 1, 1, 1, 512)         \
    U(double, KM_F64, 6, 6, 1, 1, 1, 1, 4, 256)         \
    U(double, KM_F64, 5, 5, 2, 2, 1, 1, 1, 1024)        \
    U(double, KM_F64, 5, 5, 2, 1, 1, 1, 1, 256)         \
    U(double, KM_F64, 5, 5, 2, 1, 1, 0, 8, 256)         \
    U(double, KM_F64, 3, 3, 3, 2, 2, 2, 1, 1024)        \
    U(double, KM_F64, 3, 3, 2, 2, 2, 2, 1, 512)         \
    U(double, KM_F64, 2, 2, 4, 4, 3, 3, 1, 1024)        \
    U(double, KM_F64, 2, 2, 4, 3, 3, 3, 1, 512)         \
    U(float, KM_F32, 6, 6, 1, 1, 1, 1, 4, 256)          \
    U(float, KM_F32, 11, 11, 1, 1, 1, 0, 4, 256)        \
    U(float, KM_F32, 12, 12, 1, 1, 1, 0, 3, 256)        \
    U(float, KM_F32, 13, 13, 1, 1, 1, 0, 2, 256)        \
    U(float, KM_F32, 14, 14, 1, 1, 1, 0, 2, 256)        \
    U(float, KM_F32, 15, 15, 1, 1, 1, 0, 1, 256)        \
    U(double, KM_F64, 11, 11, 1, 1, 1, 0, 4, 256)       \
    U(double, KM_F64, 12, 12, 1, 1, 1, 0, 3, 256)       \
    U(double, KM_F64, 13, 13, 1, 1, 1, 0, 2, 256)       \
    U(double, KM_F64, 14, 14, 1, 1, 1, 0, 2, 256)       \
    U(double, KM_F64, 15, 15, 1, 1, 1, 0, 1, 256)       \
    U(float, KM_F32, 2, 4, 2, 2, 2, 0, 1, 256)          \
    U(float, KM_F32, 2, 4, 2, 2, 2, 1, 1, 512)          \
    U(float, KM_F32, 4, 2, 2, 2, 2, 0, 1, 256)          \
    U(float, KM_F32, 4, 2, 2, 2, 2, 1, 1, 512)          \
    U(float, KM_F32, 4, 8, 2, 1, 1, 0, 1, 256)          \
    U(float, KM_F32, 4, 8, 2, 1, 1, 1, 1, 512)          \
    U(float, KM_F32, 8, 4, 1, 1, 1, 1, 1, 256)          \
    U(float, KM_F32, 8, 4, 2, 1, 1, 1, 1, 1024)         \
    U(double, KM_F64, 2, 4, 2, 2, 2, 0, 1, 256)         \
    U(double, KM_F64, 2, 4, 2, 2, 2, 1, 1, 512)         \
    U(double, KM_F64, 4, 2, 2, 2, 2, 0, 1, 256)         \
    U(double, KM_F64, 4, 2, 2, 2, 2, 1, 1, 1024)        \
    U(double, KM_F64, 4, 8, 2, 1, 1, 0, 1, 256)         \
    U(double, KM_F64, 4, 8, 2, 1, 1, 1, 1, 1024)        \
    U(double, KM_F64, 8, 4, 1, 1, 1, 1, 1, 256)
