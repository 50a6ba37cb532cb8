// Device-side building blocks shared by the FPS kernels (gfx950, wave64).
//
// Everything that decides a pick is written so that the result does not depend
// on the launch shape: distances use individually rounded fp32 operations (no
// FMA), and every reduction orders candidates by (value descending, index
// ascending), which is a total order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace ffps {

constexpr int kWave = 64;

// Squared distance of Eq. 1's norm: ((dx*dx) + (dy*dy)) + (dz*dz), each
// operation rounded to nearest-even fp32, never contracted.
__device__ __forceinline__ float sqdist(float x, float y, float z, float lx, float ly, float lz) {
    float dx = __fsub_rn(x, lx);
    float dy = __fsub_rn(y, ly);
    float dz = __fsub_rn(z, lz);
    float xx = __fmul_rn(dx, dx);
    float yy = __fmul_rn(dy, dy);
    float zz = __fmul_rn(dz, dz);
    return __fadd_rn(__fadd_rn(xx, yy), zz);
}

// min of two distances as one instruction.  fminf would first canonicalise its
// operands (an extra instruction per call) to quiet signalling NaNs, which
// cannot occur here: distances of finite points are never NaN.
__device__ __forceinline__ float min_dist(float a, float b) {
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// The same for two new distances at once: with two waves on a SIMD a minimum costs
// about twice an addition, and the three-operand form costs no more than the plain one.
__device__ __forceinline__ float min3_dist(float a, float b, float c) {
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Distances are >= +0 (or +inf), so their IEEE bit patterns order like
// unsigned integers; reductions run on the bits.
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// --- DPP cross-lane moves (GFX9 encodings) ----------------------------------
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    // lanes whose source is out of range, or whose row is masked off, get 0:
    // the identity of an unsigned max
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Unsigned max over each row of 16 lanes; the result is in lanes 15, 31, 47, 63.
__device__ __forceinline__ uint32_t row16_max_u32(uint32_t v) {
    v = umax(v, dpp_or_zero<kDppRowShr1>(v));
    v = umax(v, dpp_or_zero<kDppRowShr2>(v));
    v = umax(v, dpp_or_zero<kDppRowShr4>(v));
    v = umax(v, dpp_or_zero<kDppRowShr8>(v));
    return v;
}

// Unsigned max over the 64 lanes of a wave, returned as a wave-uniform value:
// rows of 16, then pairs of rows (lanes 31 and 63 hold the halves' maxima), and
// the last step on the scalar unit, which is shorter than a third cross-row move.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = row16_max_u32(v);
    v = umax(v, dpp_or_zero<kDppRowBcast15, 0xa>(v));
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
    return lo > hi ? lo : hi;
}

// Lowest lane for which pred holds (pred must hold in at least one lane).
__device__ __forceinline__ int first_lane(bool pred) {
    return (int)__builtin_ctzll(__builtin_amdgcn_ballot_w64(pred));
}

__device__ __forceinline__ float readlane_f(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ int readlane_i(int v, int lane) {
    return __builtin_amdgcn_readlane(v, lane);
}

// Coordinates of element `sel` of lane `lane` (both wave-uniform) of three
// register arrays: a scalar jump picks the element, then three lane reads.
template <int P>
__device__ __forceinline__ void pick_xyz(const float (&x)[P], const float (&y)[P],
                                         const float (&z)[P], int sel, int lane, float &ox,
                                         float &oy, float &oz) {
    ox = oy = oz = 0.f;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        if (sel == j) {
            ox = readlane_f(x[j], lane);
            oy = readlane_f(y[j], lane);
            oz = readlane_f(z[j], lane);
        }
    }
}

}  // namespace ffps
