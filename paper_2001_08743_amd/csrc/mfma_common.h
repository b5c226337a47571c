// Pieces shared by the matrix-core kernels (resident and streaming): fragment types, the error
// bound of the f16 hi/lo screen, half-wave exchange and score-index decoding.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cham {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kRecCap = 64;            // queued rows whose knob values are kept in LDS
constexpr float kBiasScale = 256.0f;   // value of the bias slot in B (exact in f16)
constexpr float kPadBiasHi = 65504.0f; // A value of the bias slot for padding centroid rows:
                                       // 256 * 65504 exceeds every real score (<= 4 * 31 * 255^2)

// Error bound of the matrix-core screen, relative to (|x'|^2 + 2 max|mu'|^2), in units of 2^-24:
// w = fl32(-2mu') and the bias are rounded once (1 each) and hi + lo keeps 22 bits (4);
// each instruction adds 16 exact products to the running value: the hardware aligns the 17 addends
// to the largest and rounds once, modelled generously as 18 units per instruction (NS2 chained
// instructions).  The factor 2.5 = 2 (two scores are compared) x 1.25 headroom.  The absolute
// term covers f16 underflow of the low parts.
template <int NS2>
__device__ __forceinline__ float mfma_bound(float x2, float m2)
{
    constexpr float kE = 2.5f * (float)(18 * NS2 + 6) * 5.9604644775390625e-8f;
    return kE * (x2 + 2.0f * m2) + 4.0e-5f;
}

__device__ __forceinline__ float min3f(float a, float b, float c)
{
    return __builtin_fminf(__builtin_fminf(a, b), c);
}

// Both 32-lane halves of a value: lo = the value held by lanes 0..31, hi = by lanes 32..63
// (v_permlane32_swap: a VALU exchange, no LDS round trip).
__device__ __forceinline__ void both_halves(unsigned v, unsigned &lo, unsigned &hi)
{
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    lo = r[0];
    hi = r[1];
}
__device__ __forceinline__ float min_halves(float v)
{
    unsigned lo, hi;
    both_halves(__float_as_uint(v), lo, hi);
    return __builtin_fminf(__uint_as_float(lo), __uint_as_float(hi));
}

// centroid index of score q (processing order: m-tile, then accumulator register) in lane half hh
__device__ __forceinline__ int centroid_of(int q, int hh)
{
    return 32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * hh + (q & 3);
}

}  // namespace cham
