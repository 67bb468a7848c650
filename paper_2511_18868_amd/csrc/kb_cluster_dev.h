// Device helpers shared by the clustering kernels.
#pragma once
#include "kb_internal.h"

namespace kb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kFlagBit = (int)0x80000000u;
constexpr float kBig = 1.0e30f;    // score of a centroid row that does not exist

// Fixed-point image of one feature value: x * 2^sh cut to a 64-bit integer
// (toward zero, so the image of -x is minus the image of x), from fsh = sh - 32.
// Only exact fp32 steps are used: |x| * 2^fsh (a power-of-two scaling; < 2^31 by
// the choice of sh) is cut into its integer part, which becomes the high word,
// and its fraction, whose first 32 bits become the low word.  The same value
// results every time a feature is added to or taken out of a sum.
__device__ __forceinline__ long long to_fixed(float x, int fsh) {
    const float t = ldexpf(fabsf(x), fsh);
    const float hi = floorf(t);
    const float lo = ldexpf(t - hi, 32);          // t - hi is exact and in [0, 1)
    const unsigned ihi = (unsigned)hi;
    const unsigned ilo = (unsigned)lo;           // truncates
    const long long mag = (long long)(((unsigned long long)ihi << 32) | ilo);
    return x < 0.f ? -mag : mag;
}

// Shift of the fixed-point grid for a search: |x| < 2^e and N_g < 2^bits give
// |sum of q| < 2^62 for sh = 62 - e - bits.  e is rounded up to a multiple of 4,
// so that an estimate of max |x| from part of the rows usually yields the same
// shift as the true maximum (the grid stays finer than 2^-37 of max |x| for
// searches of up to 2^20 candidates, far below an fp32 ulp of any centroid).
__device__ __forceinline__ int fixed_shift(float amax, int ng) {
    int e = 0;
    if (amax > 0.f) (void)frexpf(amax, &e);
    e = clampi(e, -126, 129);
    e = ((e + 3) >> 2) << 2;
    return 62 - e - (32 - __clz(ng));
}

// v = hi + mid + rest with hi = bf16(v), mid = bf16(v - hi), round to nearest even
__device__ __forceinline__ void split8(const float (&v)[8], bf16x8& hi, bf16x8& mid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const __bf16 h = (__bf16)v[i];
        hi[i] = h;
        mid[i] = (__bf16)(v[i] - (float)h);
    }
}

// (best, second best, index of best) of the union of two sets
__device__ __forceinline__ void merge_best(float& b1, float& s1, int& i1, float b2, float s2, int i2) {
    const bool take = b2 < b1;
    const float hi2 = take ? b1 : b2;        // the larger of the two bests
    const float sm = s2 < s1 ? s2 : s1;
    s1 = sm < hi2 ? sm : hi2;
    i1 = take ? i2 : i1;
    b1 = take ? b2 : b1;
}

// error bound factor of the matrix-core scores, see the scorer's comment; the last
// term covers the position bits written into a score (|score| <= 2 (|x|^2 + max |c|^2),
// moved by less than 2^-18 of itself)
__device__ __forceinline__ float mfma_kappa(int DS) {
    return 3.1f * 1.52587890625e-05f + (float)(3 * 16 * DS + 4) * 2.384185791015625e-07f +
           7.62939453125e-06f;
}

// Plain v_min_f32 / v_max_f32.  (fminf would first quiet a signalling NaN with one
// more instruction per operand, because the compiler cannot see that scores
// with rewritten low bits are ordinary numbers.)
__device__ __forceinline__ float vmin(float x, float y) {
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}
__device__ __forceinline__ float vmax(float x, float y) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}

}  // namespace kb
