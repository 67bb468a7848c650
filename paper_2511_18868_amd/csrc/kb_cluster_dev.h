// Device helpers shared by the clustering kernels.
#pragma once
#include "kb_internal.h"

namespace kb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kFlagBit = (int)0x80000000u;
constexpr int kRefinedBit = 0x40000000;     // proposal decided by the scan over all candidates, not yet applied
constexpr float kBig = 1.0e30f;    // score of a centroid row that does not exist

// Fixed-point image of one feature value: x * 2^sh as a 64-bit integer, from
// fsh = sh - 32.  t = x * 2^fsh (a power-of-two scaling; below 2^31 in size by the
// choice of sh) is cut into its floor, which becomes the (signed) high word, and
// its fractional part t - floor(t) (the hardware's fract, which stays below 1),
// whose first 32 bits become the low word - five vector instructions.  The
// fractional part is exact for t >= 0 and for t <= -1; for -1 < t < 0 it is 1 + t
// rounded to fp32, off by at most 2^-25 (of a high-word unit, i.e. 2^-25 of the
// 2^-fsh that already lies 30 - log2(N_g) bits below max |x|).  What matters is
// that the same value results every time a feature is added to or taken out of
// a sum.
__device__ __forceinline__ long long to_fixed(float x, int fsh) {
    const float t = ldexpf(x, fsh);
    int ihi;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(ihi) : "v"(t));          // floor and conversion in one
    const float lo = ldexpf(__builtin_amdgcn_fractf(t), 32);      // below 2^32
    const unsigned ilo = (unsigned)lo;                            // truncates
    return (long long)(((unsigned long long)(unsigned)ihi << 32) | ilo);
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

// the value lane l holds, l the same in every lane (a scalar-register read, no
// cross-lane traffic through LDS)
__device__ __forceinline__ float lane_value(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// v = hi + mid + rest with hi = bf16(v), mid = bf16(v - hi), round to nearest even;
// two features per conversion instruction
__device__ __forceinline__ void split8(const float (&v)[8], bf16x8& hi, bf16x8& mid) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const f32x2 x = {v[2 * p], v[2 * p + 1]};
        const bf16x2 h = __builtin_convertvector(x, bf16x2);
        const unsigned hb = __builtin_bit_cast(unsigned, h);
        const f32x2 r = {x.x - __uint_as_float(hb << 16), x.y - __uint_as_float(hb & 0xffff0000u)};
        const bf16x2 m = __builtin_convertvector(r, bf16x2);
        hi[2 * p] = h.x; hi[2 * p + 1] = h.y;
        mid[2 * p] = m.x; mid[2 * p + 1] = m.y;
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
