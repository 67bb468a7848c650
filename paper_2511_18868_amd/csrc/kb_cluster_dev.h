// Device helpers shared by the clustering kernels.
#pragma once
#include "kb_internal.h"

namespace kb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kFlagBit = (int)0x80000000u;
constexpr float kBig = 1.0e30f;    // score of a centroid row that does not exist

// Fixed-point image of one feature value: floor(x * 2^sh) as a 64-bit integer.
// x * scale is exact (power-of-two scale); it is cut into a high and a low
// 32-bit half with exact fp64 operations, so only the final cut below one unit
// of the fixed-point grid rounds (toward -inf, the same way every time a value
// is added or taken away).
__device__ __forceinline__ long long to_fixed(float x, double scale) {
    const double d = (double)x * scale;
    const double hi = floor(d * 2.3283064365386963e-10);          // d / 2^32
    const double lo = fma(hi, -4294967296.0, d);                   // in [0, 2^32)
    const int ihi = __double2int_rz(hi);
    const unsigned ilo = __double2uint_rz(lo);
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

// error bound factor of the matrix-core scores, see the scorer's comment
__device__ __forceinline__ float mfma_kappa(int DS) {
    return 3.1f * 1.52587890625e-05f + (float)(3 * 16 * DS + 4) * 2.384185791015625e-07f;
}

}  // namespace kb
