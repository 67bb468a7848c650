// Counter-based random variates for the reproducible draws (in-cluster draw of
// k_t, randomised seeding): Philox4x32 with 10 rounds (Salmon, Moraes, Dror,
// Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11), written from its
// published definition.
#pragma once
#include "kb_internal.h"

namespace kb {

// Each round multiplies counter words 0 and 2 by the two round constants, mixes
// the high halves with the other two words and the key, and the key advances by
// the Weyl constants between rounds.  Returns the first two output words.
__device__ __forceinline__ void philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3,
                                              unsigned k0, unsigned k1, unsigned& o0, unsigned& o1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const unsigned h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const unsigned h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        c0 = h1 ^ c1 ^ k0;
        c1 = l1;
        c2 = h0 ^ c3 ^ k1;
        c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    o0 = c0;
    o1 = c1;
}

// The standard Gumbel variate -ln(-ln u) of candidate k (global index) in draw
// (draw_hi, draw_lo) under the key (seed_hi, seed_lo): counter (k, 0, draw_lo,
// draw_hi); u = (m + 1/2) 2^-52 with m the first 52 output bits, strictly inside
// (0, 1) and exact in fp64.
__device__ __forceinline__ double gumbel_variate(unsigned seed_lo, unsigned seed_hi, unsigned draw_lo,
                                                 unsigned draw_hi, int k) {
    unsigned x0, x1;
    philox4x32_10((unsigned)k, 0u, draw_lo, draw_hi, seed_lo, seed_hi, x0, x1);
    const unsigned long long m = ((unsigned long long)x0 << 20) | (unsigned long long)(x1 >> 12);
    const double u = ((double)m + 0.5) * (1.0 / 4503599627370496.0);
    return -log(-log(u));
}

}  // namespace kb
