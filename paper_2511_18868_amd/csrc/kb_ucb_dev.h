// Device pieces of the selection step (Eq. 6, Sec. 3.4) shared by the selection
// kernels and the one-launch round of very short searches.
#pragma once
#include "kb_internal.h"

namespace kb {

struct UcbArgs {
    int G, S, Ksum, Kmax;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const int32_t* assign;
    const uint8_t* alive;       // NULL: every candidate alive
    const float* bound;         // NULL: all bounds equal (k* = lowest-index member)
    const uint8_t* M;           // NULL or [Ksum*S]: cluster arms allowed by the strategy mask
    const int32_t* visits;
    const float* rsum;
    const int64_t* t;
    float c, prior_n, prior_mu;
    int32_t* Ncs;
    float* mu;
    float* ucb;
    int32_t* sel;
    const int32_t* order;
    unsigned* gN;               // [Ksum*S]  global tables of the chunked path
    unsigned long long* gR;     // [Ksum*S]
    unsigned* gnalive;          // [Ksum]
    unsigned long long* gkmin;  // [Ksum]
    int64_t Nll;
    int mixed;                  // 1: searches of up to kUcbLong candidates go to ucb_kernel, longer ones to the
                                //    range kernels, in the same call
    int keep;                   // 1: ucb_kernel leaves a copy of its LDS tables in the global ones
};

constexpr double kRewardInv = 1.0 / 1073741824.0;

// Monotone map from float to uint32 (a < b  <=>  key(a) < key(b)), so an
// integer atomic min orders bounds of any sign.
__device__ __forceinline__ unsigned ordered_bits(float f) {
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One alive candidate's visits and reward sums (row `row` of the two arrays) into the
// tables of its cluster j; p is its index inside the search and bd its roofline bound
// (the member with the smallest bound, lowest index on ties, is the cluster's k*).
// For the kernels in which a lane owns a whole candidate.
__device__ __forceinline__ void ucb_add_candidate(const UcbArgs& a, size_t row, int p, int j, float bd,
                                                  unsigned* Ncnt, unsigned long long* R,
                                                  unsigned* nalive, unsigned long long* kmin) {
    const int S = a.S;
    const int32_t* vis = a.visits + row * S;
    const float* rs = a.rsum + row * S;
    unsigned* nc = Ncnt + (size_t)j * S;
    unsigned long long* rr = R + (size_t)j * S;
    if ((S & 3) == 0) {
        for (int s = 0; s < S; s += 4) {
            const int4 v = *reinterpret_cast<const int4*>(vis + s);
            const float4 r = *reinterpret_cast<const float4*>(rs + s);
            atomicAdd(nc + s + 0, (unsigned)v.x); atomicAdd(nc + s + 1, (unsigned)v.y);
            atomicAdd(nc + s + 2, (unsigned)v.z); atomicAdd(nc + s + 3, (unsigned)v.w);
            atomicAdd(rr + s + 0, reward_fixed(r.x)); atomicAdd(rr + s + 1, reward_fixed(r.y));
            atomicAdd(rr + s + 2, reward_fixed(r.z)); atomicAdd(rr + s + 3, reward_fixed(r.w));
        }
    } else {
        for (int s = 0; s < S; ++s) {
            atomicAdd(nc + s, (unsigned)vis[s]);
            atomicAdd(rr + s, reward_fixed(rs[s]));
        }
    }
    atomicAdd(&nalive[j], 1u);
    atomicMin(&kmin[j], ((unsigned long long)ordered_bits(bd) << 32) | (unsigned)p);
}

// Scores, outputs and selection of one search from its accumulated tables
// (which may live in LDS or in global memory).  Called by a whole workgroup of NT
// threads, or, with NT = 64, by one wave on its own (tid = the lane; redv and redi
// are then unused and no workgroup barrier is reached).
template <int NT>
__device__ __forceinline__ void ucb_finish(const UcbArgs& a, int g, int n0, int k0, int K,
                                           const unsigned* Ncnt, const unsigned long long* R,
                                           const unsigned* nalive, const unsigned long long* kmin,
                                           double* redv, int* redi, int tid) {
    const int S = a.S;
    const int KS = K * S;
    long long tg = a.t[g];
    if (tg < 1) tg = 1;
    const double lnt = log((double)tg);
    const double pn = (double)a.prior_n, pm = (double)a.prior_mu, cc = (double)a.c;

    double bu = -INFINITY;
    int bf = -1;
    for (int i = tid; i < KS; i += NT) {
        const int cl = i / S;
        const unsigned n = Ncnt[i];
        const double nt = (double)n + pn;
        const double rt = (double)(long long)R[i] * kRewardInv + pn * pm;
        const double m = nt > 0.0 ? rt / nt : NAN;
        double u;
        const bool valid = nalive[cl] > 0u && (!a.M || a.M[(size_t)k0 * S + i] != 0);
        if (!valid) u = -INFINITY;
        else if (nt > 0.0) u = m + cc * sqrt(lnt / nt);
        else u = INFINITY;
        const size_t o = (size_t)k0 * S + i;
        a.Ncs[o] = (int32_t)n;
        a.mu[o] = (float)m;
        a.ucb[o] = (float)u;
        if (valid && (bf < 0 || u > bu)) { bu = u; bf = i; }
    }
    // argmax with the lowest flat index on ties: waves, then the block
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double ou = __shfl_xor(bu, o);
        const int of = __shfl_xor(bf, o);
        if (of >= 0 && (bf < 0 || ou > bu || (ou == bu && of < bf))) { bu = ou; bf = of; }
    }
    if constexpr (NT > 64) {
        if ((tid & 63) == 0) { redv[tid >> 6] = bu; redi[tid >> 6] = bf; }
        __syncthreads();
    }
    if (tid == 0) {
        for (int w = 1; w < NT / 64; ++w) {
            const double ou = redv[w];
            const int of = redi[w];
            if (of >= 0 && (bf < 0 || ou > bu || (ou == bu && of < bf))) { bu = ou; bf = of; }
        }
        int I = -1, Ss = -1, ks = -1;
        if (bf >= 0) {
            I = bf / S;
            Ss = bf - I * S;
            ks = n0 + (int)(unsigned)(kmin[I] & 0xffffffffull);
        }
        a.sel[(size_t)g * 3 + 0] = I;
        a.sel[(size_t)g * 3 + 1] = Ss;
        a.sel[(size_t)g * 3 + 2] = ks;
    }
}

// The argument block of a selection call on batch b.
inline UcbArgs make_ucb_args(const kb_batch& b, const UcbCall& c) {
    UcbArgs a;
    a.G = b.G; a.S = b.S; a.Ksum = b.Ksum; a.Kmax = b.Kmax > 0 ? b.Kmax : 1; a.N = b.N;
    a.seg_off = b.seg_off; a.koff = b.koff; a.assign = c.assign; a.alive = c.alive;
    a.bound = c.bound; a.M = c.M; a.visits = c.visits; a.rsum = c.rsum; a.t = c.t; a.c = c.c;
    a.prior_n = c.prior_n; a.prior_mu = c.prior_mu; a.Ncs = c.Ncs; a.mu = c.mu; a.ucb = c.ucb;
    a.sel = c.sel;
    a.order = b.G > 1 ? c.order : nullptr;       // (one search: the order is the identity and was not computed)
    a.gN = c.gN; a.gR = c.gR; a.gnalive = c.gnalive; a.gkmin = c.gkmin; a.Nll = b.N;
    a.mixed = 0;
    a.keep = 0;
    return a;
}

}  // namespace kb
