// Cluster-arm statistics, masked UCB index and arm selection (Eq. 6, Sec. 3.4).
//
// One workgroup per search streams the search's visits / reward-sum rows once
// (flat, coalesced 16-byte loads) and scatters them into K x S accumulators in
// LDS keyed by the candidate's cluster.  All accumulators are integers - visit
// counts as they are, reward sums in 2^-30 fixed point (a cluster's reward sum
// is below its visit count, which is below 2^31) - so the LDS atomics commute
// and the statistics are bit-identical from run to run.  The per-cluster "most
// headroom" candidate is a 64-bit atomic min over (ordered bound bits, index).
// Scores are formed in fp64 from the accumulators, compared in fp64, and
// rounded to fp32 on output.
#include "kb_internal.h"

namespace kb {

namespace {

struct UcbArgs {
    int G, S, Ksum, Kmax;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const int32_t* assign;
    const uint8_t* alive;
    const float* bound;
    const int32_t* visits;
    const float* rsum;
    const int64_t* t;
    float c, prior_n, prior_mu;
    int32_t* Ncs;
    float* mu;
    float* ucb;
    int32_t* sel;
    const int32_t* order;
};

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr double kRewardScale = 1073741824.0;          // 2^30
constexpr double kRewardInv = 1.0 / 1073741824.0;

// Monotone map from float to uint32 (a < b  <=>  key(a) < key(b)), so an
// integer atomic min orders bounds of any sign.
__device__ __forceinline__ unsigned ordered_bits(float f) {
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(kThreads) ucb_kernel(UcbArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int S = a.S;

    int g = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;
    g = clampi(g, 0, a.G - 1);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (ng <= 0 || K <= 0) {
        if (tid < 3) a.sel[(size_t)g * 3 + tid] = -1;
        return;
    }
    const int KS = K * S;

    double* redv = reinterpret_cast<double*>(smem);                                      // [kWaves]
    int* redi = reinterpret_cast<int*>(smem + 32);                                       // [kWaves]
    unsigned long long* R = reinterpret_cast<unsigned long long*>(smem + 64);            // [Kmax*S]
    unsigned long long* kmin = R + (size_t)a.Kmax * S;                                   // [Kmax]
    unsigned* Ncnt = reinterpret_cast<unsigned*>(kmin + a.Kmax);                         // [Kmax*S]
    unsigned* nalive = Ncnt + (size_t)a.Kmax * S;                                        // [Kmax]

    for (int i = tid; i < KS; i += kThreads) { R[i] = 0ull; Ncnt[i] = 0u; }
    for (int i = tid; i < K; i += kThreads) { kmin[i] = ~0ull; nalive[i] = 0u; }
    __syncthreads();

    const int32_t* vis = a.visits + (size_t)n0 * S;
    const float* rs = a.rsum + (size_t)n0 * S;
    if ((S & 3) == 0) {
        const int S4 = S >> 2;
        const size_t quads = (size_t)ng * S4;
        for (size_t q = tid; q < quads; q += kThreads) {
            const int p = (int)(q / S4);
            const int s0 = (int)(q - (size_t)p * S4) * 4;
            if (!a.alive[(size_t)n0 + p]) continue;
            int j = a.assign[(size_t)n0 + p];
            j = (j >= 0 && j < K) ? j : 0;
            const int4 v = reinterpret_cast<const int4*>(vis)[q];
            const float4 r = reinterpret_cast<const float4*>(rs)[q];
            unsigned* nc = Ncnt + (size_t)j * S + s0;
            unsigned long long* rr = R + (size_t)j * S + s0;
            atomicAdd(nc + 0, (unsigned)v.x); atomicAdd(nc + 1, (unsigned)v.y);
            atomicAdd(nc + 2, (unsigned)v.z); atomicAdd(nc + 3, (unsigned)v.w);
            atomicAdd(rr + 0, (unsigned long long)__double2ll_rn((double)r.x * kRewardScale));
            atomicAdd(rr + 1, (unsigned long long)__double2ll_rn((double)r.y * kRewardScale));
            atomicAdd(rr + 2, (unsigned long long)__double2ll_rn((double)r.z * kRewardScale));
            atomicAdd(rr + 3, (unsigned long long)__double2ll_rn((double)r.w * kRewardScale));
            if (s0 == 0) {
                atomicAdd(&nalive[j], 1u);
                const unsigned long long key =
                    ((unsigned long long)ordered_bits(a.bound[(size_t)n0 + p]) << 32) | (unsigned)p;
                atomicMin(&kmin[j], key);
            }
        }
    } else {
        const size_t total = (size_t)ng * S;
        for (size_t q = tid; q < total; q += kThreads) {
            const int p = (int)(q / S);
            const int s = (int)(q - (size_t)p * S);
            if (!a.alive[(size_t)n0 + p]) continue;
            int j = a.assign[(size_t)n0 + p];
            j = (j >= 0 && j < K) ? j : 0;
            atomicAdd(&Ncnt[(size_t)j * S + s], (unsigned)vis[q]);
            atomicAdd(&R[(size_t)j * S + s],
                      (unsigned long long)__double2ll_rn((double)rs[q] * kRewardScale));
            if (s == 0) {
                atomicAdd(&nalive[j], 1u);
                const unsigned long long key =
                    ((unsigned long long)ordered_bits(a.bound[(size_t)n0 + p]) << 32) | (unsigned)p;
                atomicMin(&kmin[j], key);
            }
        }
    }
    __syncthreads();

    long long tg = a.t[g];
    if (tg < 1) tg = 1;
    const double lnt = log((double)tg);
    const double pn = (double)a.prior_n, pm = (double)a.prior_mu, cc = (double)a.c;

    double bu = -INFINITY;
    int bf = -1;
    for (int i = tid; i < KS; i += kThreads) {
        const int cl = i / S;
        const unsigned n = Ncnt[i];
        const double nt = (double)n + pn;
        const double rt = (double)(long long)R[i] * kRewardInv + pn * pm;
        const double m = nt > 0.0 ? rt / nt : NAN;
        double u;
        const bool valid = nalive[cl] > 0u;
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
    if ((tid & 63) == 0) { redv[tid >> 6] = bu; redi[tid >> 6] = bf; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w) {
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

}  // namespace

hipError_t launch_ucb(const kb_batch& b, const UcbCall& c, hipStream_t st) {
    UcbArgs a;
    a.G = b.G; a.S = b.S; a.Ksum = b.Ksum; a.Kmax = b.Kmax > 0 ? b.Kmax : 1; a.N = b.N;
    a.seg_off = b.seg_off; a.koff = b.koff; a.assign = c.assign; a.alive = c.alive;
    a.bound = c.bound; a.visits = c.visits; a.rsum = c.rsum; a.t = c.t; a.c = c.c;
    a.prior_n = c.prior_n; a.prior_mu = c.prior_mu; a.Ncs = c.Ncs; a.mu = c.mu; a.ucb = c.ucb;
    a.sel = c.sel; a.order = c.order;
    const size_t lds = 64 + (size_t)a.Kmax * b.S * 12 + (size_t)a.Kmax * 12;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ucb_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ucb_kernel, dim3((unsigned)b.G), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}

}  // namespace kb
