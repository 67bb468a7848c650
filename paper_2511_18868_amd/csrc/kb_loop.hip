// The small steps that close the loop of Alg. 1 around the scoring pass:
// the strategy mask in the paper's own form (Eq. 5) and the statistics update
// that ends an iteration.  Both touch a few bytes per cluster arm or per search.
#include "kb_internal.h"

namespace kb {

namespace {

constexpr int kThreads = 256;

// M[i,s] = [ h(rep_i)[target(s)] < theta_sat ], one wave per search; nvalid[g] =
// number of valid cluster arms of the search.
__global__ void __launch_bounds__(kThreads)
strategy_mask_kernel(int G, int S, int R, int Ksum, int64_t N, const int32_t* __restrict__ koff,
                     const float* __restrict__ h, const int32_t* __restrict__ target,
                     const int32_t* __restrict__ rep, float theta_sat, uint8_t* __restrict__ M,
                     int32_t* __restrict__ nvalid) {
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6);
    if (g >= G) return;
    const int k0 = clampi(koff[g], 0, Ksum);
    const int k1 = clampi(koff[g + 1], k0, Ksum);
    const int arms = (k1 - k0) * S;
    int n = 0;
    for (int q = lane; q < arms; q += kWave) {
        const int i = k0 + q / S, s = q - (q / S) * S;
        const int r = rep[i];
        int m = 0;
        if (r >= 0 && (int64_t)r < N) {
            const int col = clampi(target[s], 0, R - 1);
            m = h[(size_t)r * R + col] < theta_sat ? 1 : 0;
        }
        M[(size_t)k0 * S + q] = (uint8_t)m;
        n += m;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o);
    if (lane == 0) nvalid[g] = n;
}

// One thread per search.  Searches own disjoint cluster arms and candidates, so
// the read-modify-write steps need no atomics.
__global__ void __launch_bounds__(kThreads)
update_stats_kernel(int G, int S, int Ksum, int64_t N, const int32_t* __restrict__ seg_off,
                    const int32_t* __restrict__ koff, const int32_t* __restrict__ sel,
                    const int32_t* __restrict__ ksel, const float* __restrict__ reward,
                    const uint8_t* __restrict__ ok, double prior_n, int32_t* __restrict__ visits,
                    float* __restrict__ rsum, int32_t* __restrict__ Ncs, float* __restrict__ mu,
                    int64_t* __restrict__ t, const int32_t* __restrict__ assign,
                    const uint8_t* __restrict__ alive, unsigned* __restrict__ gN,
                    unsigned long long* __restrict__ gR) {
    const int g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= G) return;
    t[g] += 1;
    int n0, ng, k0, K;
    search_bounds(seg_off, koff, g, N, Ksum, n0, ng, k0, K);
    const int I = sel[(size_t)g * 3], s = sel[(size_t)g * 3 + 1], k = ksel[g];
    if (!ok[g] || I < 0 || I >= K || s < 0 || s >= S || k < n0 || k >= n0 + ng) return;
    const size_t arm = ((size_t)k0 + I) * S + s;
    const int nn = Ncs[arm] + 1;
    Ncs[arm] = nn;
    const double r = (double)reward[g];
    const double m = (double)mu[arm];
    mu[arm] = (float)(m + (r - m) / ((double)nn + prior_n));
    const size_t cell = (size_t)k * S + s;
    visits[cell] += 1;
    const float r_old = rsum[cell];
    const float r_new = (float)((double)r_old + r);
    rsum[cell] = r_new;
    if (gN && (!alive || alive[k])) {
        // the tables an aggregation over the alive candidates would now give: one more
        // visit and the change of this cell's fixed-point image, in the candidate's cluster
        int j = assign[k];
        j = (j >= 0 && j < K) ? j : 0;
        const size_t tarm = ((size_t)k0 + j) * S + s;
        gN[tarm] += 1u;
        gR[tarm] += reward_fixed(r_new) - reward_fixed(r_old);
    }
}

}  // namespace

hipError_t launch_strategy_mask(const kb_batch& b, int R, const float* h, const int32_t* target,
                                const int32_t* rep, float theta_sat, uint8_t* M, int32_t* nvalid,
                                hipStream_t st) {
    const int per = kThreads / kWave;
    hipLaunchKernelGGL(strategy_mask_kernel, dim3((unsigned)((b.G + per - 1) / per)), dim3(kThreads),
                       0, st, b.G, b.S, R, b.Ksum, b.N, b.koff, h, target, rep, theta_sat, M, nvalid);
    return hipGetLastError();
}

hipError_t launch_update_stats(const kb_batch& b, float prior_n, const int32_t* sel,
                               const int32_t* ksel, const float* reward, const uint8_t* ok,
                               int32_t* visits, float* rsum, int32_t* Ncs, float* mu, int64_t* t,
                               hipStream_t st, const int32_t* assign, const uint8_t* alive,
                               unsigned* gN, unsigned long long* gR) {
    if (gN && (!gR || !assign)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(update_stats_kernel, dim3((unsigned)((b.G + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, b.G, b.S, b.Ksum, b.N, b.seg_off, b.koff, sel, ksel,
                       reward, ok, (double)prior_n, visits, rsum, Ncs, mu, t, assign, alive, gN, gR);
    return hipGetLastError();
}

}  // namespace kb
