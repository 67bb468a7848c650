// Draw of k_t inside the chosen cluster (Sec. 3.4; Alg. 1 "Sample k_t"):
// P(k) proportional to exp(V(k)/tau) over the alive members of cluster I_t, with
// V the candidate's remaining headroom.  The draw is a deterministic argmax: the
// Gumbel-max identity turns the softmax into argmax_k (V(k)/tau - ln(-ln u_k)),
// and u_k comes from the counter-based generator Philox4x32-10 (Salmon, Moraes,
// Dror, Shaw, SC'11) keyed by the seed and addressed by (candidate, draw), so
// a draw depends on nothing but its arguments.
//
// One pass over assign (and over alive / bound of the members only).  The
// candidate axis is cut into flat ranges of kSampleRange candidates, one workgroup
// each; a workgroup walks the searches that intersect its range.  A search that
// lies inside one range is finished there.  A search that crosses range borders
// leaves one partial (key, index) per range in the workspace - the piece that
// starts before the range in its "left" slot, the piece that starts inside and
// runs past the end in its "right" slot - and sample_final merges the slots of
// each such search in index order.  Keys are fp64 and compared exactly, lowest
// index on ties, so the result does not depend on the cutting.
#include "kb_internal.h"
#include "kb_rng_dev.h"

namespace kb {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kNone = 0x7fffffff;
// Searches of at most short_n candidates are drawn by one wave each (sample_wave).  In a
// batch of many searches (1024 candidates or fewer on average, so that a range of the
// range kernels holds several) that is 4096: a lane then walks up to 64 candidates,
// reading 4 bytes of each and a little more of the chosen cluster's members.  Measured:
// 1024 searches of 512 candidates 36 -> 12 us, the largest benchmark (64-4096) 41 -> 23
// us against the range kernels; at 16384 a batch of 64 searches of that length went 27 ->
// 198 us.  In a batch of few long searches a wave per search is the slower way (8
// searches of 4000: 27 -> 44 us) and the limit stays at kShortSearch.
constexpr int kSampleShortMany = 4096;
static int sample_short(const kb_batch& b) {
    return b.N <= (int64_t)1024 * b.G ? kSampleShortMany : kShortSearch;
}

struct SampleArgs {
    int G, Ksum;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const int32_t* assign;
    const uint8_t* alive;      // may be NULL: every candidate alive
    const float* bound;
    const float* incumbent;
    const int32_t* sel;        // [G,3]
    // paper-form potential (mode 1): V = theta_sat - h[k, target[S*]]
    const float* h;
    const int32_t* target;
    int R, S, mode;
    float theta_sat;
    unsigned seed_lo, seed_hi, draw_lo, draw_hi;
    double tau;
    int32_t* ksel;             // [G]
    double* slot_key;          // [2 * ranges]  left slot of range r at 2r, right slot at 2r+1
    int32_t* slot_idx;         // [2 * ranges]
    int short_n;               // sample_short() of the batch
    int mixed;                 // 1: searches of at most short_n candidates go to sample_wave, longer
                               //    ones to the range kernels, in the same call
};

// (key, index) pairs ordered by larger key, then lower index; index kNone = empty
__device__ __forceinline__ bool better(double ka, int ia, double kb_, int ib) {
    return ia != kNone && (ib == kNone || ka > kb_ || (ka == kb_ && ia < ib));
}

__device__ __forceinline__ double sample_key(const SampleArgs& a, int k, double pot_scale,
                                             int tcol) {
    double V;
    if (a.mode == 0) {
        V = 1.0 - (double)a.bound[k] / pot_scale;
    } else {
        V = (double)a.theta_sat - (double)a.h[(size_t)k * a.R + tcol];
    }
    return V / a.tau + gumbel_variate(a.seed_lo, a.seed_hi, a.draw_lo, a.draw_hi, k);
}

__global__ void __launch_bounds__(kThreads) sample_range(SampleArgs a) {
    __shared__ double redk[kWaves];
    __shared__ int redi[kWaves];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.x * kSampleRange;
    if (r0 >= a.N) return;
    const int64_t r1 = r0 + kSampleRange < a.N ? r0 + kSampleRange : a.N;
    if (tid == 0) {
        a.slot_idx[2 * (size_t)blockIdx.x] = kNone;
        a.slot_idx[2 * (size_t)blockIdx.x + 1] = kNone;
    }
    // largest g with seg_off[g] <= r0
    int lo = 0, hi = a.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.seg_off[mid] <= r0) lo = mid; else hi = mid;
    }
    const auto mine = [&](int n0, int ng, int k0, int K) {
        return n0 >= r1 || (ng > 0 && !(a.mixed && ng <= a.short_n));
    };
    for (int g = lo; (g = next_search(a.seg_off, a.koff, g, a.G, a.N, a.Ksum, mine)) < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (n0 >= r1) break;
        if (ng <= 0) continue;
        if (a.mixed && ng <= a.short_n) continue;      // (uniform) a wave of sample_wave takes this search
        const int n1 = n0 + ng;
        const int q0 = r0 > n0 ? (int)r0 : n0;
        const int q1 = r1 < n1 ? (int)r1 : n1;
        if (q0 >= q1) continue;
        const int I = a.sel[(size_t)g * 3];
        double bk = 0.0;
        int bi = kNone;
        if (I >= 0) {
            double pot_scale = 1.0;
            int tcol = 0;
            if (a.mode == 0) {
                pot_scale = (double)a.incumbent[g];
            } else {
                const int s = clampi(a.sel[(size_t)g * 3 + 1], 0, a.S - 1);
                tcol = clampi(a.target[s], 0, a.R - 1);
            }
            constexpr int U = 4;
            for (int pb = q0 + tid; pb < q1; pb += kThreads * U) {
                int jj[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int p = pb + u * kThreads;
                    jj[u] = p < q1 ? a.assign[p] : -1;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int p = pb + u * kThreads;
                    if (jj[u] != I) continue;
                    if (a.alive && !a.alive[p]) continue;
                    const double key = sample_key(a, p, pot_scale, tcol);
                    if (better(key, p, bk, bi)) { bk = key; bi = p; }
                }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double ok = __shfl_xor(bk, o);
                const int oi = __shfl_xor(bi, o);
                if (better(ok, oi, bk, bi)) { bk = ok; bi = oi; }
            }
            if ((tid & 63) == 0) { redk[tid >> 6] = bk; redi[tid >> 6] = bi; }
            __syncthreads();
            if (tid == 0) {
                for (int w = 1; w < kWaves; ++w)
                    if (better(redk[w], redi[w], bk, bi)) { bk = redk[w]; bi = redi[w]; }
            }
        }
        if (tid == 0) {
            if (n0 >= r0 && n1 <= r1) {
                a.ksel[g] = bi == kNone ? -1 : bi;
            } else {
                const size_t slot = 2 * (size_t)blockIdx.x + (n0 < r0 ? 0 : 1);
                a.slot_key[slot] = bk;
                a.slot_idx[slot] = bi;
            }
        }
        __syncthreads();
    }
}

// One thread per search: searches without candidates get -1; searches that
// cross range borders merge their slots in increasing range order.
__global__ void __launch_bounds__(kThreads) sample_final(SampleArgs a) {
    const int g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= a.G) return;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (ng <= 0) { a.ksel[g] = -1; return; }
    if (a.mixed && ng <= a.short_n) return;
    const int rf = n0 / kSampleRange, rl = (n0 + ng - 1) / kSampleRange;
    if (rf == rl) return;
    double bk = a.slot_key[2 * (size_t)rf + 1];
    int bi = a.slot_idx[2 * (size_t)rf + 1];
    for (int r = rf + 1; r <= rl; ++r) {
        const double ok = a.slot_key[2 * (size_t)r];
        const int oi = a.slot_idx[2 * (size_t)r];
        if (better(ok, oi, bk, bi)) { bk = ok; bi = oi; }
    }
    a.ksel[g] = bi == kNone ? -1 : bi;
}

// Batches of short searches: one wave per search, four searches per workgroup, one
// launch.  (A workgroup of sample_range walks the searches of its range one after
// the other, a barrier per search; with a few dozen candidates per search that is
// hundreds of searches in a row.)  Same keys, same exact comparison, so the same draw.
__global__ void __launch_bounds__(kThreads) sample_wave(SampleArgs a) {
    const int lane = threadIdx.x & 63;
    const int g = (int)blockIdx.x * kWaves + (int)(threadIdx.x >> 6);
    if (g >= a.G) return;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (ng <= 0) {
        if (lane == 0) a.ksel[g] = -1;
        return;
    }
    if (a.mixed && ng > a.short_n) return;         // the range kernels take this search
    const int I = a.sel[(size_t)g * 3];
    double bk = 0.0;
    int bi = kNone;
    if (I >= 0) {
        double pot_scale = 1.0;
        int tcol = 0;
        if (a.mode == 0) {
            pot_scale = (double)a.incumbent[g];
        } else {
            const int s = clampi(a.sel[(size_t)g * 3 + 1], 0, a.S - 1);
            tcol = clampi(a.target[s], 0, a.R - 1);
        }
        for (int p = n0 + lane; p < n0 + ng; p += kWave) {
            if (a.assign[p] != I) continue;
            if (a.alive && !a.alive[p]) continue;
            const double key = sample_key(a, p, pot_scale, tcol);
            if (better(key, p, bk, bi)) { bk = key; bi = p; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double ok = __shfl_xor(bk, o);
            const int oi = __shfl_xor(bi, o);
            if (better(ok, oi, bk, bi)) { bk = ok; bi = oi; }
        }
    }
    if (lane == 0) a.ksel[g] = bi == kNone ? -1 : bi;
}

}  // namespace

hipError_t launch_sample(const kb_batch& b, const SampleCall& c, hipStream_t st) {
    SampleArgs a;
    a.G = b.G; a.Ksum = b.Ksum; a.N = b.N; a.seg_off = b.seg_off; a.koff = b.koff;
    a.assign = c.assign; a.alive = c.alive; a.bound = c.bound; a.incumbent = c.incumbent;
    a.sel = c.sel; a.h = c.h; a.target = c.target; a.R = c.R; a.S = b.S; a.mode = c.h ? 1 : 0;
    a.theta_sat = c.theta_sat;
    a.seed_lo = (unsigned)c.seed; a.seed_hi = (unsigned)(c.seed >> 32);
    a.draw_lo = (unsigned)c.draw; a.draw_hi = (unsigned)(c.draw >> 32);
    a.tau = (double)c.tau;
    a.ksel = c.ksel; a.slot_key = c.slot_key; a.slot_idx = c.slot_idx;
    // a batch of short searches only: a wave per search, one launch; a batch of several
    // searches with longer ones among them: both kernels, each skipping the other's searches
    // (an empty launch of the other kernel costs a few microseconds)
    a.short_n = sample_short(b);
    a.mixed = b.Nmax > a.short_n && b.G > 1;
    if ((b.Nmax <= a.short_n || a.mixed) && b.G > 0) {
        hipLaunchKernelGGL(sample_wave, dim3((unsigned)((b.G + kWaves - 1) / kWaves)), dim3(kThreads), 0, st, a);
        if (!a.mixed) return hipGetLastError();
    }
    const unsigned ranges = (unsigned)((b.N + kSampleRange - 1) / kSampleRange);
    if (ranges) hipLaunchKernelGGL(sample_range, dim3(ranges), dim3(kThreads), 0, st, a);
    hipLaunchKernelGGL(sample_final, dim3((unsigned)((b.G + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace kb
