// Farthest-point initial centroids (greedy cover of a search's frontier): the
// first centroid is the search's first row, every further one the candidate
// farthest from the centroids chosen so far.  The largest cluster radius of this
// cover is within a factor two of the smallest possible one - the covering
// radius that the approximation term of Theorem 1 is linear in.
//
// One workgroup per search, K_g passes over the search's rows.  A thread owns the
// rows tid, tid + 512, ... (four of them in flight at a time); per pass it forms each row's squared distance to the
// newest centroid exactly as the plain definition does (fp64, direct
// differences, summed over the features in index order with separate multiply and
// add), lowers the row's running minimum (kept in the workspace) and remembers
// its largest; the workgroup reduces to the maximum with the lowest index on
// ties.  Distances are exact, so the choice needs no tolerance.
#include "kb_internal.h"
#include "kb_rng_dev.h"

namespace kb {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;

struct SeedArgs {
    int G, D, Ksum;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const float* X;
    float* cent;
    int32_t* pick;       // may be NULL
    double* mind;        // [N] running minimum of every candidate
    const int32_t* order;
    // randomised (D^2-weighted) seeding instead of the farthest point
    int dsquared;
    unsigned seed_lo, seed_hi;
    unsigned long long draw0;
};

__global__ void __launch_bounds__(kThreads) seed_farthest_kernel(SeedArgs a) {
    __shared__ __align__(16) float c[KB_MAX_D];
    __shared__ double redv[kWaves];
    __shared__ int redi[kWaves];
    __shared__ int chosen_s;
    const int tid = threadIdx.x;
    const int D = a.D;
    const bool vec = (D & 3) == 0;
    int g = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;
    g = clampi(g, 0, a.G - 1);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (ng <= 0 || K <= 0) return;
    const float* Xg = a.X + (size_t)n0 * D;
    double* mind = a.mind + n0;
    // largest (value, lowest index) of the workgroup; every thread returns the index
    auto block_argmax = [&](double far, int arg) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double of = __shfl_xor(far, o);
            const int oa = __shfl_xor(arg, o);
            if (of > far || (of == far && oa < arg)) { far = of; arg = oa; }
        }
        if ((tid & 63) == 0) { redv[tid >> 6] = far; redi[tid >> 6] = arg; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kWaves; ++w)
                if (redv[w] > far || (redv[w] == far && redi[w] < arg)) { far = redv[w]; arg = redi[w]; }
            chosen_s = (arg >= 0 && arg < ng) ? arg : 0;
        }
        __syncthreads();
        return chosen_s;
    };
    int chosen = 0;
    if (a.dsquared) {
        // first centroid: a uniform draw, i.e. the largest variate of draw number draw0
        double far = -INFINITY;
        int arg = 0x7fffffff;
        for (int k = tid; k < ng; k += kThreads) {
            const double key = gumbel_variate(a.seed_lo, a.seed_hi, (unsigned)a.draw0,
                                              (unsigned)(a.draw0 >> 32), n0 + k);
            if (key > far || (key == far && k < arg)) { far = key; arg = k; }
        }
        chosen = block_argmax(far, arg);
    }
    for (int j = 0; j < K; ++j) {
        // what the next centroid maximises: the running minimum itself (farthest
        // point), or ln(minimum) plus the variate of draw number draw0 + j + 1 (a draw
        // with probability proportional to the minimum)
        const unsigned long long drawn = a.draw0 + (unsigned long long)j + 1ull;
        const bool need_key = a.dsquared && j + 1 < K;
        if (tid < D) {
            const float v = Xg[(size_t)chosen * D + tid];
            c[tid] = v;
            a.cent[((size_t)k0 + j) * D + tid] = v;
        }
        if (tid == 0 && a.pick) a.pick[k0 + j] = n0 + chosen;
        __syncthreads();
        double far = -INFINITY;
        int arg = 0x7fffffff;
        constexpr int U = 4;      // rows in flight per thread
        for (int kb = tid; kb < ng; kb += U * kThreads) {
            double acc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = 0.0;
            if (vec) {
                // 16 features of each of the U rows are requested together; the sum of a
                // row still runs over its features in index order
                for (int d0 = 0; d0 < D; d0 += 16) {
                    float4 xv[U][4];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int k = kb + u * kThreads;
                        const float* xr = Xg + (size_t)(k < ng ? k : kb) * D + d0;
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            xv[u][q] = d0 + 4 * q < D ? *reinterpret_cast<const float4*>(xr + 4 * q)
                                                      : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (d0 + 4 * q < D) {
                            const float4 cv = *reinterpret_cast<const float4*>(c + d0 + 4 * q);
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                double diff = __dsub_rn((double)xv[u][q].x, (double)cv.x);
                                acc[u] = __dadd_rn(acc[u], __dmul_rn(diff, diff));
                                diff = __dsub_rn((double)xv[u][q].y, (double)cv.y);
                                acc[u] = __dadd_rn(acc[u], __dmul_rn(diff, diff));
                                diff = __dsub_rn((double)xv[u][q].z, (double)cv.z);
                                acc[u] = __dadd_rn(acc[u], __dmul_rn(diff, diff));
                                diff = __dsub_rn((double)xv[u][q].w, (double)cv.w);
                                acc[u] = __dadd_rn(acc[u], __dmul_rn(diff, diff));
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = kb + u * kThreads;
                    const float* xr = Xg + (size_t)(k < ng ? k : kb) * D;
                    for (int d = 0; d < D; ++d) {
                        const double diff = __dsub_rn((double)xr[d], (double)c[d]);
                        acc[u] = __dadd_rn(acc[u], __dmul_rn(diff, diff));
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = kb + u * kThreads;
                if (k < ng) {
                    double mk = acc[u];
                    if (j > 0) {
                        const double old = mind[k];
                        mk = old < acc[u] ? old : acc[u];
                    }
                    mind[k] = mk;
                    double v = mk;
                    if (a.dsquared)
                        v = need_key ? log(mk) + gumbel_variate(a.seed_lo, a.seed_hi, (unsigned)drawn,
                                                                (unsigned)(drawn >> 32), n0 + k)
                                     : 0.0;
                    if (v > far || (v == far && k < arg)) { far = v; arg = k; }
                }
            }
        }
        chosen = block_argmax(far, arg);
    }
}

}  // namespace

hipError_t launch_seed(const kb_batch& b, const float* X, float* cent, int32_t* pick, double* mind,
                       const int32_t* order, int dsquared, uint64_t seed, uint64_t draw0,
                       hipStream_t st) {
    SeedArgs a;
    a.dsquared = dsquared; a.seed_lo = (unsigned)seed; a.seed_hi = (unsigned)(seed >> 32);
    a.draw0 = draw0;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.N = b.N; a.seg_off = b.seg_off; a.koff = b.koff;
    a.X = X; a.cent = cent; a.pick = pick; a.mind = mind; a.order = order;
    hipLaunchKernelGGL(seed_farthest_kernel, dim3((unsigned)b.G), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace kb
