// K-Means (Lloyd) clustering of the behavioural feature vectors (Sec. 3.3;
// L2 norm of Assumption 2 / Eq. 3): one workgroup owns one search and runs all
// of its Lloyd steps, so the search's rows stay in L2 / Infinity Cache between
// steps and the centroids never leave LDS.
//
// One step is three phases separated by workgroup barriers:
//
//   A  score   fast fp32 scores s_j = |c_j|^2 - 2 x.c_j for every centroid, the
//              best and second-best per candidate, and a proved error bound E.
//              If second - best > 2E the winner is certain; otherwise the
//              candidate is marked for exact re-evaluation.
//   R  refine  marked candidates get their squared distances in fp64, direct
//              difference form, summed over the features in index order with
//              separate multiply and add - exactly the plain definition - and
//              the lowest index attaining the minimum wins.
//   B  update  only candidates whose cluster changed touch the running sums:
//              their features are converted to 64-bit fixed point and moved
//              from the old to the new cluster with integer LDS atomics.
//              Integer addition commutes, so the sums (and with them the new
//              centroids) do not depend on the order the waves run in: results
//              are bit-identical from run to run without any sorting.
//
// New centroid = (fixed-point sum / 2^shift) / count in fp64, rounded once to
// fp32; an empty cluster keeps its centroid.
#include "kb_internal.h"

namespace kb {

namespace {

struct ClusterArgs {
    int G, D, Ksum, Kmax;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const float* X;
    const float* cent_init;
    int iters;
    int early_exit;
    int32_t* assign;
    float* cent_out;
    int32_t* counts;
    float* objective;
    int32_t* a_new;
    const int32_t* order;
};

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kFlagBit = (int)0x80000000u;

__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Block-wide reductions over kThreads threads.  `red` is LDS scratch of at
// least kWaves doubles.  Both end with every thread holding the result and
// with a barrier behind them, and combine the per-wave values in a fixed order.
__device__ __forceinline__ float block_max_f(float v, double* red) {
    v = wave_max_f(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) reinterpret_cast<float*>(red)[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = reinterpret_cast<float*>(red)[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = fmaxf(r, reinterpret_cast<float*>(red)[w]);
    __syncthreads();
    return r;
}
__device__ __forceinline__ double block_sum_d(double v, double* red) {
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = red[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r += red[w];
    __syncthreads();
    return r;
}
__device__ __forceinline__ int block_or_i(int v, double* red) {
    v = __any(v) ? 1 : 0;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) reinterpret_cast<int*>(red)[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) r |= reinterpret_cast<int*>(red)[w];
    __syncthreads();
    return r;
}

// ---- phase A, vector-ALU scorer ---------------------------------------------
// One candidate per lane with its (zero-padded) feature row in registers; the
// centroids are broadcast from LDS.  Error bound of a score, with u = 2^-24,
// dot accumulated by a chain of D fused multiply-adds and s = fma(-2, dot, cn):
//   |s' - s| <= (D + 3) u (1 + o(1)) (|x|^2 + max_j |c_j|^2)
// (2 gamma_D |x||c| <= gamma_D (|x|^2+|c|^2) for the dot, u(|c|^2 + 2|x||c|) for
// the final rounding, u |c|^2 for the rounded norm).  kappa = (D + 4) u leaves
// room for the rounding of |x|^2, of E itself and of the gap.
template <int DV4>
__device__ __forceinline__ void score_valu(const ClusterArgs& a, const float* __restrict__ Xg,
                                           int n0, int ng, int K, int D, int DP,
                                           const float* cent, const float* cn, float cnmax) {
    const float kappa = (float)(D + 4) * 5.9604644775390625e-08f;
    const bool vec = (D & 3) == 0;
    for (int p = threadIdx.x; p < ng; p += kThreads) {
        float x[4 * DV4];
        const float* xr = Xg + (size_t)p * D;
        if (vec) {
#pragma unroll
            for (int c = 0; c < DV4; ++c) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (4 * c < D) v = reinterpret_cast<const float4*>(xr)[c];
                x[4 * c] = v.x; x[4 * c + 1] = v.y; x[4 * c + 2] = v.z; x[4 * c + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int d = 0; d < 4 * DV4; ++d) x[d] = d < D ? xr[d] : 0.f;
        }
        float xn = 0.f;
#pragma unroll
        for (int d = 0; d < 4 * DV4; ++d) xn = fmaf(x[d], x[d], xn);
        float best = INFINITY, second = INFINITY;
        int bi = 0;
        for (int j = 0; j < K; ++j) {
            const float4* cr = reinterpret_cast<const float4*>(cent + (size_t)j * DP);
            float d0 = 0.f, d1 = 0.f;
#pragma unroll
            for (int c = 0; c < DV4; ++c) {
                const float4 cv = cr[c];
                d0 = fmaf(x[4 * c], cv.x, d0);
                d1 = fmaf(x[4 * c + 1], cv.y, d1);
                d0 = fmaf(x[4 * c + 2], cv.z, d0);
                d1 = fmaf(x[4 * c + 3], cv.w, d1);
            }
            const float s = fmaf(-2.f, d0 + d1, cn[j]);
            const bool lt = s < best;
            second = lt ? best : fminf(second, s);
            bi = lt ? j : bi;
            best = lt ? s : best;
        }
        const float E = kappa * (xn + cnmax);
        const bool certain = (K == 1) || ((second - best) > 2.f * E);
        a.a_new[(size_t)n0 + p] = certain ? bi : (bi | kFlagBit);
    }
}

// ---- phase R -----------------------------------------------------------------
// Exact nearest centroid of the marked candidates: lanes take centroids, each
// lane sums (x_d - c_d)^2 over d in index order in fp64 with separate multiply
// and add; the wave then reduces to the minimum, lowest index on ties.
__device__ __forceinline__ void refine(const ClusterArgs& a, const float* __restrict__ Xg, int n0,
                                       int ng, int K, int D, int DP, const float* cent) {
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    for (int base = wid * kWave; base < ng; base += kThreads) {
        const int p = base + lane;
        const int v = p < ng ? a.a_new[(size_t)n0 + p] : 0;
        unsigned long long mask = __ballot(v < 0);
        while (mask) {
            const int b = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const float* xr = Xg + (size_t)(base + b) * D;
            double bd = INFINITY;
            int bj = 0x7fffffff;
            for (int j = lane; j < K; j += kWave) {
                const float* cr = cent + (size_t)j * DP;
                double acc = 0.0;
                for (int d = 0; d < D; ++d) {
                    const double diff = __dsub_rn((double)xr[d], (double)cr[d]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                }
                if (acc < bd) { bd = acc; bj = j; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double od = __shfl_xor(bd, o);
                const int oj = __shfl_xor(bj, o);
                if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
            }
            if (lane == 0) a.a_new[(size_t)n0 + base + b] = bj < K ? bj : 0;
        }
    }
}

// ---- phase B -----------------------------------------------------------------
// Move every candidate whose cluster changed: lanes take features, one
// candidate at a time, so the atomics of one instruction hit consecutive LDS
// addresses.  Returns whether this thread's wave saw any change.
__device__ __forceinline__ int update(const ClusterArgs& a, const float* __restrict__ Xg, int n0,
                                      int ng, int K, int D, bool first, double scale,
                                      long long* sums, int* cnt) {
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    int any = 0;
    for (int base = wid * kWave; base < ng; base += kThreads) {
        const int p = base + lane;
        int na = 0, oa = -1;
        bool chg = false;
        if (p < ng) {
            na = a.a_new[(size_t)n0 + p];
            na = (na >= 0 && na < K) ? na : 0;
            oa = first ? -1 : a.assign[(size_t)n0 + p];
            oa = oa < K ? oa : -1;
            chg = na != oa;
            if (chg) a.assign[(size_t)n0 + p] = na;
        }
        unsigned long long mask = __ballot(chg);
        any |= mask != 0;
        while (mask) {
            const int b = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const int nb = __shfl(na, b);
            const int ob = __shfl(oa, b);
            const float* xr = Xg + (size_t)(base + b) * D;
            for (int d = lane; d < D; d += kWave) {
                const long long q = __double2ll_rn((double)xr[d] * scale);
                atomicAdd(reinterpret_cast<unsigned long long*>(&sums[(size_t)nb * D + d]),
                          (unsigned long long)q);
                if (ob >= 0)
                    atomicAdd(reinterpret_cast<unsigned long long*>(&sums[(size_t)ob * D + d]),
                              (unsigned long long)(-q));
            }
            if (lane == 0) {
                atomicAdd(&cnt[nb], 1);
                if (ob >= 0) atomicSub(&cnt[ob], 1);
            }
        }
    }
    return any;
}

template <int DV4>
__global__ void __launch_bounds__(kThreads) cluster_fused_kernel(ClusterArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int D = a.D;
    const int DP = 4 * DV4 + 4;

    int g = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;
    g = clampi(g, 0, a.G - 1);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;   // LDS is sized from the host copy of Kmax
    if (ng <= 0 || K <= 0) {
        if (tid == 0 && a.iters > 0 && a.objective) a.objective[g] = 0.f;
        return;
    }

    double* red = reinterpret_cast<double*>(smem);                       // 16 doubles
    long long* sums = reinterpret_cast<long long*>(smem + 128);          // [Kmax][D]
    float* cent = reinterpret_cast<float*>(sums + (((size_t)a.Kmax * D + 1) & ~(size_t)1));  // [Kmax][DP], 16-byte aligned
    float* cn = cent + (size_t)a.Kmax * DP;                              // [Kmax]
    int* cnt = reinterpret_cast<int*>(cn + a.Kmax);                      // [Kmax]

    const float* Xg = a.X + (size_t)n0 * D;

    for (int idx = tid; idx < K * DP; idx += kThreads) {
        const int j = idx / DP, d = idx - j * DP;
        float v = 0.f;
        if (d < D)
            v = a.cent_init ? a.cent_init[(size_t)(k0 + j) * D + d]
                            : Xg[(size_t)(j < ng ? j : ng - 1) * D + d];
        cent[idx] = v;
    }
    for (int idx = tid; idx < K * D; idx += kThreads) sums[idx] = 0;
    for (int j = tid; j < K; j += kThreads) cnt[j] = 0;
    __syncthreads();

    if (a.iters == 0) {
        for (int idx = tid; idx < K * D; idx += kThreads) {
            const int j = idx / D, d = idx - j * D;
            a.cent_out[(size_t)(k0 + j) * D + d] = cent[(size_t)j * DP + d];
        }
        return;
    }

    // fixed-point scale: |x| < 2^e, N_g < 2^bits  =>  |sum of q| < 2^62
    float am = 0.f;
    {
        const size_t total = (size_t)ng * D;
        for (size_t i = tid; i < total; i += kThreads) am = fmaxf(am, fabsf(Xg[i]));
    }
    am = block_max_f(am, red);
    int e = 0;
    if (am > 0.f) (void)frexpf(am, &e);
    e = clampi(e, -126, 129);
    const int sh = 62 - e - (32 - __clz(ng));
    const double scale = ldexp(1.0, sh);
    const double inv = ldexp(1.0, -sh);

    bool first = true;
    for (int it = 0; it < a.iters; ++it) {
        float cm = 0.f;
        for (int j = tid; j < K; j += kThreads) {
            double s = 0.0;
            for (int d = 0; d < D; ++d) {
                const double c = (double)cent[(size_t)j * DP + d];
                s += c * c;
            }
            const float f = (float)s;
            cn[j] = f;
            cm = fmaxf(cm, f);
        }
        cm = block_max_f(cm, red);

        score_valu<DV4>(a, Xg, n0, ng, K, D, DP, cent, cn, cm);
        __syncthreads();
        refine(a, Xg, n0, ng, K, D, DP, cent);
        __syncthreads();
        const int changed = block_or_i(update(a, Xg, n0, ng, K, D, first, scale, sums, cnt), red);
        first = false;

        const bool last = (it == a.iters - 1) || (a.early_exit && !changed);
        if (last) {
            // objective relative to the centroids that entered this step
            double acc = 0.0;
            for (int p = tid; p < ng; p += kThreads) {
                int j = a.assign[(size_t)n0 + p];
                j = (j >= 0 && j < K) ? j : 0;
                const float* xr = Xg + (size_t)p * D;
                const float* cr = cent + (size_t)j * DP;
                double s = 0.0;
                for (int d = 0; d < D; ++d) {
                    const double diff = (double)xr[d] - (double)cr[d];
                    s += diff * diff;
                }
                acc += s;
            }
            acc = block_sum_d(acc, red);
            if (tid == 0) a.objective[g] = (float)acc;
        }
        for (int idx = tid; idx < K * D; idx += kThreads) {
            const int j = idx / D, d = idx - j * D;
            const int c = cnt[j];
            if (c > 0) cent[(size_t)j * DP + d] = (float)(((double)sums[idx] * inv) / (double)c);
        }
        __syncthreads();
        if (last) break;
    }

    for (int idx = tid; idx < K * D; idx += kThreads) {
        const int j = idx / D, d = idx - j * D;
        a.cent_out[(size_t)(k0 + j) * D + d] = cent[(size_t)j * DP + d];
    }
    for (int j = tid; j < K; j += kThreads) a.counts[k0 + j] = cnt[j];
}

constexpr size_t kMaxLds = 160 * 1024;

size_t fused_lds_bytes(int Kmax, int D, int DP) {
    return 128 + (((size_t)Kmax * D + 1) & ~(size_t)1) * 8 + (size_t)Kmax * DP * 4 + (size_t)Kmax * 8;
}

}  // namespace

bool cluster_supported(const kb_batch& b) {
    const int kmax = b.Kmax > 0 ? b.Kmax : 1;
    const int dv4 = (b.D + 15) / 16 * 4;
    return fused_lds_bytes(kmax, b.D, 4 * dv4 + 4) <= kMaxLds;
}

hipError_t launch_cluster(const kb_batch& b, const ClusterCall& c, hipStream_t st) {
    ClusterArgs a;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.Kmax = b.Kmax > 0 ? b.Kmax : 1; a.N = b.N;
    a.seg_off = b.seg_off; a.koff = b.koff; a.X = c.X; a.cent_init = c.cent_init;
    a.iters = c.iters; a.early_exit = 0; a.assign = c.assign; a.cent_out = c.cent_out;
    a.counts = c.counts; a.objective = c.objective; a.a_new = c.a_new; a.order = c.order;

    const int dv4 = (b.D + 15) / 16 * 4;   // 4, 8, 12 or 16 float4 chunks
    const size_t lds = fused_lds_bytes(a.Kmax, b.D, 4 * dv4 + 4);
    if (lds > kMaxLds) return hipErrorInvalidValue;
    const dim3 grid((unsigned)b.G), block(kThreads);
#define KB_LAUNCH(DV)                                                                          \
    do {                                                                                       \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(cluster_fused_kernel<DV>), \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                         \
        hipLaunchKernelGGL(cluster_fused_kernel<DV>, grid, block, lds, st, a);                 \
    } while (0)
    switch (dv4) {
        case 4: KB_LAUNCH(4); break;
        case 8: KB_LAUNCH(8); break;
        case 12: KB_LAUNCH(12); break;
        default: KB_LAUNCH(16); break;
    }
#undef KB_LAUNCH
    return hipGetLastError();
}

}  // namespace kb
