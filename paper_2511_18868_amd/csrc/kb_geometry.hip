// Cluster representatives and radii (Sec. 3.3 "Representative profiling"; Alg. 1
// "Update centroids k_c"; covering term of Theorem 1).
//
// For every candidate the squared distance to its own centroid is formed exactly
// as the plain definition does - fp64, direct differences, summed over the
// features in index order with separate multiply and add - so the per-cluster
// minimum (the representative, lowest index on ties) and maximum (the radius)
// are exact and need no tolerance.
//
//   geo_init   per-cluster tables: min = all ones, max = 0, rep = none
//   geo_dist   one workgroup per flat range of candidates walks the searches that
//              intersect it.  Per search piece the centroids are staged in LDS;
//              tiles of 256 rows are fetched with coalesced 16-byte loads (the
//              next tile is requested before the current one is worked on),
//              transposed through LDS (padded row stride: conflict-free) so
//              that each thread owns one candidate, and the distances are reduced
//              per cluster with 64-bit integer LDS atomics on their bit patterns
//              (non-negative doubles order like unsigned integers), then merged
//              into the global tables.  The distance of every candidate is kept.
//   geo_rep    second, light pass (12 bytes per candidate): the candidates whose
//              distance equals their cluster's minimum compete for the lowest
//              index with an integer atomic min.
//   geo_final  rep = -1 for empty clusters, radius = sqrt(max) rounded to fp32.
#include "kb_internal.h"

namespace kb {

namespace {

constexpr int kThreads = 256;
constexpr int kNone = 0x7fffffff;

struct GeoArgs {
    int G, D, Ksum, Kmax;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const float* X;
    const float* cent;
    const int32_t* assign;
    int32_t* rep;
    float* radius;
    double* d2;                    // [N]
    unsigned long long* gmin;      // [Ksum]
    unsigned long long* gmax;      // [Ksum]
    int mixed;                     // 1: searches of at most kShortSearch candidates go to geo_wave, longer
                                   //    ones to the range kernels, in the same call
};

__global__ void __launch_bounds__(kThreads) geo_init(GeoArgs a) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < a.Ksum) { a.gmin[i] = ~0ull; a.gmax[i] = 0ull; a.rep[i] = kNone; }
}

// VEC = 4: D is a multiple of 4, rows are moved as 16-byte pieces; VEC = 1: any D.
template <int VEC>
__global__ void __launch_bounds__(kThreads) geo_dist(GeoArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    // row stride of the transposed tile: D + 4 words keeps 16-byte pieces aligned and
    // spreads consecutive rows over the banks (conflict-free 16-byte reads whenever
    // D/4 is even); the next odd number for the scalar path
    const int D = a.D, DP = VEC == 4 ? D + 4 : (D | 1);
    unsigned long long* lmin = reinterpret_cast<unsigned long long*>(smem);          // [Kmax]
    unsigned long long* lmax = lmin + a.Kmax;                                         // [Kmax]
    float* lc = reinterpret_cast<float*>(lmax + a.Kmax);                              // [Kmax * D]
    float* lx = lc + (size_t)a.Kmax * D;                                              // [256 * DP]

    const int64_t r0 = (int64_t)blockIdx.x * kGeoRange;
    if (r0 >= a.N) return;
    const int64_t r1 = r0 + kGeoRange < a.N ? r0 + kGeoRange : a.N;

    // position of this thread's pieces inside a tile: piece i of the thread is
    // element VEC * (tid + 256 i) of the tile = (row, col); advancing i adds
    // (qd, rd) with a carry
    constexpr int kPieces = 64 / VEC;             // D <= 64: at most D / VEC pieces per thread
    const int step = VEC * kThreads;
    const int qd = step / D, rd = step - qd * D;
    const int row0 = (VEC * tid) / D, col0 = VEC * tid - row0 * D;
    const int npieces = (D + VEC - 1) / VEC;      // pieces per thread of a full tile (D / VEC when VEC = 4)

    int lo = 0, hi = a.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.seg_off[mid] <= r0) lo = mid; else hi = mid;
    }
    const auto mine = [&](int n0, int ng, int k0, int K) {
        return n0 >= r1 || (ng > 0 && K > 0 && !(a.mixed && ng <= kShortSearch));
    };
    for (int g = lo; (g = next_search(a.seg_off, a.koff, g, a.G, a.N, a.Ksum, mine)) < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (K > a.Kmax) K = a.Kmax;
        if (n0 >= r1) break;
        if (ng <= 0 || K <= 0) continue;
        if (a.mixed && ng <= kShortSearch) continue;      // (uniform) a wave of geo_wave takes this search
        const int q0 = r0 > n0 ? (int)r0 : n0;
        const int q1 = r1 < (int64_t)n0 + ng ? (int)r1 : n0 + ng;
        if (q0 >= q1) continue;

        // centroids of the search -> LDS
        {
            const float* cg = a.cent + (size_t)k0 * D;
            const int total = K * D;
            if constexpr (VEC == 4) {
                for (int i = tid; i < total / 4; i += kThreads)
                    reinterpret_cast<float4*>(lc)[i] = reinterpret_cast<const float4*>(cg)[i];
            } else {
                for (int i = tid; i < total; i += kThreads) lc[i] = cg[i];
            }
            for (int j = tid; j < K; j += kThreads) { lmin[j] = ~0ull; lmax[j] = 0ull; }
        }

        float xr[kPieces][VEC];
        auto fetch = [&](int tb) {
            const int cnt = q1 - tb < kThreads ? q1 - tb : kThreads;
            const int total = cnt * D / VEC;       // pieces in the tile (exact: VEC divides D or is 1)
            const float* src = a.X + (size_t)tb * D;
#pragma unroll
            for (int i = 0; i < kPieces; ++i) {
                const int idx = tid + i * kThreads;
                if (i < npieces && idx < total) {
                    if constexpr (VEC == 4) {
                        const float4 v = reinterpret_cast<const float4*>(src)[idx];
                        xr[i][0] = v.x; xr[i][1] = v.y; xr[i][2] = v.z; xr[i][3] = v.w;
                    } else {
                        xr[i][0] = src[idx];
                    }
                }
            }
        };
        if constexpr (VEC == 4) fetch(q0);
        for (int tb = q0; tb < q1; tb += kThreads) {
            const int cnt = q1 - tb < kThreads ? q1 - tb : kThreads;
            const int total = cnt * D / VEC;
            if constexpr (VEC == 1) {
                // feature by feature: straight from memory into the transposed tile, eight
                // values in flight per thread (holding a whole tile's 64 values per thread
                // for the next round, as the 16-byte form does, leaves room for one
                // workgroup per compute unit only)
                const float* src = a.X + (size_t)tb * D;
                int row = row0, col = col0;
                for (int i0 = 0; i0 < npieces; i0 += 8) {
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int idx = tid + (i0 + u) * kThreads;
                        v[u] = (i0 + u < npieces && idx < total) ? src[idx] : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int idx = tid + (i0 + u) * kThreads;
                        if (i0 + u < npieces && idx < total) lx[row * DP + col] = v[u];
                        row += qd; col += rd;
                        if (col >= D) { col -= D; row += 1; }
                    }
                }
            } else
            // registers -> LDS, one row per candidate
            {
                int row = row0, col = col0;
#pragma unroll
                for (int i = 0; i < kPieces; ++i) {
                    const int idx = tid + i * kThreads;
                    if (i < npieces && idx < total) {
                        float* dst = lx + row * DP + col;
                        if constexpr (VEC == 4) {
                            *reinterpret_cast<float4*>(dst) = make_float4(xr[i][0], xr[i][1], xr[i][2], xr[i][3]);
                        } else {
                            dst[0] = xr[i][0];
                        }
                    }
                    row += qd; col += rd;
                    if (col >= D) { col -= D; row += 1; }
                }
            }
            const int p = tb + tid;
            int j = p < q1 ? a.assign[p] : 0;
            j = (j >= 0 && j < K) ? j : 0;
            __syncthreads();
            if constexpr (VEC == 4) {
                if (tb + kThreads < q1) fetch(tb + kThreads);
            }
            if (tid < cnt) {
                const float* xrow = lx + tid * DP;
                const float* crow = lc + (size_t)j * D;
                double acc = 0.0;
                if constexpr (VEC == 4) {
                    // 16-byte LDS reads, eight features in flight; the sum itself stays
                    // in index order
#pragma unroll 2
                    for (int d = 0; d < D; d += 4) {
                        const float4 xv = *reinterpret_cast<const float4*>(xrow + d);
                        const float4 cv = *reinterpret_cast<const float4*>(crow + d);
                        double diff = __dsub_rn((double)xv.x, (double)cv.x);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)xv.y, (double)cv.y);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)xv.z, (double)cv.z);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)xv.w, (double)cv.w);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    }
                } else {
                    // eight features' values requested before the first is used; the sum
                    // itself stays in index order
                    int d = 0;
                    for (; d + 8 <= D; d += 8) {
                        float xv[8], cv[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) { xv[u] = xrow[d + u]; cv[u] = crow[d + u]; }
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const double diff = __dsub_rn((double)xv[u], (double)cv[u]);
                            acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        }
                    }
                    for (; d < D; ++d) {
                        const double diff = __dsub_rn((double)xrow[d], (double)crow[d]);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    }
                }
                a.d2[p] = acc;
                const unsigned long long bits = (unsigned long long)__double_as_longlong(acc);
                atomicMin(&lmin[j], bits);
                atomicMax(&lmax[j], bits);
            }
            __syncthreads();
        }
        for (int j = tid; j < K; j += kThreads) {
            if (lmin[j] != ~0ull) {
                atomicMin(&a.gmin[k0 + j], lmin[j]);
                atomicMax(&a.gmax[k0 + j], lmax[j]);
            }
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(kThreads) geo_rep(GeoArgs a) {
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.x * kGeoRange;
    if (r0 >= a.N) return;
    const int64_t r1 = r0 + kGeoRange < a.N ? r0 + kGeoRange : a.N;
    int lo = 0, hi = a.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.seg_off[mid] <= r0) lo = mid; else hi = mid;
    }
    const auto mine = [&](int n0, int ng, int k0, int K) {
        return n0 >= r1 || (ng > 0 && K > 0 && !(a.mixed && ng <= kShortSearch));
    };
    for (int g = lo; (g = next_search(a.seg_off, a.koff, g, a.G, a.N, a.Ksum, mine)) < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (K > a.Kmax) K = a.Kmax;
        if (n0 >= r1) break;
        if (ng <= 0 || K <= 0) continue;
        if (a.mixed && ng <= kShortSearch) continue;
        const int q0 = r0 > n0 ? (int)r0 : n0;
        const int q1 = r1 < (int64_t)n0 + ng ? (int)r1 : n0 + ng;
        for (int p = q0 + tid; p < q1; p += kThreads) {
            int j = a.assign[p];
            j = (j >= 0 && j < K) ? j : 0;
            const unsigned long long bits = (unsigned long long)__double_as_longlong(a.d2[p]);
            if (bits == a.gmin[k0 + j]) atomicMin(&a.rep[k0 + j], p);
        }
    }
}

__global__ void __launch_bounds__(kThreads) geo_final(GeoArgs a) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= a.Ksum) return;
    if (a.rep[i] == kNone) a.rep[i] = -1;
    a.radius[i] = (float)sqrt(__longlong_as_double((long long)a.gmax[i]));
}

// Batches of short searches: one wave per search, four searches per workgroup, the
// whole pass in one launch.  (A workgroup of the range kernels above walks the
// searches of its range one after the other with barriers around each; with a few
// dozen candidates per search that is hundreds of searches in a row.)  Same distances
// - the same fp64 operations in the same order - and the same exact comparisons, so
// the same representatives and radii.  Any search length is handled (the distances
// wait in d2 between the two sweeps); short ones are what it is launched for.
template <int VEC>
__global__ void __launch_bounds__(kThreads) geo_wave(GeoArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = (int)blockIdx.x * (kThreads / kWave) + wv;
    if (g >= a.G) return;                 // (a whole wave leaves: no wave waits for another in this kernel)
    const int D = a.D;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (K <= 0) return;
    if (a.mixed && ng > kShortSearch) return;         // the range kernels take this search
    unsigned long long* lmin = reinterpret_cast<unsigned long long*>(smem) + (size_t)wv * 2 * a.Kmax;   // [Kmax]
    unsigned long long* lmax = lmin + a.Kmax;                                                            // [Kmax]
    int* lrep = reinterpret_cast<int*>(smem + (size_t)(kThreads / kWave) * 16 * a.Kmax) + (size_t)wv * a.Kmax;   // [Kmax]
    for (int j = lane; j < K; j += kWave) { lmin[j] = ~0ull; lmax[j] = 0ull; lrep[j] = kNone; }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    for (int p = n0 + lane; p < n0 + ng; p += kWave) {
        int j = a.assign[p];
        j = (j >= 0 && j < K) ? j : 0;
        const float* xrow = a.X + (size_t)p * D;
        const float* crow = a.cent + (size_t)(k0 + j) * D;
        double acc = 0.0;
        if constexpr (VEC == 4) {
            for (int d = 0; d < D; d += 4) {
                const float4 xv = *reinterpret_cast<const float4*>(xrow + d);
                const float4 cv = *reinterpret_cast<const float4*>(crow + d);
                double diff = __dsub_rn((double)xv.x, (double)cv.x);
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                diff = __dsub_rn((double)xv.y, (double)cv.y);
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                diff = __dsub_rn((double)xv.z, (double)cv.z);
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                diff = __dsub_rn((double)xv.w, (double)cv.w);
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
            }
        } else {
            for (int d = 0; d < D; ++d) {
                const double diff = __dsub_rn((double)xrow[d], (double)crow[d]);
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
            }
        }
        a.d2[p] = acc;
        const unsigned long long bits = (unsigned long long)__double_as_longlong(acc);
        atomicMin(&lmin[j], bits);
        atomicMax(&lmax[j], bits);
    }
    // (a lane reads back only the distances it wrote itself)
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    for (int p = n0 + lane; p < n0 + ng; p += kWave) {
        int j = a.assign[p];
        j = (j >= 0 && j < K) ? j : 0;
        const unsigned long long bits = (unsigned long long)__double_as_longlong(a.d2[p]);
        if (bits == lmin[j]) atomicMin(&lrep[j], p);
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    for (int j = lane; j < K; j += kWave) {
        if (a.mixed) {
            // geo_final finishes every cluster of the batch from the global tables
            a.rep[k0 + j] = lrep[j];
            a.gmax[k0 + j] = lmax[j];
        } else {
            a.rep[k0 + j] = lrep[j] == kNone ? -1 : lrep[j];
            a.radius[k0 + j] = (float)sqrt(__longlong_as_double((long long)lmax[j]));
        }
    }
}

}  // namespace

size_t geometry_lds_bytes(int Kmax, int D) {
    return (size_t)16 * Kmax + (size_t)4 * Kmax * D + (size_t)4 * kThreads * (D + 4);
}

hipError_t launch_geometry(const kb_batch& b, const GeoCall& c, hipStream_t st) {
    GeoArgs a;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.Kmax = b.Kmax > 0 ? b.Kmax : 1; a.N = b.N;
    a.seg_off = b.seg_off; a.koff = b.koff; a.X = c.X; a.cent = c.cent; a.assign = c.assign;
    a.rep = c.rep; a.radius = c.radius; a.d2 = c.d2; a.gmin = c.gmin; a.gmax = c.gmax;
    if (b.Ksum <= 0) return hipSuccess;
    // a batch of short searches only: a wave per search, one launch; a batch of mostly
    // short searches (256 candidates or fewer on average) with longer ones among them: the
    // wave kernel after the tables are initialised, then the range kernels, each skipping
    // the other's searches.  (Where short searches are the exception the range kernels
    // take them in passing: on the largest benchmark the extra launch cost more than it saved.)
    a.mixed = b.Nmax > kShortSearch && b.G > 1 && b.N <= (int64_t)kShortSearch * b.G;
    const size_t wlds = (size_t)(kThreads / kWave) * 20 * a.Kmax;
    const dim3 wgrid((unsigned)((b.G + kThreads / kWave - 1) / (kThreads / kWave)));
    if (wlds > 64 * 1024) return hipErrorInvalidValue;
    if (b.Nmax <= kShortSearch && b.G > 0) {
        if ((b.D & 3) == 0) hipLaunchKernelGGL(geo_wave<4>, wgrid, dim3(kThreads), wlds, st, a);
        else hipLaunchKernelGGL(geo_wave<1>, wgrid, dim3(kThreads), wlds, st, a);
        return hipGetLastError();
    }
    const unsigned kblocks = (unsigned)((b.Ksum + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(geo_init, dim3(kblocks), dim3(kThreads), 0, st, a);
    if (a.mixed) {
        if ((b.D & 3) == 0) hipLaunchKernelGGL(geo_wave<4>, wgrid, dim3(kThreads), wlds, st, a);
        else hipLaunchKernelGGL(geo_wave<1>, wgrid, dim3(kThreads), wlds, st, a);
    }
    const unsigned ranges = (unsigned)((b.N + kGeoRange - 1) / kGeoRange);
    if (ranges) {
        const size_t lds = geometry_lds_bytes(a.Kmax, b.D);
        if (lds > 160 * 1024) return hipErrorInvalidValue;
        if ((b.D & 3) == 0) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(geo_dist<4>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(geo_dist<4>, dim3(ranges), dim3(kThreads), lds, st, a);
        } else {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(geo_dist<1>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(geo_dist<1>, dim3(ranges), dim3(kThreads), lds, st, a);
        }
        hipLaunchKernelGGL(geo_rep, dim3(ranges), dim3(kThreads), 0, st, a);
    }
    hipLaunchKernelGGL(geo_final, dim3(kblocks), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace kb
