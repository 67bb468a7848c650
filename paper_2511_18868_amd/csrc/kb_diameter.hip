// Cluster diameters: diam(C_i) = the largest distance between two members of
// cluster i, the quantity in the approximation term L * max_i diam(C_i) of
// Theorem 1.
//
//   dia_zero     per-cluster counters and maxima <- 0
//   dia_hist     cluster sizes: flat candidate ranges walk the searches that
//                intersect them, LDS histogram per search piece, one global atomic
//                per touched cluster and piece
//   dia_bsum / dia_bscan / dia_apply
//                exclusive prefix sums of the sizes and of the tile counts,
//                counters reset
//   dia_scatter  candidate indices grouped by cluster (same walk; a piece reserves
//                its slots per cluster with one global atomic, positions inside the
//                piece come from LDS atomics).  The order inside a cluster varies
//                from run to run; the maximum over its pairs does not.
//   dia_pairs    the tiles of 64 x 64 member pairs of all clusters (32 x 32 for
//                clusters of up to 32 members) are numbered in one sequence and
//                every workgroup takes an equal share; a thread owns 4 x 4 (2 x 2)
//                pairs of a tile, features pass through LDS 16 at a time; squared
//                distances from direct differences in fp32 (relative error at most
//                (D + 2) 2^-24 each, being sums of non-negative terms)
//   dia_final    square root
#include "kb_internal.h"

namespace kb {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kRange = 4096;     // candidates per workgroup of the histogram / scatter walks
constexpr int kDiaShort = 64;    // searches of at most this many candidates: all pairs by one wave (dia_wave);
                                 // beyond, a lane's loop over the later members gets long (a search of 256
                                 // candidates took 0.34 ms that way against 0.03 ms through the tiles)

struct DiaArgs {
    int G, D, Ksum, Kmax;
    int64_t N;
    const int32_t* seg_off;
    const int32_t* koff;
    const float* X;
    const int32_t* assign;
    float* diam;          // [Ksum] out
    int32_t* cnt;         // [Ksum] sizes, then cursors
    int32_t* off;         // [Ksum + 1] first slot of every cluster in perm
    int32_t* toff;        // [Ksum + 1] first tile of every cluster in the global tile numbering
    long long* bsum;      // [2 * blocks of the prefix sum] (members, tiles) per block
    unsigned* dmax;       // [Ksum] bits of the largest squared distance (aliases diam)
    int32_t* perm;        // [N]
    int mixed;            // 1: searches of at most kDiaShort candidates go to dia_wave, longer ones
                          //    through the grouping and the pair tiles, in the same call
};

__global__ void __launch_bounds__(kThreads) dia_zero(DiaArgs a) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < a.Ksum) { a.cnt[i] = 0; a.dmax[i] = 0u; }
}

// SCATTER = false: sizes; true: grouped indices
template <bool SCATTER>
__global__ void __launch_bounds__(kThreads) dia_walk(DiaArgs a) {
    __shared__ int lcnt[KB_MAX_K];
    __shared__ int lbase[KB_MAX_K];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.x * kRange;
    if (r0 >= a.N) return;
    const int64_t r1 = r0 + kRange < a.N ? r0 + kRange : a.N;
    int lo = 0, hi = a.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.seg_off[mid] <= r0) lo = mid; else hi = mid;
    }
    const auto mine = [&](int n0, int ng, int k0, int K) {
        return n0 >= r1 || (ng > 0 && K > 0 && !(a.mixed && ng <= kDiaShort));
    };
    for (int g = lo; (g = next_search(a.seg_off, a.koff, g, a.G, a.N, a.Ksum, mine)) < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (K > KB_MAX_K) K = KB_MAX_K;
        if (n0 >= r1) break;
        if (ng <= 0 || K <= 0) continue;
        if (a.mixed && ng <= kDiaShort) continue;         // (uniform) a wave of dia_wave takes this search:
                                                          // its clusters keep size 0 here and get no tiles
        const int q0 = r0 > n0 ? (int)r0 : n0;
        const int q1 = r1 < (int64_t)n0 + ng ? (int)r1 : n0 + ng;
        if (q0 >= q1) continue;
        for (int j = tid; j < K; j += kThreads) lcnt[j] = 0;
        __syncthreads();
        for (int p = q0 + tid; p < q1; p += kThreads) {
            int j = a.assign[p];
            j = (j >= 0 && j < K) ? j : 0;
            atomicAdd(&lcnt[j], 1);
        }
        __syncthreads();
        if (!SCATTER) {
            for (int j = tid; j < K; j += kThreads)
                if (lcnt[j]) atomicAdd(&a.cnt[k0 + j], lcnt[j]);
        } else {
            for (int j = tid; j < K; j += kThreads) {
                lbase[j] = lcnt[j] ? a.off[k0 + j] + atomicAdd(&a.cnt[k0 + j], lcnt[j]) : 0;
                lcnt[j] = 0;
            }
            __syncthreads();
            for (int p = q0 + tid; p < q1; p += kThreads) {
                int j = a.assign[p];
                j = (j >= 0 && j < K) ? j : 0;
                const int64_t pos = (int64_t)lbase[j] + atomicAdd(&lcnt[j], 1);
                if (pos >= 0 && pos < a.N) a.perm[pos] = p;
            }
        }
        __syncthreads();
    }
}

// Tiles of member pairs of a cluster of n members: none below two members, one tile
// of 32 x 32 up to 32 members, otherwise the tiles of 64 x 64 on and above the diagonal.
__device__ __forceinline__ long long tiles_of(int n) {
    if (n < 2) return 0;
    if (n <= 32) return 1;
    const long long T = (n + 63) >> 6;
    return T * (T + 1) / 2;
}

// off = exclusive prefix sum of cnt, toff = that of the tile counts, cnt <- 0, in
// three launches with coalesced accesses: sums of blocks of kScanBlock entries,
// their prefix sums (one workgroup), then the entries of every block.
constexpr int kScanBlock = 4096;
constexpr int kScanU = kScanBlock / kThreads;

// (members, tiles) summed over the workgroup; every thread gets the result
__device__ __forceinline__ void block_sum2(long long& m, long long& t, long long* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { m += __shfl_xor(m, o); t += __shfl_xor(t, o); }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { red[2 * (threadIdx.x >> 6)] = m; red[2 * (threadIdx.x >> 6) + 1] = t; }
    __syncthreads();
    m = 0; t = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) { m += red[2 * w]; t += red[2 * w + 1]; }
}

__global__ void __launch_bounds__(kThreads) dia_bsum(DiaArgs a) {
    __shared__ long long red[2 * kWaves];
    const int i0 = blockIdx.x * kScanBlock + threadIdx.x;
    long long m = 0, t = 0;
#pragma unroll
    for (int u = 0; u < kScanU; ++u) {
        const int i = i0 + u * kThreads;
        const int v = i < a.Ksum ? a.cnt[i] : 0;
        m += v;
        t += tiles_of(v);
    }
    block_sum2(m, t, red);
    if (threadIdx.x == 0) { a.bsum[2 * blockIdx.x] = m; a.bsum[2 * blockIdx.x + 1] = t; }
}

// exclusive prefix sums of the block sums, in place; one workgroup, blocks in order
__global__ void __launch_bounds__(kThreads) dia_bscan(DiaArgs a, int nblocks) {
    __shared__ long long red[2 * kWaves];
    __shared__ long long carry[2];
    const int tid = threadIdx.x;
    if (tid == 0) { carry[0] = 0; carry[1] = 0; }
    __syncthreads();
    for (int b0 = 0; b0 < nblocks; b0 += kThreads) {
        const int b = b0 + tid;
        const long long m = b < nblocks ? a.bsum[2 * b] : 0, t = b < nblocks ? a.bsum[2 * b + 1] : 0;
        // inclusive scan over the workgroup: inside the waves, then over the wave totals
        long long im = m, it = t;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const long long um = __shfl_up(im, o), ut = __shfl_up(it, o);
            if ((tid & 63) >= o) { im += um; it += ut; }
        }
        if ((tid & 63) == 63) { red[2 * (tid >> 6)] = im; red[2 * (tid >> 6) + 1] = it; }
        __syncthreads();
        long long pm = carry[0], pt = carry[1];
        for (int w = 0; w < (tid >> 6); ++w) { pm += red[2 * w]; pt += red[2 * w + 1]; }
        if (b < nblocks) { a.bsum[2 * b] = pm + im - m; a.bsum[2 * b + 1] = pt + it - t; }
        __syncthreads();
        if (tid == kThreads - 1) { carry[0] = pm + im; carry[1] = pt + it; }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(kThreads) dia_apply(DiaArgs a) {
    __shared__ long long red[2 * kWaves];
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kScanBlock + tid;
    int v[kScanU];
#pragma unroll
    for (int u = 0; u < kScanU; ++u) {
        const int i = i0 + u * kThreads;
        v[u] = i < a.Ksum ? a.cnt[i] : 0;
    }
    long long cm = a.bsum[2 * blockIdx.x], ct = a.bsum[2 * blockIdx.x + 1];
    const long long tcap = 0x7fffffffll;
    // entries i0 + u * 256: one pass of the workgroup per u keeps the index order
#pragma unroll
    for (int u = 0; u < kScanU; ++u) {
        const int i = i0 + u * kThreads;
        const long long m = v[u], t = tiles_of(v[u]);
        long long im = m, it = t;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const long long um = __shfl_up(im, o), ut = __shfl_up(it, o);
            if ((tid & 63) >= o) { im += um; it += ut; }
        }
        __syncthreads();
        if ((tid & 63) == 63) { red[2 * (tid >> 6)] = im; red[2 * (tid >> 6) + 1] = it; }
        __syncthreads();
        long long pm = cm, pt = ct, tm = 0, tt = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (w < (tid >> 6)) { pm += red[2 * w]; pt += red[2 * w + 1]; }
            tm += red[2 * w]; tt += red[2 * w + 1];
        }
        if (i < a.Ksum) {
            const long long om = pm + im - m, ot = pt + it - t;
            a.off[i] = (int)(om < a.N ? om : a.N);
            a.toff[i] = (int)(ot < tcap ? ot : tcap);
            a.cnt[i] = 0;
            if (i == a.Ksum - 1) {
                a.off[a.Ksum] = (int)(om + m < a.N ? om + m : a.N);
                a.toff[a.Ksum] = (int)(ot + t < tcap ? ot + t : tcap);
            }
        }
        cm += tm; ct += tt;
    }
}

// Squared distances of a tile of T x T member pairs, T = 16 * R: the 256 threads
// form a 16 x 16 grid and each owns R x R pairs.  Features pass through LDS 16 at
// a time, feature-major, so that a thread reads its R rows' and R columns' values
// of one feature with one LDS read each and spends R * R subtract / multiply-add
// pairs on them.  Rows beyond the cluster are replaced by its last member, whose
// distances are genuine ones, so nothing needs masking.
template <int R>
__device__ __forceinline__ float tile_pairs_max(const DiaArgs& a, int base, int n, int ta, int tb,
                                                float* As, float* Bs) {
    constexpr int T = 16 * R;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int D = a.D;
    float acc[R][R];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int j = 0; j < R; ++j) acc[i][j] = 0.f;
    // loader: thread -> (row of the tile, group of features); T rows x 16 features per
    // side and step = T * 16 values, 256 threads -> T / 16 = R values each
    const int lrow = tid % T, lf0 = (tid / T) * R;        // R consecutive features of one row
    int ia = ta * T + lrow, ib = tb * T + lrow;
    ia = ia < n ? ia : n - 1;
    ib = ib < n ? ib : n - 1;
    int ra = a.perm[base + ia], rb = a.perm[base + ib];
    ra = (ra >= 0 && ra < a.N) ? ra : 0;
    rb = (rb >= 0 && rb < a.N) ? rb : 0;
    const float* xa = a.X + (size_t)ra * D;
    const float* xb = a.X + (size_t)rb * D;
    const bool vec = (D & 3) == 0 && R == 4;     // the R = 4 features of a thread are one 16-byte piece
    float va[R], vb[R];
    auto fetch = [&](int d0) {
        if (vec) {
            const int d = d0 + lf0;
            const float4 pa = d < D ? *reinterpret_cast<const float4*>(xa + d) : make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 pb = d < D ? *reinterpret_cast<const float4*>(xb + d) : make_float4(0.f, 0.f, 0.f, 0.f);
            va[0] = pa.x; va[1 % R] = pa.y; va[2 % R] = pa.z; va[3 % R] = pa.w;
            vb[0] = pb.x; vb[1 % R] = pb.y; vb[2 % R] = pb.z; vb[3 % R] = pb.w;
        } else {
#pragma unroll
            for (int e = 0; e < R; ++e) {
                const int d = d0 + lf0 + e;
                va[e] = d < D ? xa[d] : 0.f;
                vb[e] = d < D ? xb[d] : 0.f;
            }
        }
    };
    fetch(0);
    for (int d0 = 0; d0 < D; d0 += 16) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < R; ++e) {
            As[(lf0 + e) * T + lrow] = va[e];
            Bs[(lf0 + e) * T + lrow] = vb[e];
        }
        __syncthreads();
        if (d0 + 16 < D) fetch(d0 + 16);      // the next step's values travel while this one is worked on
#pragma unroll
        for (int f = 0; f < 16; ++f) {
            float av[R], bv[R];
#pragma unroll
            for (int i = 0; i < R; ++i) av[i] = As[f * T + ty * R + i];
#pragma unroll
            for (int j = 0; j < R; ++j) bv[j] = Bs[f * T + tx * R + j];
#pragma unroll
            for (int i = 0; i < R; ++i)
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const float e = av[i] - bv[j];
                    acc[i][j] = fmaf(e, e, acc[i][j]);
                }
        }
    }
    float far = 0.f;
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int j = 0; j < R; ++j) far = fmaxf(far, acc[i][j]);
    return far;
}

// All tiles of all clusters are numbered in one sequence (toff); every workgroup
// takes an equal, contiguous share of the numbers, so the work is balanced
// whatever the cluster sizes are.  The maximum of a run of tiles of one cluster
// goes to the cluster's maximum with an integer atomic max on the float's bits
// (non-negative floats order like their bit patterns).
__global__ void __launch_bounds__(kThreads) dia_pairs(DiaArgs a) {
    __shared__ __align__(16) float As[16 * 64];
    __shared__ __align__(16) float Bs[16 * 64];
    __shared__ float redm[kWaves];
    const int tid = threadIdx.x;
    const long long total = a.toff[a.Ksum];
    const long long per = (total + gridDim.x - 1) / gridDim.x;
    long long t = per * blockIdx.x;
    const long long t1 = t + per < total ? t + per : total;
    if (t >= t1) return;
    // cluster of the first tile: the last c with toff[c] <= t
    int c = 0;
    {
        int lo = 0, hi = a.Ksum;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long long)a.toff[mid] <= t) lo = mid; else hi = mid;
        }
        c = lo;
    }
    auto flush = [&](int cid, float far) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) far = fmaxf(far, __shfl_xor(far, o));
        __syncthreads();
        if ((tid & 63) == 0) redm[tid >> 6] = far;
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kWaves; ++w) far = fmaxf(far, redm[w]);
            if (far > 0.f) atomicMax(&a.dmax[cid], __float_as_uint(far));
        }
    };
    while (t < t1) {
        while (c + 1 < a.Ksum && (long long)a.toff[c + 1] <= t) ++c;      // skips clusters without tiles
        const int base = a.off[c];
        const int n = a.off[c + 1] - base;
        const long long tend = (long long)a.toff[c + 1] < t1 ? (long long)a.toff[c + 1] : t1;
        if (base < 0 || n < 2 || (long long)base + n > a.N || tend <= t) { t = tend > t ? tend : t + 1; continue; }
        float far = 0.f;
        if (n <= 32) {
            far = tile_pairs_max<2>(a, base, n, 0, 0, As, Bs);
            ++t;
        } else {
            // tiles of the cluster are numbered row by row over the upper triangle
            const int T = (n + 63) >> 6;
            int ta = 0;
            long long rem = t - a.toff[c];
            while (ta < T && rem >= T - ta) { rem -= T - ta; ++ta; }
            for (; t < tend && ta < T; ++t) {
                far = fmaxf(far, tile_pairs_max<4>(a, base, n, ta, ta + (int)rem, As, Bs));
                if (++rem >= T - ta) { rem = 0; ++ta; }
            }
            if (ta >= T) t = tend;
        }
        flush(c, far);
    }
}

// Short searches: one wave per search, four searches per workgroup.  (The walks above
// take the searches of a range one after the other with barriers around each, and the
// grouping, the prefix sums and the tile numbering are seven launches: 0.34 ms for 183
// searches of a few dozen candidates.)  Lane l takes candidates l, l + 64, ... and
// compares each with the later members of its cluster; a pair's squared distance is
// the same chain of fused multiply-adds over the features in index order as in the
// tiles above, so the maxima are the same bits.
__global__ void __launch_bounds__(kThreads) dia_wave(DiaArgs a) {
    extern __shared__ unsigned wmax[];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = (int)blockIdx.x * kWaves + wv;
    if (g >= a.G) return;                 // (a whole wave leaves: no wave waits for another in this kernel)
    const int D = a.D;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (K <= 0) return;
    if (a.mixed && ng > kDiaShort) return;            // the tile kernels take this search
    unsigned* lmax = wmax + (size_t)wv * a.Kmax;      // [Kmax] bits of the largest squared distance
    for (int j = lane; j < K; j += kWave) lmax[j] = 0u;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    const bool vec = (D & 3) == 0;
    for (int p = lane; p < ng; p += kWave) {
        int jp = a.assign[(size_t)n0 + p];
        jp = (jp >= 0 && jp < K) ? jp : 0;
        const float* xp = a.X + ((size_t)n0 + p) * D;
        float far = 0.f;
        for (int q = p + 1; q < ng; ++q) {
            int jq = a.assign[(size_t)n0 + q];
            jq = (jq >= 0 && jq < K) ? jq : 0;
            if (jq != jp) continue;
            const float* xq = a.X + ((size_t)n0 + q) * D;
            float acc = 0.f;
            if (vec) {
                for (int d = 0; d < D; d += 4) {
                    const float4 u = *reinterpret_cast<const float4*>(xp + d);
                    const float4 v = *reinterpret_cast<const float4*>(xq + d);
                    float e = u.x - v.x; acc = fmaf(e, e, acc);
                    e = u.y - v.y; acc = fmaf(e, e, acc);
                    e = u.z - v.z; acc = fmaf(e, e, acc);
                    e = u.w - v.w; acc = fmaf(e, e, acc);
                }
            } else {
                for (int d = 0; d < D; ++d) {
                    const float e = xp[d] - xq[d];
                    acc = fmaf(e, e, acc);
                }
            }
            far = fmaxf(far, acc);
        }
        if (far > 0.f) atomicMax(&lmax[jp], __float_as_uint(far));
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    for (int j = lane; j < K; j += kWave) {
        if (a.mixed) a.dmax[k0 + j] = lmax[j];        // dia_final takes the root of every cluster
        else a.diam[k0 + j] = sqrtf(__uint_as_float(lmax[j]));
    }
}

__global__ void __launch_bounds__(kThreads) dia_final(DiaArgs a) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < a.Ksum) a.diam[i] = sqrtf(__uint_as_float(a.dmax[i]));
}

}  // namespace

hipError_t launch_diameter(const kb_batch& b, const DiameterCall& c, hipStream_t st) {
    if (b.Ksum <= 0) return hipSuccess;
    DiaArgs a;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.Kmax = b.Kmax > 0 ? b.Kmax : 1; a.N = b.N;
    a.seg_off = b.seg_off; a.koff = b.koff; a.X = c.X; a.assign = c.assign; a.diam = c.diam;
    a.cnt = c.cnt; a.off = c.off; a.toff = c.toff; a.bsum = c.bsum; a.dmax = reinterpret_cast<unsigned*>(c.diam); a.perm = c.perm;
    const unsigned kblocks = (unsigned)((b.Ksum + kThreads - 1) / kThreads);
    const unsigned ranges = (unsigned)((b.N + kRange - 1) / kRange);
    // a batch of short searches only: a wave per search, one launch; a batch of mostly
    // short searches (256 candidates or fewer on average) with longer ones among them: the
    // wave kernel after the maxima are zeroed, then the grouping and the tiles, which leave
    // the short searches out
    a.mixed = b.Nmax > kDiaShort && b.G > 1 && b.N <= (int64_t)kShortSearch * b.G;
    const size_t wlds = (size_t)kWaves * 4 * (b.Kmax > 0 ? b.Kmax : 1);
    const dim3 wgrid((unsigned)((b.G + kWaves - 1) / kWaves));
    if (b.Nmax <= kDiaShort && b.G > 0) {
        hipLaunchKernelGGL(dia_wave, wgrid, dim3(kThreads), wlds, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(dia_zero, dim3(kblocks), dim3(kThreads), 0, st, a);
    if (a.mixed) hipLaunchKernelGGL(dia_wave, wgrid, dim3(kThreads), wlds, st, a);
    if (ranges) hipLaunchKernelGGL(dia_walk<false>, dim3(ranges), dim3(kThreads), 0, st, a);
    const int nscan = (b.Ksum + kScanBlock - 1) / kScanBlock;
    hipLaunchKernelGGL(dia_bsum, dim3((unsigned)nscan), dim3(kThreads), 0, st, a);
    hipLaunchKernelGGL(dia_bscan, dim3(1), dim3(kThreads), 0, st, a, nscan);
    hipLaunchKernelGGL(dia_apply, dim3((unsigned)nscan), dim3(kThreads), 0, st, a);
    if (ranges) hipLaunchKernelGGL(dia_walk<true>, dim3(ranges), dim3(kThreads), 0, st, a);
    // enough workgroups to fill the chip several times over; each takes an equal share of
    // the tiles, whose number is only known on the device
    hipLaunchKernelGGL(dia_pairs, dim3(8192), dim3(kThreads), 0, st, a);
    hipLaunchKernelGGL(dia_final, dim3(kblocks), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace kb
