// Farthest-point initial centroids (greedy cover of a search's frontier): the
// first centroid is the search's first row, every further one the candidate
// farthest from the centroids chosen so far.  The largest cluster radius of this
// cover is within a factor two of the smallest possible one - the covering
// radius that the approximation term of Theorem 1 is linear in.
//
// One workgroup per search, K_g passes over the search's rows.  A thread owns the
// rows tid, tid + 512, ...  The first R of them are read once and stay in
// registers for all passes, together with their running minima (R x 512 rows,
// 2048 at 48 features: a whole search in most cases, and the workgroup then
// touches memory only for the newest centroid); rows beyond that are streamed
// again in every pass, four in flight per thread, with their minima in the
// workspace.  Per pass a row's squared distance to the newest centroid is formed
// exactly as the plain definition does (fp64, direct differences, summed over the
// features in index order with separate multiply and add); the workgroup reduces
// to the maximum with the lowest index on ties.  Distances are exact, so the
// choice needs no tolerance.
//
// Searches longer than kBigRows rows would keep one compute unit busy for K_g
// passes over memory; they take one launch per centroid instead.  The candidate
// axis is cut into flat ranges of kRange rows, one workgroup each; a workgroup
// first finds the newest centroid of its search - the best of the (key, row)
// pairs that the ranges of the previous launch left in the workspace - then does
// the pass over its own rows and leaves its pair for the next launch.  Two sets of
// pairs alternate between launches.
#include "kb_internal.h"
#include "kb_rng_dev.h"

namespace kb {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int kBigRows = 4096;     // longer searches take the launch-per-centroid path
constexpr int kRange = 1024;       // its rows per workgroup (at most kBigRows, so that a range
                                   // meets at most two long searches: one that began before
                                   // it, one that begins inside)
constexpr int kBigThreads = 256;
constexpr int kNone = 0x7fffffff;
// rows a workgroup keeps in LDS after the registers are full: padded to 16 DS + 4
// words (16-byte reads of consecutive rows fall into different banks), at most
// two per thread, within 155 KB
constexpr int lds_stride(int DS) { return 16 * DS + 4; }
constexpr int lds_rows(int DS) {
    return 158720 / (4 * lds_stride(DS)) < 2 * kThreads ? 158720 / (4 * lds_stride(DS)) : 2 * kThreads;
}

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
    // launch-per-centroid path: pair (key, row in its search) of range r, slot s
    // (0: the search that began before the range, 1: the one that begins inside),
    // set b at index (b * nranges + r) * 2 + s
    double* skey;
    int32_t* sidx;
    int nranges;
};

// exact squared difference added to a running sum, the three roundings kept apart
__device__ __forceinline__ double add_sq(double acc, float x, double c) {
    const double diff = __dsub_rn((double)x, c);
    return __dadd_rn(acc, __dmul_rn(diff, diff));
}

// DS: features padded to 16 DS (zeros add +0.0 to a sum); R: rows per thread kept in registers
template <int DS, int R, bool DSQ>
__global__ void __launch_bounds__(kThreads) seed_farthest_kernel(SeedArgs a) {
    constexpr int Q = 4 * DS;
    constexpr int RS = lds_stride(DS), LROWS = lds_rows(DS), LV = (LROWS + kThreads - 1) / kThreads;
    extern __shared__ __align__(16) float lx[];        // [LROWS][RS]
    __shared__ __align__(16) float c[16 * DS];
    __shared__ double redv[kWaves];
    __shared__ int redi[kWaves];
    const int tid = threadIdx.x;
    const int D = a.D;
    const bool vec = (D & 3) == 0;
    int g = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;
    g = clampi(g, 0, a.G - 1);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (ng <= 0 || K <= 0 || ng > kBigRows) return;
    const float* Xg = a.X + (size_t)n0 * D;
    double* mind = a.mind + n0;
    // largest (value, lowest index) of the workgroup; every thread returns the index.
    // (One barrier: every thread merges the waves' results itself.  The slots are
    // written again only after the barrier that follows the staging of the next
    // centroid, which every thread passes after it has read them.)
    auto block_argmax = [&](double far, int arg) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double of = __shfl_xor(far, o);
            const int oa = __shfl_xor(arg, o);
            if (of > far || (of == far && oa < arg)) { far = of; arg = oa; }
        }
        if ((tid & 63) == 0) { redv[tid >> 6] = far; redi[tid >> 6] = arg; }
        __syncthreads();
        far = redv[0]; arg = redi[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            const double of = redv[w];
            const int oa = redi[w];
            if (of > far || (of == far && oa < arg)) { far = of; arg = oa; }
        }
        return (arg >= 0 && arg < ng) ? arg : 0;
    };
    // what a row contributes to the choice of the next centroid: its running minimum
    // (farthest point), or ln(minimum) plus the variate of this pass's draw (a draw
    // with probability proportional to the minimum)
    auto offer = [&](double mk, int k, bool need_key, unsigned long long drawn, double& far, int& arg) {
        double v = mk;
        if constexpr (DSQ)
            v = need_key ? log(mk) + gumbel_variate(a.seed_lo, a.seed_hi, (unsigned)drawn,
                                                    (unsigned)(drawn >> 32), n0 + k)
                         : 0.0;
        if (v > far || (v == far && k < arg)) { far = v; arg = k; }
    };

    // the rows that stay in registers; `ru`: how many of them any lane of this wave has
    float4 xr[R][Q];
    double mk[R];
    int ru = 0;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        if ((tid & ~63) + u * kThreads < ng) ru = u + 1;
        const int k = tid + u * kThreads;
        const bool ex = k < ng;
        const float* row = Xg + (size_t)(ex ? k : 0) * D;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int d = 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ex && d < D) {
                if (vec) {
                    v = *reinterpret_cast<const float4*>(row + d);
                } else {
                    v.x = row[d];
                    if (d + 1 < D) v.y = row[d + 1];
                    if (d + 2 < D) v.z = row[d + 2];
                    if (d + 3 < D) v.w = row[d + 3];
                }
            }
            xr[u][q] = v;
        }
        mk[u] = INFINITY;
    }

    // the next LROWS rows go to LDS, row R * 512 + tid + 512 v to thread tid
    double ml[LV];
#pragma unroll
    for (int v = 0; v < LV; ++v) {
        const int sl = tid + v * kThreads, k = R * kThreads + sl;
        ml[v] = INFINITY;
        if (sl < LROWS && k < ng) {
            const float* row = Xg + (size_t)k * D;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int d = 4 * q;
                float4 x4 = make_float4(0.f, 0.f, 0.f, 0.f);
                if (d < D) {
                    if (vec) {
                        x4 = *reinterpret_cast<const float4*>(row + d);
                    } else {
                        x4.x = row[d];
                        if (d + 1 < D) x4.y = row[d + 1];
                        if (d + 2 < D) x4.z = row[d + 2];
                        if (d + 3 < D) x4.w = row[d + 3];
                    }
                }
                *reinterpret_cast<float4*>(lx + (size_t)sl * RS + d) = x4;
            }
        }
    }

    int chosen = 0;
    if constexpr (DSQ) {
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
        const unsigned long long drawn = a.draw0 + (unsigned long long)j + 1ull;
        const bool need_key = DSQ && j + 1 < K;
        // the chosen row becomes centroid j: out of its owner's registers, or from
        // memory if it is one of the streamed rows
        chosen = __builtin_amdgcn_readfirstlane(chosen);     // (the same in every thread)
        if (chosen < R * kThreads) {
#pragma unroll
            for (int u = 0; u < R; ++u) {
                if (u == chosen / kThreads && tid == (chosen & (kThreads - 1))) {
#pragma unroll
                    for (int q = 0; q < Q; ++q) reinterpret_cast<float4*>(c)[q] = xr[u][q];
                    if (a.pick) a.pick[k0 + j] = n0 + chosen;
                }
            }
        } else if (tid < 16 * DS) {
            c[tid] = chosen < R * kThreads + LROWS ? lx[(size_t)(chosen - R * kThreads) * RS + tid]
                     : tid < D                     ? Xg[(size_t)chosen * D + tid]
                                                   : 0.f;
            if (tid == 0 && a.pick) a.pick[k0 + j] = n0 + chosen;
        }
        __syncthreads();
        if (tid < D) a.cent[((size_t)k0 + j) * D + tid] = c[tid];
        if (j + 1 == K) break;         // the last centroid is followed by no choice
        double far = -INFINITY;
        int arg = 0x7fffffff;
        // rows in registers
        if (ru > 0) {
            double acc[R];
#pragma unroll
            for (int u = 0; u < R; ++u) acc[u] = 0.0;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (4 * q < D) {
                    const float4 cv = *reinterpret_cast<const float4*>(c + 4 * q);
                    const double cx = (double)cv.x, cy = (double)cv.y, cz = (double)cv.z, cw = (double)cv.w;
#pragma unroll
                    for (int u = 0; u < R; ++u) {
                        if (u < ru) {
                            // (opaque to the compiler, which would otherwise widen every
                            // row to fp64 once, outside the passes, at twice the registers)
                            asm volatile("" : "+v"(xr[u][q].x), "+v"(xr[u][q].y), "+v"(xr[u][q].z),
                                              "+v"(xr[u][q].w));
                            acc[u] = add_sq(acc[u], xr[u][q].x, cx);
                            acc[u] = add_sq(acc[u], xr[u][q].y, cy);
                            acc[u] = add_sq(acc[u], xr[u][q].z, cz);
                            acc[u] = add_sq(acc[u], xr[u][q].w, cw);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int k = tid + u * kThreads;
                if (k < ng) {
                    mk[u] = mk[u] < acc[u] ? mk[u] : acc[u];
                    offer(mk[u], k, need_key, drawn, far, arg);
                }
            }
        }
        // rows in LDS
        if ((tid & ~63) + R * kThreads < ng) {
            double acc[LV];
#pragma unroll
            for (int v = 0; v < LV; ++v) acc[v] = 0.0;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (4 * q < D) {
                    const float4 cv = *reinterpret_cast<const float4*>(c + 4 * q);
                    const double cx = (double)cv.x, cy = (double)cv.y, cz = (double)cv.z, cw = (double)cv.w;
#pragma unroll
                    for (int v = 0; v < LV; ++v) {
                        // (a slot beyond the search's rows is read all the same: inside the array)
                        const int sl = tid + v * kThreads < LROWS ? tid + v * kThreads : tid;
                        const float4 x4 = *reinterpret_cast<const float4*>(lx + (size_t)sl * RS + 4 * q);
                        acc[v] = add_sq(acc[v], x4.x, cx);
                        acc[v] = add_sq(acc[v], x4.y, cy);
                        acc[v] = add_sq(acc[v], x4.z, cz);
                        acc[v] = add_sq(acc[v], x4.w, cw);
                    }
                }
            }
#pragma unroll
            for (int v = 0; v < LV; ++v) {
                const int sl = tid + v * kThreads, k = R * kThreads + sl;
                if (sl < LROWS && k < ng) {
                    ml[v] = ml[v] < acc[v] ? ml[v] : acc[v];
                    offer(ml[v], k, need_key, drawn, far, arg);
                }
            }
        }
        // rows beyond the registers' and the LDS's share
        constexpr int U = 2;      // rows in flight per thread
        for (int kb = tid + R * kThreads + LROWS; kb < ng; kb += U * kThreads) {
            double acc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] = 0.0;
            if (vec) {
                // 8 features of each of the U rows are requested together; the sum of a
                // row still runs over its features in index order
                for (int d0 = 0; d0 < D; d0 += 8) {
                    float4 xv[U][2];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int k = kb + u * kThreads;
                        const float* row = Xg + (size_t)(k < ng ? k : kb) * D + d0;
#pragma unroll
                        for (int q = 0; q < 2; ++q)
                            xv[u][q] = d0 + 4 * q < D ? *reinterpret_cast<const float4*>(row + 4 * q)
                                                      : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        if (d0 + 4 * q < D) {
                            const float4 cv = *reinterpret_cast<const float4*>(c + d0 + 4 * q);
                            const double cx = (double)cv.x, cy = (double)cv.y, cz = (double)cv.z,
                                         cw = (double)cv.w;
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                acc[u] = add_sq(acc[u], xv[u][q].x, cx);
                                acc[u] = add_sq(acc[u], xv[u][q].y, cy);
                                acc[u] = add_sq(acc[u], xv[u][q].z, cz);
                                acc[u] = add_sq(acc[u], xv[u][q].w, cw);
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = kb + u * kThreads;
                    const float* row = Xg + (size_t)(k < ng ? k : kb) * D;
                    for (int d = 0; d < D; ++d) acc[u] = add_sq(acc[u], row[d], (double)c[d]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = kb + u * kThreads;
                if (k < ng) {
                    double m = acc[u];
                    if (j > 0) {
                        const double old = mind[k];
                        m = old < acc[u] ? old : acc[u];
                    }
                    mind[k] = m;
                    offer(m, k, need_key, drawn, far, arg);
                }
            }
        }
        chosen = block_argmax(far, arg);
    }
}

// One launch per centroid for the searches of more than kBigRows rows.  `j`: the
// centroid this launch places (-1: only the keys of the uniform first draw);
// `wset`: the set of pairs this launch writes, the other one holds the previous
// launch's.
template <bool DSQ>
__global__ void __launch_bounds__(kBigThreads) seed_big_pass(SeedArgs a, int j, int wset) {
    constexpr int kW = kBigThreads / kWave;
    __shared__ __align__(16) float c[KB_MAX_D];
    __shared__ double redv[kW];
    __shared__ int redi[kW];
    __shared__ int chosen_s;
    const int tid = threadIdx.x;
    const int D = a.D;
    const bool vec = (D & 3) == 0;
    const int r = blockIdx.x;
    const int64_t r0 = (int64_t)r * kRange;
    if (r >= a.nranges || r0 >= a.N) return;
    const int64_t r1 = r0 + kRange < a.N ? r0 + kRange : a.N;
    double* wkey = a.skey + ((size_t)wset * a.nranges + r) * 2;
    int32_t* widx = a.sidx + ((size_t)wset * a.nranges + r) * 2;
    const double* pkey = a.skey + (size_t)(wset ^ 1) * a.nranges * 2;
    const int32_t* pidx = a.sidx + (size_t)(wset ^ 1) * a.nranges * 2;
    if (tid == 0) { widx[0] = kNone; widx[1] = kNone; }
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
            for (int w = 1; w < kW; ++w)
                if (redv[w] > far || (redv[w] == far && redi[w] < arg)) { far = redv[w]; arg = redi[w]; }
            redv[0] = far;
            chosen_s = arg;
        }
        __syncthreads();
        const int res = chosen_s;
        return res;
    };
    // largest g with seg_off[g] <= r0
    int lo = 0, hi = a.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.seg_off[mid] <= r0) lo = mid; else hi = mid;
    }
    for (int g = lo; g < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (n0 >= r1) break;
        if (ng <= kBigRows || K <= 0 || j >= K) continue;
        const int n1 = n0 + ng;
        const int q0 = r0 > n0 ? (int)r0 : n0;
        const int q1 = r1 < n1 ? (int)r1 : n1;
        if (q0 >= q1) continue;
        const float* Xg = a.X + (size_t)n0 * D;
        double* mind = a.mind + n0;
        const int slot = n0 < r0 ? 0 : 1;
        double far = -INFINITY;
        int arg = kNone;
        if (j < 0) {
            for (int k = q0 - n0 + tid; k < q1 - n0; k += kBigThreads) {
                const double key = gumbel_variate(a.seed_lo, a.seed_hi, (unsigned)a.draw0,
                                                  (unsigned)(a.draw0 >> 32), n0 + k);
                if (key > far || (key == far && k < arg)) { far = key; arg = k; }
            }
        } else {
            int chosen = 0;
            if (DSQ || j > 0) {
                // the newest centroid: best pair of the previous launch over the search's ranges
                const int rf = n0 / kRange, rl = (n1 - 1) / kRange;
                double bk = -INFINITY;
                int bi = kNone;
                for (int q = rf + tid; q <= rl; q += kBigThreads) {
                    const int sl = n0 < q * kRange ? 0 : 1;
                    const double ok = pkey[2 * (size_t)q + sl];
                    const int oi = pidx[2 * (size_t)q + sl];
                    if (oi != kNone && (ok > bk || (ok == bk && oi < bi))) { bk = ok; bi = oi; }
                }
                chosen = block_argmax(bk, bi);
                chosen = (chosen >= 0 && chosen < ng) ? chosen : 0;
            }
            if (tid < KB_MAX_D) {
                const float v = tid < D ? Xg[(size_t)chosen * D + tid] : 0.f;
                c[tid] = v;
                if (slot == 1 && tid < D) a.cent[((size_t)k0 + j) * D + tid] = v;
            }
            if (slot == 1 && tid == 0 && a.pick) a.pick[k0 + j] = n0 + chosen;
            __syncthreads();
            if (j + 1 < K) {
                const unsigned long long drawn = a.draw0 + (unsigned long long)j + 1ull;
                constexpr int U = kRange / kBigThreads;     // this thread's rows, all in flight
                const int kb = q0 - n0 + tid, ke = q1 - n0;
                double acc[U];
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u] = 0.0;
                if (vec) {
                    for (int d0 = 0; d0 < D; d0 += 16) {
                        float4 xv[U][4];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const int k = kb + u * kBigThreads;
                            const float* row = Xg + (size_t)(k < ke ? k : q0 - n0) * D + d0;
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                xv[u][q] = d0 + 4 * q < D ? *reinterpret_cast<const float4*>(row + 4 * q)
                                                          : make_float4(0.f, 0.f, 0.f, 0.f);
                        }
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            if (d0 + 4 * q < D) {
                                const float4 cv = *reinterpret_cast<const float4*>(c + d0 + 4 * q);
                                const double cx = (double)cv.x, cy = (double)cv.y, cz = (double)cv.z,
                                             cw = (double)cv.w;
#pragma unroll
                                for (int u = 0; u < U; ++u) {
                                    acc[u] = add_sq(acc[u], xv[u][q].x, cx);
                                    acc[u] = add_sq(acc[u], xv[u][q].y, cy);
                                    acc[u] = add_sq(acc[u], xv[u][q].z, cz);
                                    acc[u] = add_sq(acc[u], xv[u][q].w, cw);
                                }
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int k = kb + u * kBigThreads;
                        const float* row = Xg + (size_t)(k < ke ? k : q0 - n0) * D;
                        for (int d = 0; d < D; ++d) acc[u] = add_sq(acc[u], row[d], (double)c[d]);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = kb + u * kBigThreads;
                    if (k < ke) {
                        double m = acc[u];
                        if (j > 0) {
                            const double old = mind[k];
                            m = old < acc[u] ? old : acc[u];
                        }
                        mind[k] = m;
                        double v = m;
                        if constexpr (DSQ)
                            v = log(m) + gumbel_variate(a.seed_lo, a.seed_hi, (unsigned)drawn,
                                                        (unsigned)(drawn >> 32), n0 + k);
                        if (v > far || (v == far && k < arg)) { far = v; arg = k; }
                    }
                }
            }
        }
        arg = block_argmax(far, arg);
        if (tid == 0) { wkey[slot] = redv[0]; widx[slot] = arg; }
        __syncthreads();
    }
}

}  // namespace

size_t seed_ranges(const kb_batch& b) { return (size_t)((b.N + kRange - 1) / kRange) + 1; }

hipError_t launch_seed(const kb_batch& b, const float* X, float* cent, int32_t* pick, double* mind,
                       double* skey, int32_t* sidx, const int32_t* order, int dsquared,
                       uint64_t seed, uint64_t draw0, hipStream_t st) {
    SeedArgs a;
    a.dsquared = dsquared; a.seed_lo = (unsigned)seed; a.seed_hi = (unsigned)(seed >> 32);
    a.draw0 = draw0;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.N = b.N; a.seg_off = b.seg_off; a.koff = b.koff;
    a.X = X; a.cent = cent; a.pick = pick; a.mind = mind; a.order = order;
    a.skey = skey; a.sidx = sidx; a.nranges = (int)seed_ranges(b);
    const dim3 grid((unsigned)b.G), block(kThreads);
    hipError_t err = hipSuccess;
    auto go = [&](auto far, auto dsq, int DS) {
        const size_t lds = (size_t)4 * lds_stride(DS) * lds_rows(DS);
        auto kern = dsquared ? dsq : far;
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (err == hipSuccess) hipLaunchKernelGGL(kern, grid, block, lds, st, a);
    };
    if (b.D <= 16) go(seed_farthest_kernel<1, 8, false>, seed_farthest_kernel<1, 8, true>, 1);
    else if (b.D <= 32) go(seed_farthest_kernel<2, 6, false>, seed_farthest_kernel<2, 6, true>, 2);
    else if (b.D <= 48) go(seed_farthest_kernel<3, 4, false>, seed_farthest_kernel<3, 4, true>, 3);
    else go(seed_farthest_kernel<4, 3, false>, seed_farthest_kernel<4, 3, true>, 4);
    if (err != hipSuccess) return err;
    if (b.Nmax > kBigRows) {
        const dim3 bgrid((unsigned)a.nranges), bblock(kBigThreads);
        int launches = 0;
        if (dsquared) hipLaunchKernelGGL(seed_big_pass<true>, bgrid, bblock, 0, st, a, -1, launches++ & 1);
        for (int j = 0; j < b.Kmax; ++j) {
            if (dsquared) hipLaunchKernelGGL(seed_big_pass<true>, bgrid, bblock, 0, st, a, j, launches++ & 1);
            else hipLaunchKernelGGL(seed_big_pass<false>, bgrid, bblock, 0, st, a, j, launches++ & 1);
        }
    }
    return hipGetLastError();
}

}  // namespace kb
