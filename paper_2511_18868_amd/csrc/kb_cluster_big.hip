// K-Means (Lloyd) clustering, multi-workgroup path: for searches too large for
// one workgroup or with more than 64 clusters (Sec. 3.3; L2 norm of Eq. 3).
//
// Same three phases per step as the one-workgroup kernel - fast matrix-core
// scores with a proved error bound, exact fp64 re-evaluation of the doubtful
// candidates, and 64-bit fixed-point centroid sums moved by integer atomics
// (order-independent, so results are bit-identical from run to run) - but every
// phase is its own launch and the shared state lives in global memory:
//
//   init      centroids <- initial rows, sums/counts <- 0
//   presplit  feature rows -> bf16 (hi, mid) operand-ordered tiles, |x|^2, max|x|
//   per step:
//     renew   centroid = sum/count for clusters whose membership changed, then
//             |c|^2 and the split centroid operands (-2c) of those clusters
//     score   one workgroup per chunk of 32 tiles of one search: centroid
//             operands staged in LDS, bf16x3 MFMA scores, running best/second
//             over the centroid tiles; writes the proposed cluster of every
//             candidate and appends the doubtful ones to a list
//     exact   fp64 direct-difference distances for the listed candidates
//             (centroid rows resident in registers), proposal overwritten
//     update  candidates whose proposal differs from their cluster: partial
//             fixed-point sums per (candidate range, cluster group) in LDS,
//             flushed with 64-bit global integer atomics
//             (the assignment is kept in two buffers that swap roles every
//             step, chosen so that the last step writes the caller's array)
//   objective (before the last renewal, so it refers to the centroids that
//             entered the last step), then the last renewal.
#include "kb_cluster_dev.h"

namespace kb {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

struct BigArgs {
    int G, D, Ksum, Kmax, Kpad, it, final_pass;
    int guard;              // 1: searches with N_g < 2 K_g are left as they are
    int limit_n;            // searches of up to this many candidates (and 64 clusters) are the one-workgroup kernel's
    int mixed;              // 1: searches of the one-workgroup path (K_g <= 64, N_g <= 65536) are left to it
    int64_t N, max_tiles;
    const int32_t* seg_off;
    const int32_t* koff;
    const float* X;
    const float* cent_init;
    int32_t* assign;        // [N] the caller's output; holds the last step's assignment
    const int32_t* prev;    // [N] assignment before this step (unused in the first step)
    int32_t* next;          // [N] assignment proposed by this step
    float* cent;
    int32_t* counts;
    float* objective;
    const int32_t* tile_off;
    const int32_t* chunk_off;
    float* xn;
    bf16x8* split;
    long long* sums;        // [Ksum][D]
    float* cnpad;           // [G][Kpad]
    float* centT;           // [G][D][Kpad] centroids, feature-major (coalesced reads with lanes over centroids)
    bf16x8* aop;            // [G][Kpad/32][DS][2][64]
    int* dirty;             // [Ksum]
    unsigned* amax_bits;    // [G]
    unsigned* cnmax_bits;   // [2][G]
    int* nflag;             // [2]: candidates listed for the full exact pass, records for the short one
    int32_t* flist;         // [N] global candidate indices
    int4* few;              // [N] (candidate, count, contenders 0..3, contenders 4..7 as bytes)
    double* partJ;          // [chunks]
    double* tsq_part;       // [tiles] sum of x^2 over the rows of every tile (exact products, fp64 sums)
    int* needfull;          // [G] 1: the objective of this search has to be summed member by member
};

// searches this launch sequence leaves untouched
__device__ __forceinline__ bool skipped(const BigArgs& a, int ng, int K) {
    return (a.guard && ng < 2 * K) || (a.mixed && !search_is_big(ng, K, a.limit_n));
}

// largest g with off[g] <= v (off non-decreasing, off[0] = 0, v < off[G])
__device__ __forceinline__ int upper_search(const int32_t* off, int G, int64_t v) {
    int lo = 0, hi = G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)off[mid] <= v) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ void __launch_bounds__(kThreads) big_init(BigArgs a) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int D = a.D;
    for (int64_t idx = t0; idx < (int64_t)a.Ksum * D; idx += stride) {
        const int r = (int)(idx / D), d = (int)(idx - (int64_t)r * D);
        float v;
        a.sums[idx] = 0;
        if (a.cent_init && !a.guard && !a.mixed) {
            v = a.cent_init[idx];
        } else {
            const int g = upper_search(a.koff, a.G, r);
            int n0, ng, k0, K;
            search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
            if (skipped(a, ng, K)) continue;
            const int j = r - k0;
            v = a.cent_init ? a.cent_init[idx]
                            : (ng > 0 ? a.X[(size_t)(n0 + (j < ng ? j : ng - 1)) * D + d] : 0.f);
        }
        a.cent[idx] = v;
    }
    if (a.it < 0) return;   // iters == 0: only the initial centroids
    for (int64_t r = t0; r < a.Ksum; r += stride) {
        a.dirty[r] = 0;
        if (a.guard || a.mixed) {
            const int g = upper_search(a.koff, a.G, r);
            int n0, ng, k0, K;
            search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
            if (skipped(a, ng, K)) continue;
        }
        a.counts[r] = 0;
    }
    for (int64_t g = t0; g < a.G; g += stride) {
        a.amax_bits[g] = 0u;
        a.cnmax_bits[g] = 0u;
        a.cnmax_bits[a.G + g] = 0u;
    }
    if (t0 == 0) { a.nflag[0] = 0; a.nflag[1] = 0; }
}

template <int DS>
__global__ void __launch_bounds__(kThreads) big_presplit(BigArgs a) {
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int64_t gt = (int64_t)blockIdx.x * kWaves + wid;
    if (gt >= a.tile_off[a.G] || gt >= a.max_tiles) return;
    const int g = upper_search(a.tile_off, a.G, gt);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    const int tile = (int)(gt - a.tile_off[g]);
    if (tile * 32 >= ng) return;
    if (a.mixed && !search_is_big(ng, K, a.limit_n)) return;      // (the one-workgroup kernel splits its own rows)
    const int D = a.D;
    const bool vec = (D & 3) == 0;
    const int p = tile * 32 + m;
    const bool valid = p < ng;
    const float* xr = a.X + (size_t)(n0 + (valid ? p : 0)) * D;
    bf16x8* tp = a.split + (size_t)gt * (DS * 2 * 64) + lane;
    float xnp = 0.f, am = 0.f;
    double sq = 0.0;
#pragma unroll
    for (int s = 0; s < DS; ++s) {
        const int d0 = 16 * s + 8 * h;
        float x[8];
        if (vec) {
            float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
            if (valid && d0 < D) v0 = *reinterpret_cast<const float4*>(xr + d0);
            if (valid && d0 + 4 < D) v1 = *reinterpret_cast<const float4*>(xr + d0 + 4);
            x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
            x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = (valid && d0 + i < D) ? xr[d0 + i] : 0.f;
        }
        bf16x8 hi, mid;
        split8(x, hi, mid);
        tp[(2 * s) * 64] = hi;
        tp[(2 * s + 1) * 64] = mid;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            xnp = fmaf(x[i], x[i], xnp);
            am = fmaxf(am, fabsf(x[i]));
            sq = fma((double)x[i], (double)x[i], sq);
        }
    }
    xnp += __shfl_xor(xnp, 32);
    if (valid && h == 0) a.xn[(size_t)n0 + p] = xnp;
    sq = wave_sum_d(sq);                      // fixed order: the same bits in every run
    if (lane == 0) a.tsq_part[gt] = sq;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) am = fmaxf(am, __shfl_xor(am, o));
    // non-negative floats order like their bit patterns; most waves find a value
    // at least as large already recorded and skip the atomic (the plain read may
    // be stale, which only costs an unnecessary atomic)
    if (lane == 0) {
        const unsigned bits = __float_as_uint(am);
        if (bits > *reinterpret_cast<volatile unsigned*>(&a.amax_bits[g])) atomicMax(&a.amax_bits[g], bits);
    }
}

// One wave per (search, padded centroid row).
template <int DS>
__global__ void __launch_bounds__(kThreads) big_renew(BigArgs a) {
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * kWaves + wid;
    if (r >= (int64_t)a.G * a.Kpad) return;
    const int g = (int)(r / a.Kpad), j = (int)(r - (int64_t)g * a.Kpad);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kpad) K = a.Kpad;
    if (r == 0 && lane == 0) { a.nflag[0] = 0; a.nflag[1] = 0; }
    if (skipped(a, ng, K)) return;
    const int D = a.D;
    const int mt = j >> 5, lane_row = j & 31;
    __bf16* ap = reinterpret_cast<__bf16*>(a.aop + (size_t)g * (a.Kpad / 32) * (DS * 2 * 64));
    auto store_operand = [&](float v) {
        // feature `lane` of row j: K-step s, half h, element i of the 16-byte entry
        if (lane < 16 * DS) {
            const int s = lane >> 4, h = (lane >> 3) & 1, i = lane & 7;
            const __bf16 hi = (__bf16)v;
            const __bf16 mid = (__bf16)(v - (float)hi);
            const size_t e = (((size_t)(mt * DS + s) * 2) * 64 + (lane_row + 32 * h)) * 8 + i;
            ap[e] = hi;
            ap[e + 64 * 8] = mid;
        }
    };
    if (j >= K || ng <= 0) {
        if (a.it == 0 && !a.final_pass) {
            if (lane == 0) a.cnpad[r] = kBig;
            store_operand(0.f);
        }
        return;
    }
    const int row = k0 + j;
    const int was_dirty = a.dirty[row];
    if ((a.it > 0 || a.final_pass) && was_dirty) {
        const int c = a.counts[row];
        if (c > 0 && lane < D) {
            const int sh = fixed_shift(__uint_as_float(a.amax_bits[g]), ng);
            const double inv = ldexp(1.0, -sh);
            a.cent[(size_t)row * D + lane] =
                (float)(((double)a.sums[(size_t)row * D + lane] * inv) / (double)c);
        }
    }
    if (a.final_pass) return;
    float f;
    if (a.it == 0 || was_dirty) {
        const float c = lane < D ? a.cent[(size_t)row * D + lane] : 0.f;
        f = (float)wave_sum_d((double)c * (double)c);
        if (lane == 0) a.cnpad[r] = f;
        if (lane < D) a.centT[((size_t)g * D + lane) * a.Kpad + j] = c;
        store_operand(-2.f * c);
    } else {
        f = a.cnpad[r];
    }
    if (lane == 0) {
        a.dirty[row] = 0;
        atomicMax(&a.cnmax_bits[(a.it & 1) * a.G + g], __float_as_uint(f));
        if (j == 0) a.cnmax_bits[((a.it + 1) & 1) * a.G + g] = 0u;
    }
}

// One workgroup per chunk of kTilesPerChunk tiles of one search.
//
// The centroid operands stay in registers for the whole chunk: the centroids are
// cut into groups of 64 (two matrix-core tiles) and every wave owns one group -
// its bf16 (hi, mid) operands (16 * DS VGPRs) and, as the accumulator input of
// the first product, its |c|^2.  The candidate tiles are what moves: four tiles
// at a time are copied from global memory into LDS (the copy of the next four is
// requested before the current four are scored) and every wave reads each tile's
// operands from there, 2 * DS 16-byte LDS reads per 6 * DS matrix instructions.
// With fewer than four centroid groups the waves that share a group split the
// tiles among themselves.
//
// Best and second best of a lane's 32 scores are tracked with two vector
// instructions per score (median-of-three, minimum) on scores whose 5 lowest
// mantissa bits have been replaced by the score's position; the position of the
// minimum is read back from those bits.  The replacement moves a score by less
// than 2^-18 of its magnitude, which the error bound below accounts for.  The
// per-group results of a tile meet in LDS and one wave per tile merges them,
// decides whether the nearest centroid is certain, and writes the proposal.
constexpr int kGroupTiles = 4;     // candidate tiles staged in LDS at a time
constexpr int kListCap = 512;      // doubtful candidates of a chunk collected in LDS per list; further ones
                                   // are appended to the global lists one by one

template <int DS>
__global__ void __launch_bounds__(kThreads, 2) big_score(BigArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int c = blockIdx.x;
    if (c >= a.chunk_off[a.G]) return;
    const int g = upper_search(a.chunk_off, a.G, c);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kpad) K = a.Kpad;
    if (ng <= 0 || K <= 0) return;
    if (skipped(a, ng, K)) return;
    const int ntiles = (ng + 31) >> 5;
    const int t0 = (c - a.chunk_off[g]) * kTilesPerChunk;
    const int t1 = t0 + kTilesPerChunk < ntiles ? t0 + kTilesPerChunk : ntiles;
    const int64_t tb = a.tile_off[g];
    if (t0 >= t1 || tb + ntiles > a.max_tiles) return;
    const int mtiles = (K + 31) >> 5;
    const int ngroups = (mtiles + 1) >> 1;          // centroid groups of 64: 1..4
    const int nx = kWaves / ngroups;                // waves per centroid group
    const int cgroup = wid % ngroups, xsub = wid / ngroups;
    const bool active = xsub < nx;                  // with three groups the fourth wave only copies
    const bool have1 = 2 * cgroup + 1 < mtiles;     // the group's second tile of 32 centroids exists

    constexpr int kTileUnits = DS * 2 * 64;         // 16-byte units of one candidate tile
    bf16x8* stage = reinterpret_cast<bf16x8*>(smem);                                  // [kGroupTiles][kTileUnits]
    // per (centroid group, tile, lane): best and second best of the lane's 32 scores
    float2* res = reinterpret_cast<float2*>(smem + (size_t)kGroupTiles * kTileUnits * 16);   // [4][kGroupTiles][64]
    // doubtful candidates of this chunk: those with at most one possible nearest
    // centroid per lane part go to `lfew` with the list of those centroids, the
    // others to `lflag` for the full exact pass
    int4* lfew = reinterpret_cast<int4*>(res + 4 * kGroupTiles * 64);   // [kListCap]
    int* lflag = reinterpret_cast<int*>(lfew + kListCap);               // [kListCap]
    int* lcount = lflag + kListCap;                 // [4]: counts, bases in the global lists
    if (tid < 2) lcount[tid] = 0;

    // this wave's centroid operands and |c|^2, resident for the whole chunk
    bf16x8 Ah[2][DS], Am[2][DS];
    f32x16 cnr[2];
    {
        const bf16x8* src = a.aop + (size_t)g * (a.Kpad / 32) * kTileUnits;
        const float* cnp = a.cnpad + (size_t)g * a.Kpad;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int mt = (t == 0 || have1) ? 2 * cgroup + t : 2 * cgroup;
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                Ah[t][s] = src[((mt * DS + s) * 2 + 0) * 64 + lane];
                Am[t][s] = src[((mt * DS + s) * 2 + 1) * 64 + lane];
            }
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 c4 = *reinterpret_cast<const float4*>(cnp + mt * 32 + 8 * g4 + 4 * h);
                cnr[t][4 * g4 + 0] = c4.x; cnr[t][4 * g4 + 1] = c4.y;
                cnr[t][4 * g4 + 2] = c4.z; cnr[t][4 * g4 + 3] = c4.w;
            }
        }
    }
    const float cnmax = __uint_as_float(a.cnmax_bits[(a.it & 1) * a.G + g]);
    const float kappa = mfma_kappa(DS);    // matrix-core products and position bits
    const bf16x8* sp = a.split + (size_t)tb * kTileUnits;

    // copy of a group of tiles: global -> registers (early) -> LDS (when the
    // previous group has been scored)
    constexpr int kPre = kGroupTiles * kTileUnits / kThreads;     // = 2 * DS units per thread
    bf16x8 pre[kPre];
    auto prefetch = [&](int gt0) {
        const int cnt = t1 - gt0 < kGroupTiles ? t1 - gt0 : kGroupTiles;
        const bf16x8* src = sp + (size_t)gt0 * kTileUnits;
#pragma unroll
        for (int i = 0; i < kPre; ++i) {
            const int u = tid + i * kThreads;
            // clamped, not skipped: the number of loads in flight is then fixed
            pre[i] = src[u < cnt * kTileUnits ? u : 0];
        }
    };
    prefetch(t0);
    for (int gt0 = t0; gt0 < t1; gt0 += kGroupTiles) {
        const int cnt = t1 - gt0 < kGroupTiles ? t1 - gt0 : kGroupTiles;
#pragma unroll
        for (int i = 0; i < kPre; ++i) stage[tid + i * kThreads] = pre[i];
        __syncthreads();
        if (gt0 + kGroupTiles < t1) prefetch(gt0 + kGroupTiles);

        // |x|^2 of the tile this wave closes below, requested before the scoring
        float xn_close = 0.f;
        {
            const int p = (gt0 + wid) * 32 + m;
            if (wid < cnt && p < ng) xn_close = a.xn[(size_t)n0 + p];
        }

        // best and second best of the 16 scores of one accumulator, position
        // (offset `base`) in the 5 lowest bits; three vector instructions per score
        auto argmin16 = [&](const f32x16& acc, unsigned base, float& cb, float& cs) {
            cb = kBig * 8.f; cs = kBig * 8.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v = __uint_as_float((__float_as_uint(acc[r]) & 0xffffffe0u) | (base + (unsigned)r));
                cs = __builtin_amdgcn_fmed3f(cb, cs, v);
                cb = vmin(cb, v);
            }
        };
        // union of the two accumulators' results: this lane's part of tile tt
        auto close_tile = [&](int tt, float cb0, float cs0, float cb1, float cs1) {
            const float lo = vmin(cb0, cb1);
            const float hi = vmax(cb0, cb1);
            const float second = vmin(vmin(cs0, cs1), hi);
            res[(cgroup * kGroupTiles + tt) * 64 + lane] = make_float2(lo, second);
        };

        if (active && have1) {
            // Two accumulators, one per tile of 32 centroids, used in turn: while the
            // matrix cores fill one, the vector unit takes the minimum of the other
            // (the previous half of the work), so neither waits for the other.
            bf16x8 Bh[DS], Bm[DS];
            {
                const bf16x8* bt = stage + (xsub < cnt ? xsub : 0) * kTileUnits + lane;
#pragma unroll
                for (int s = 0; s < DS; ++s) { Bh[s] = bt[(2 * s) * 64]; Bm[s] = bt[(2 * s + 1) * 64]; }
            }
            f32x16 acc0, acc1;
            float cb0, cs0, cb1, cs1;
            auto chain0 = [&]() {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[0][0], Bh[0], cnr[0], 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[0][0], Bm[0], acc0, 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Am[0][0], Bh[0], acc0, 0, 0, 0);
#pragma unroll
                for (int s = 1; s < DS; ++s) {
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[0][s], Bh[s], acc0, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[0][s], Bm[s], acc0, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Am[0][s], Bh[s], acc0, 0, 0, 0);
                }
            };
            if (xsub < cnt) {
                chain0();
                for (int tt = xsub;;) {
                    // second tile of centroids of candidate tile tt, while the vector
                    // unit takes the minimum of the first; the candidate operands of a
                    // step are replaced by the next tile's as soon as they are spent
                    const int nt = tt + nx;
                    const bf16x8* bt = stage + (nt < cnt ? nt : tt) * kTileUnits + lane;
#pragma unroll
                    for (int s = 0; s < DS; ++s) {
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[1][s], Bh[s], s == 0 ? cnr[1] : acc1, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[1][s], Bm[s], acc1, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Am[1][s], Bh[s], acc1, 0, 0, 0);
                        Bh[s] = bt[(2 * s) * 64];
                        Bm[s] = bt[(2 * s + 1) * 64];
                    }
                    argmin16(acc0, 0u, cb0, cs0);
#pragma unroll
                    for (int r = 0; r < DS * 3; ++r) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                        __builtin_amdgcn_sched_group_barrier(0x002, 5, 1);
                    }
                    if (nt >= cnt) {
                        argmin16(acc1, 16u, cb1, cs1);
                        close_tile(tt, cb0, cs0, cb1, cs1);
                        break;
                    }
                    // first tile of centroids of the next candidate tile, while the
                    // vector unit finishes this one
                    chain0();
                    argmin16(acc1, 16u, cb1, cs1);
                    close_tile(tt, cb0, cs0, cb1, cs1);
#pragma unroll
                    for (int r = 0; r < DS * 3; ++r) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                    }
                    tt = nt;
                }
            }
        } else if (active) {
            // one tile of 32 centroids in this group: the third product goes to a
            // second accumulator so that two chains are in flight
            for (int tt = xsub; tt < cnt; tt += nx) {
                const bf16x8* bt = stage + tt * kTileUnits + lane;
                f32x16 acc0 = cnr[0], acc1;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc1[r] = 0.f;
#pragma unroll
                for (int s = 0; s < DS; ++s) {
                    const bf16x8 Bh = bt[(2 * s) * 64], Bm = bt[(2 * s + 1) * 64];
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[0][s], Bh, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[0][s], Bm, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Am[0][s], Bh, acc0, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) acc0[r] += acc1[r];
                float cb0, cs0;
                argmin16(acc0, 0u, cb0, cs0);
                close_tile(tt, cb0, cs0, kBig * 8.f, kBig * 8.f);
            }
        }
        __syncthreads();
        // wave w closes tile w of the group: merge the lanes' parts over the centroid
        // groups and the two half-waves, read the position of the minimum back from
        // its lowest bits, decide
        if (wid < cnt) {
            const int tile = gt0 + wid;
            const int p = tile * 32 + m;
            const bool mine = h == 0 && p < ng;
            float best = kBig * 16.f, second = kBig * 16.f;
            int slot = 0;           // 2 * centroid group + half-wave of the best so far
            if (mine) {
                for (int cg = 0; cg < ngroups; ++cg) {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const float2 r = res[(cg * kGroupTiles + wid) * 64 + hh * 32 + m];
                        merge_best(best, second, slot, r.x, r.y, 2 * cg + hh);
                    }
                }
            }
            const int code = (int)(__float_as_uint(best) & 31u);
            const int bi = (slot >> 1) * 64 + (code >> 4) * 32 + 8 * ((code & 15) >> 2) + (code & 3) +
                           4 * (slot & 1);
            const float E = kappa * (xn_close + cnmax);
            // a best score next to zero may have lost its position bits to a flush of
            // subnormal numbers: leave that candidate to the full exact pass
            const bool sane = fabsf(best) > 1.0e-30f && bi < K;
            const bool certain = (K == 1) || (((second - best) > 2.f * E) && sane);
            if (mine) a.next[(size_t)n0 + p] = bi < K ? bi : 0;
            // Doubtful candidates, one at a time with the whole wave.  Every centroid
            // that can be the true nearest one has a score within 2E of the best.  Lane
            // q looks at lane part q of the candidate: the part contributes its own
            // best if that is within the threshold; if its second best is too, the
            // part holds more such centroids than it can name and the candidate goes
            // to the full exact pass.  Otherwise the named centroids (at most eight)
            // are recorded for the short one.
            const float thr = best + 2.f * E;
            unsigned long long todo = __ballot(mine && !certain);
            while (todo) {
                const int bl = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                const float thr_b = __shfl(thr, bl);
                const int sane_b = __shfl((int)sane, bl);
                const int q = lane;
                bool is = false, over = false;
                int idx = 0;
                if (q < 2 * ngroups) {
                    const float2 r = res[((q >> 1) * kGroupTiles + wid) * 64 + (q & 1) * 32 + bl];
                    const int cd = (int)(__float_as_uint(r.x) & 31u);
                    idx = (q >> 1) * 64 + (cd >> 4) * 32 + 8 * ((cd & 15) >> 2) + (cd & 3) + 4 * (q & 1);
                    is = r.x <= thr_b;
                    over = r.y <= thr_b || (is && idx >= K);
                }
                const unsigned long long cm = __ballot(is), om = __ballot(over);
                const int pcand = n0 + tile * 32 + bl;
                // at most one entry per candidate of the chunk in either list
                if (sane_b && om == 0ull && cm != 0ull) {
                    int e = 0;
                    if (lane == 0) e = atomicAdd(&lcount[1], 1);
                    e = __shfl(e, 0);
                    int4* rec = lfew + e;
                    if (e >= kListCap) {                    // (uniform) the LDS list is full
                        long long pos = 0;
                        if (lane == 0) pos = atomicAdd(&a.nflag[1], 1);
                        pos = __shfl(pos, 0);
                        rec = a.few + (pos < a.N ? pos : 0);
                        if (pos >= a.N) continue;           // (cannot happen: one record per candidate at most)
                    }
                    if (is) {
                        const int rank = __popcll(cm & ((1ull << q) - 1ull));
                        reinterpret_cast<unsigned char*>(rec)[8 + rank] = (unsigned char)idx;
                    }
                    if (lane == 0) {
                        int* hdr = reinterpret_cast<int*>(rec);
                        hdr[0] = pcand;
                        hdr[1] = __popcll(cm);
                    }
                } else if (lane == 0) {
                    const int e = atomicAdd(&lcount[0], 1);
                    if (e < kListCap) {
                        lflag[e] = pcand;
                    } else {
                        const long long pos = atomicAdd(&a.nflag[0], 1);
                        if (pos < a.N) a.flist[pos] = pcand;
                    }
                }
            }
        }
    }
    __syncthreads();
    const int nl = lcount[0] < kListCap ? lcount[0] : kListCap;
    const int nf = lcount[1] < kListCap ? lcount[1] : kListCap;
    if (nl > 0 || nf > 0) {
        if (tid == 0 && nl > 0) lcount[2] = atomicAdd(&a.nflag[0], nl);
        if (tid == 1 && nf > 0) lcount[3] = atomicAdd(&a.nflag[1], nf);
        __syncthreads();
        const int64_t pos0 = lcount[2], pos1 = lcount[3];
        for (int i = tid; i < nl; i += kThreads)
            if (pos0 + i < a.N) a.flist[pos0 + i] = lflag[i];
        for (int i = tid; i < nf; i += kThreads)
            if (pos1 + i < a.N) a.few[pos1 + i] = lfew[i];
    }
}

// The same step of the path with fp32 fused multiply-adds on the vector ALU
// (scorer mode 1): the reference the matrix-core scorer is measured against.
// One workgroup per chunk of kTilesPerChunk tiles; the search's centroids are
// staged in LDS (every lane of a wave reads the same centroid entry, which LDS
// broadcasts), a thread holds one candidate's row in registers at a time.  The
// dot product is a chain of fused multiply-adds in two interleaved parts and
// s_j = fma(-2, dot, |c_j|^2); with u = 2^-24,
//   |s' - s| <= (D + 3) u (1 + o(1)) (|x|^2 + max_j |c_j|^2),
// and kappa = (D + 4) u leaves room for the rounding of |x|^2, of E itself and of
// the gap.  A candidate whose two best scores are not 2E apart goes to the full
// exact pass.
template <int DS>
__global__ void __launch_bounds__(kThreads, 2) big_score_valu(BigArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int DP = 16 * DS;
    const int tid = threadIdx.x;
    const int c = blockIdx.x;
    if (c >= a.chunk_off[a.G]) return;
    const int g = upper_search(a.chunk_off, a.G, c);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kpad) K = a.Kpad;
    if (ng <= 0 || K <= 0) return;
    if (skipped(a, ng, K)) return;
    const int p0 = (c - a.chunk_off[g]) * kTilesPerChunk * 32;
    const int p1 = p0 + kTilesPerChunk * 32 < ng ? p0 + kTilesPerChunk * 32 : ng;
    if (p0 >= p1) return;
    const int D = a.D;

    float* cent = reinterpret_cast<float*>(smem);                   // [Kpad][DP], rows zero-padded
    float* cn = cent + (size_t)a.Kpad * DP;                          // [Kpad]
    int* lflag = reinterpret_cast<int*>(cn + a.Kpad);                // [kTilesPerChunk * 32]
    int* lcount = lflag + kTilesPerChunk * 32;                       // [2]: count, base in the global list
    if (tid == 0) lcount[0] = 0;
    for (int idx = tid; idx < K * DP; idx += kThreads) {
        const int j = idx / DP, d = idx - j * DP;
        cent[idx] = d < D ? a.cent[(size_t)(k0 + j) * D + d] : 0.f;
    }
    for (int j = tid; j < K; j += kThreads) cn[j] = a.cnpad[(size_t)g * a.Kpad + j];
    __syncthreads();

    const float cnmax = __uint_as_float(a.cnmax_bits[(a.it & 1) * a.G + g]);
    const float kappa = (float)(D + 4) * 5.9604644775390625e-08f;
    const bool vec = (D & 3) == 0;
    for (int p = p0 + tid; p < p1; p += kThreads) {
        float x[DP];
        const float* xr = a.X + (size_t)(n0 + p) * D;
        if (vec) {
#pragma unroll
            for (int q = 0; q < DP / 4; ++q) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (4 * q < D) v = reinterpret_cast<const float4*>(xr)[q];
                x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int d = 0; d < DP; ++d) x[d] = d < D ? xr[d] : 0.f;
        }
        float xn = 0.f;
#pragma unroll
        for (int d = 0; d < DP; ++d) xn = fmaf(x[d], x[d], xn);
        float best = INFINITY, second = INFINITY;
        int bi = 0;
        for (int j = 0; j < K; ++j) {
            const float4* cr = reinterpret_cast<const float4*>(cent + (size_t)j * DP);
            float d0 = 0.f, d1 = 0.f;
#pragma unroll
            for (int q = 0; q < DP / 4; ++q) {
                const float4 cv = cr[q];
                d0 = fmaf(x[4 * q], cv.x, d0);
                d1 = fmaf(x[4 * q + 1], cv.y, d1);
                d0 = fmaf(x[4 * q + 2], cv.z, d0);
                d1 = fmaf(x[4 * q + 3], cv.w, d1);
            }
            const float sc = fmaf(-2.f, d0 + d1, cn[j]);
            const bool lt = sc < best;
            second = lt ? best : fminf(second, sc);
            bi = lt ? j : bi;
            best = lt ? sc : best;
        }
        const float E = kappa * (xn + cnmax);
        const bool certain = (K == 1) || ((second - best) > 2.f * E);
        a.next[(size_t)n0 + p] = bi;
        if (!certain) lflag[atomicAdd(&lcount[0], 1)] = n0 + p;      // at most one entry per candidate of the chunk
    }
    __syncthreads();
    const int nl = lcount[0];
    if (nl > 0) {
        if (tid == 0) lcount[1] = atomicAdd(&a.nflag[0], nl);
        __syncthreads();
        const int64_t pos0 = lcount[1];
        for (int i = tid; i < nl; i += kThreads)
            if (pos0 + i < a.N) a.flist[pos0 + i] = lflag[i];
    }
}

// Short exact pass: a doubtful candidate whose possible nearest centroids are
// all named (at most eight) needs the exact distance to those only.  Eight
// threads per candidate, one per named centroid; each forms its squared distance
// exactly as the plain definition does - fp64, direct differences, summed over the
// features in index order with separate multiply and add - and the eight reduce
// to the minimum, lowest centroid index on ties.
__device__ __forceinline__ void exact_few(const BigArgs& a, int block, int nblocks) {
    int64_t n = a.nflag[1];
    if (n > a.N) n = a.N;
    const int D = a.D;
    const int64_t stride = (int64_t)nblocks * (kThreads / 8);
    const int slot = threadIdx.x & 7;
    for (int64_t i = (int64_t)block * (kThreads / 8) + (threadIdx.x >> 3); i < n; i += stride) {
        const int4 rec = a.few[i];
        const int pg = rec.x;
        double dist = INFINITY;
        int jj = 0x7fffffff;
        int K = 0;
        if (pg >= 0 && pg < a.N) {
            const int g = upper_search(a.seg_off, a.G, pg);
            int n0, ng, k0;
            search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
            if (slot < rec.y && slot < 8) {
                const unsigned packed = slot < 4 ? (unsigned)rec.z : (unsigned)rec.w;
                const int j = (int)((packed >> (8 * (slot & 3))) & 0xffu);
                if (j < K) {
                    const float* xr = a.X + (size_t)pg * D;
                    const float* cr = a.cent + (size_t)(k0 + j) * D;
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d) {
                        const double diff = __dsub_rn((double)xr[d], (double)cr[d]);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    }
                    dist = acc;
                    jj = j;
                }
            }
        }
#pragma unroll
        for (int o = 4; o > 0; o >>= 1) {
            const double od = __shfl_xor(dist, o);
            const int oj = __shfl_xor(jj, o);
            if (od < dist || (od == dist && oj < jj)) { dist = od; jj = oj; }
        }
        if (slot == 0 && jj < K) a.next[pg] = jj;
    }
}

// Exact nearest centroid for the listed candidates: a workgroup takes one
// candidate at a time, one wave per group of 64 centroids, lanes over centroids.
// A lane keeps its centroid in registers from one candidate to the next (read
// from the feature-major copy, so the loads are coalesced).  A first pass computes every squared
// distance in fp32 (direct differences, a sum of non-negative terms, so its
// relative error is at most (D + 2) 2^-24 < 5e-6); only groups that hold a
// distance within a factor 1 + 3e-5 of the smallest - every true minimiser is
// among them - are evaluated exactly: fp64 direct differences summed over the
// features in index order with separate multiply and add, lowest index on ties.
__device__ __forceinline__ void exact_full(const BigArgs& a, int block, int nblocks) {
    static_assert(KB_MAX_K <= kThreads, "one lane per centroid");
    __shared__ float redm[kWaves];
    __shared__ double redd[kWaves];
    __shared__ int redj[kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    int64_t n = *a.nflag;
    if (n > a.N) n = a.N;
    const int D = a.D;
    const int D4 = (D + 3) & ~3;
    float c[KB_MAX_D];          // this lane's centroid, kept while the search stays the same
    int g_held = -1;
    // two requests ahead: the index of the candidate after next, and the row of the
    // next one (whose index has arrived by then)
    auto index_at = [&](int64_t i) {
        const int v = i < n ? a.flist[i] : -1;
        return (v >= 0 && v < a.N) ? v : -1;
    };
    auto row_at = [&](int pgv) { return (pgv >= 0 && lane < D) ? a.X[(size_t)pgv * D + lane] : 0.f; };
    int pg_cur = index_at(block);
    int pg_nxt = index_at((int64_t)block + nblocks);
    float xv_cur = row_at(pg_cur);
    for (int64_t i = block; i < n; i += nblocks) {
        // everything up to the barriers is uniform over the workgroup
        const int pg = pg_cur;
        const float xv = xv_cur;
        pg_cur = pg_nxt;
        pg_nxt = index_at(i + 2 * (int64_t)nblocks);
        xv_cur = row_at(pg_cur);
        if (pg < 0) continue;
        const int g = upper_search(a.seg_off, a.G, pg);
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (K <= 0) continue;
        if (K > a.Kpad) K = a.Kpad;
        const int j = tid;                      // this lane's centroid
        const bool group = wid * kWave < K;     // uniform over the wave
        if (g != g_held) {
            g_held = g;
            const float* ct = a.centT + (size_t)g * D * a.Kpad + (j < K ? j : 0);
#pragma unroll
            for (int d = 0; d < KB_MAX_D; ++d) c[d] = (group && d < D) ? ct[(size_t)d * a.Kpad] : 0.f;
        }
        float d32 = INFINITY;
        if (group) {
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int d = 0; d < KB_MAX_D; d += 2) {
                if (d < D4) {
                    const float e0 = lane_value(xv, d) - c[d];
                    const float e1 = lane_value(xv, d + 1) - c[d + 1];
                    acc0 = fmaf(e0, e0, acc0);
                    acc1 = fmaf(e1, e1, acc1);
                }
            }
            if (j < K) d32 = acc0 + acc1;
        }
        float m32 = d32;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m32 = fminf(m32, __shfl_xor(m32, o));
        if (lane == 0) redm[wid] = m32;
        __syncthreads();
        m32 = fminf(fminf(redm[0], redm[1]), fminf(redm[2], redm[3]));
        const float thr = m32 * 1.00003f + 1.0e-35f;   // the constant covers sums that underflow
        double bd = INFINITY;
        int bj = 0x7fffffff;
        if (group && __any(d32 <= thr)) {
            // features beyond D are 0 on both sides: their terms add +0.0
            double acc = 0.0;
#pragma unroll
            for (int d = 0; d < KB_MAX_D; ++d) {
                if (d < D4) {
                    const double diff = __dsub_rn((double)lane_value(xv, d), (double)c[d]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                }
            }
            if (j < K) { bd = acc; bj = j; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double od = __shfl_xor(bd, o);
            const int oj = __shfl_xor(bj, o);
            if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
        }
        if (lane == 0) { redd[wid] = bd; redj[wid] = bj; }
        __syncthreads();
        if (tid == 0) {
            // groups in ascending centroid order: a strict compare keeps the lowest index
#pragma unroll
            for (int w = 1; w < kWaves; ++w)
                if (redd[w] < bd) { bd = redd[w]; bj = redj[w]; }
            a.next[pg] = bj < K ? bj : 0;
        }
    }
}

// Both exact passes in one launch: the first kFewBlocks workgroups take the short
// pass, the others the full one (their lists are disjoint, so they do not meet).
constexpr int kFewBlocks = 512, kFullBlocks = 1024;
__global__ void __launch_bounds__(kThreads) big_exact(BigArgs a) {
    if (blockIdx.x < kFewBlocks) exact_few(a, (int)blockIdx.x, kFewBlocks);       // (uniform over the workgroup)
    else exact_full(a, (int)blockIdx.x - kFewBlocks, kFullBlocks);
}

// Move the candidates whose proposal differs from their previous cluster.  A
// workgroup owns a group of kRowsPerGroup clusters of one search and a range of
// its candidates.  It works through the range in batches: the (previous,
// proposed) pairs of a batch are scanned and the candidates that join or leave
// one of its clusters are listed in LDS; then 16 lanes per listed row (features
// l, l + 16, ...) convert it to fixed point and add or subtract it in LDS
// (integer atomics), with the next row already requested.  The partial sums go
// to the global fixed-point sums once, at the end.
constexpr int kRowsPerGroup = 32;
constexpr int kUpdateRange = 8192;    // candidates per workgroup
constexpr int kUpdateBatch = 4096;    // candidates scanned per list
__global__ void __launch_bounds__(kThreads) big_update(BigArgs a) {
    __shared__ long long lsum[kRowsPerGroup * KB_MAX_D];
    __shared__ int lcnt[kRowsPerGroup];
    __shared__ int ltouched[kRowsPerGroup];
    __shared__ int list[kUpdateBatch];     // offset in the batch | (row joined + 1) << 16 | (row left + 1) << 24
    __shared__ int nlist;
    const int tid = threadIdx.x;
    const int grp = tid >> 4, l16 = tid & 15;
    constexpr int kGroups = kThreads / 16, E = KB_MAX_D / 16;
    static_assert(kRowsPerGroup < 255 && kUpdateBatch <= 65536, "list entry packing");
    // blockIdx.x = (range chunk over all candidates), blockIdx.y = cluster group
    const int64_t r0 = (int64_t)blockIdx.x * kUpdateRange;
    if (r0 >= a.N) return;
    const int64_t r1 = r0 + kUpdateRange < a.N ? r0 + kUpdateRange : a.N;
    const int jg0 = blockIdx.y * kRowsPerGroup;
    const int D = a.D;
    const bool first = a.it == 0;
    // a range may span several searches: handle them one after the other
    int g = upper_search(a.seg_off, a.G, r0);
    const auto mine = [&](int n0, int ng, int k0, int K) {
        return n0 >= r1 || (ng > 0 && jg0 < K && !skipped(a, ng, K));
    };
    for (; (g = next_search(a.seg_off, a.koff, g, a.G, a.N, a.Ksum, mine)) < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (n0 >= r1) break;
        if (jg0 >= K || ng <= 0) continue;
        if (skipped(a, ng, K)) continue;
        const int64_t q0 = r0 > n0 ? r0 : n0;
        const int64_t q1 = r1 < (int64_t)n0 + ng ? r1 : (int64_t)n0 + ng;
        if (q0 >= q1) continue;
        const int rows = K - jg0 < kRowsPerGroup ? K - jg0 : kRowsPerGroup;
        for (int i = tid; i < rows * D; i += kThreads) lsum[i] = 0;
        if (tid < kRowsPerGroup) { lcnt[tid] = 0; ltouched[tid] = 0; }
        const int fsh = fixed_shift(__uint_as_float(a.amax_bits[g]), ng) - 32;
        for (int64_t b0 = q0; b0 < q1; b0 += kUpdateBatch) {
            if (tid == 0) nlist = 0;
            __syncthreads();
            const int nb = (int)(q1 - b0 < kUpdateBatch ? q1 - b0 : kUpdateBatch);
            // scan: every thread takes kUpdateBatch / kThreads candidates, loads first
            constexpr int U = kUpdateBatch / kThreads;
            int na[U], oa[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int o = u * kThreads + tid;
                na[u] = -1; oa[u] = -1;
                if (o < nb) {
                    na[u] = a.next[b0 + o];
                    if (!first) oa[u] = a.prev[b0 + o];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int o = u * kThreads + tid;
                const int nn = (na[u] >= 0 && na[u] < K) ? na[u] : 0;
                const int oo = (oa[u] >= 0 && oa[u] < K) ? oa[u] : -1;
                const bool chg = o < nb && nn != oo;
                const int jn = (chg && nn >= jg0 && nn < jg0 + rows) ? nn - jg0 + 1 : 0;
                const int jo = (chg && oo >= jg0 && oo < jg0 + rows) ? oo - jg0 + 1 : 0;
                if (jn | jo) list[atomicAdd(&nlist, 1)] = o | (jn << 16) | (jo << 24);
            }
            __syncthreads();
            const int n = nlist;
            // process: group `grp` takes entries grp, grp + 16, ...; the order in the
            // list varies from run to run, the integer sums do not depend on it
            float xv[E], xw[E];
            int ent = grp < n ? list[grp] : 0;
            if (grp < n) {
                const float* xr = a.X + (size_t)(b0 + (ent & 0xffff)) * D;
#pragma unroll
                for (int e = 0; e < E; ++e) xv[e] = (l16 + 16 * e) < D ? xr[l16 + 16 * e] : 0.f;
            }
            for (int i = grp; i < n; i += kGroups) {
                const int inext = i + kGroups;
                int ent2 = 0;
                if (inext < n) {
                    ent2 = list[inext];
                    const float* xr = a.X + (size_t)(b0 + (ent2 & 0xffff)) * D;
#pragma unroll
                    for (int e = 0; e < E; ++e) xw[e] = (l16 + 16 * e) < D ? xr[l16 + 16 * e] : 0.f;
                }
                const int jn = ((ent >> 16) & 0xff) - 1, jo = ((ent >> 24) & 0xff) - 1;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const int d = l16 + 16 * e;
                    if (d < D) {
                        const long long q = to_fixed(xv[e], fsh);
                        if (jn >= 0) atomicAdd(reinterpret_cast<unsigned long long*>(&lsum[jn * D + d]), (unsigned long long)q);
                        if (jo >= 0) atomicAdd(reinterpret_cast<unsigned long long*>(&lsum[jo * D + d]), (unsigned long long)(-q));
                    }
                }
                if (l16 == 0) {
                    if (jn >= 0) { atomicAdd(&lcnt[jn], 1); ltouched[jn] = 1; }
                    if (jo >= 0) { atomicSub(&lcnt[jo], 1); ltouched[jo] = 1; }
                }
                ent = ent2;
#pragma unroll
                for (int e = 0; e < E; ++e) xv[e] = xw[e];
            }
            __syncthreads();   // the list is rebuilt by the next batch
        }
        for (int i = tid; i < rows * D; i += kThreads) {
            const int jr = i / D;
            if (ltouched[jr])
                atomicAdd(reinterpret_cast<unsigned long long*>(a.sums + (size_t)(k0 + jg0) * D + i),
                          (unsigned long long)lsum[i]);
        }
        if (tid < rows && ltouched[tid]) {
            atomicAdd(&a.counts[k0 + jg0 + tid], lcnt[tid]);
            a.dirty[k0 + jg0 + tid] = 1;
        }
        __syncthreads();
    }
}

// Objective of the last step without a pass over the rows.  With S_j the exact
// (fixed-point) sum and n_j the size of cluster j after the step's update, and c_j
// the centroids that entered it,
//   sum_k |x_k - c_a(k)|^2 = sum_k |x_k|^2 - sum_j c_j . (2 S_j - n_j c_j),
// everything in fp64 and in a fixed order.  The subtraction cancels; when less than
// 1e-7 of the first term is left (tight clusters far from the origin) the search is
// marked and the two kernels below sum its members one by one instead.
// One workgroup per search.
constexpr int kObjThreads = 1024;
__global__ void __launch_bounds__(kObjThreads) big_objfast(BigArgs a) {
    constexpr int W = kObjThreads / kWave, U = 8;
    __shared__ double red[2][W];
    const int g = blockIdx.x, tid = threadIdx.x;
    if (g >= a.G) return;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (tid == 0) a.needfull[g] = 0;
    if (ng <= 0 || K <= 0) {
        if (tid == 0) a.objective[g] = 0.f;
        return;
    }
    if (skipped(a, ng, K)) return;
    const int D = a.D;
    const int ntiles = (ng + 31) >> 5;
    const int64_t tb = a.tile_off[g];
    if (tb + ntiles > a.max_tiles) return;
    // (U independent loads per thread and round: a search is one workgroup, so the
    // latency of its loads has to be covered inside it)
    double tsq = 0.0;
    for (int t0 = tid; t0 < ntiles; t0 += kObjThreads * U) {
        double v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * kObjThreads;
            v[u] = t < ntiles ? a.tsq_part[tb + t] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) tsq += v[u];
    }
    const int sh = fixed_shift(__uint_as_float(a.amax_bits[g]), ng);
    const double inv = ldexp(1.0, -sh);
    double part = 0.0;
    const int KD = K * D;
    for (int i0 = tid; i0 < KD; i0 += kObjThreads * U) {
        float cj[U];
        long long Sj[U];
        int nj[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u * kObjThreads;
            const bool in = i < KD;
            cj[u] = in ? a.cent[(size_t)k0 * D + i] : 0.f;
            Sj[u] = in ? a.sums[(size_t)k0 * D + i] : 0;
            nj[u] = in ? a.counts[k0 + i / D] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const double c = (double)cj[u];
            part += c * (2.0 * ((double)Sj[u] * inv) - (double)nj[u] * c);
        }
    }
    tsq = wave_sum_d(tsq);
    part = wave_sum_d(part);
    if ((tid & 63) == 0) { red[0][tid >> 6] = tsq; red[1][tid >> 6] = part; }
    __syncthreads();
    if (tid == 0) {
        double T = red[0][0], P = red[1][0];
        for (int w = 1; w < W; ++w) { T += red[0][w]; P += red[1][w]; }
        const double J = T - P;
        if (J >= 1.0e-7 * T) a.objective[g] = (float)J;
        else a.needfull[g] = 1;
    }
}

// Per-chunk partial objective: 16 lanes per candidate (features l, l + 16, ...),
// four candidates in flight per group, per-lane fp64 partial sums in a fixed
// candidate order, fixed-order reduction.
__global__ void __launch_bounds__(kThreads) big_objective(BigArgs a) {
    __shared__ double red[kWaves];
    const int tid = threadIdx.x;
    const int c = blockIdx.x;
    if (c >= a.chunk_off[a.G]) return;
    const int g = upper_search(a.chunk_off, a.G, c);
    if (!a.needfull[g]) return;          // (uniform) the fast form was accurate enough
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    const int D = a.D;
    const int p0 = (c - a.chunk_off[g]) * kTilesPerChunk * 32;
    const int p1 = p0 + kTilesPerChunk * 32 < ng ? p0 + kTilesPerChunk * 32 : ng;
    const int sub = tid >> 4, l16 = tid & 15;
    constexpr int U = 4, GR = kThreads / 16, E = KB_MAX_D / 16;
    double acc = 0.0;
    if (K > 0)
        for (int pb = p0 + sub; pb < p1; pb += GR * U) {
            int jj[U];
            float xv[U][E], cv[U][E];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = pb + u * GR;
                jj[u] = p < p1 ? a.assign[(size_t)n0 + p] : 0;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = pb + u * GR;
                const int j = (jj[u] >= 0 && jj[u] < K) ? jj[u] : 0;
                const float* xr = a.X + (size_t)(n0 + (p < p1 ? p : p0)) * D;
                const float* cr = a.cent + (size_t)(k0 + j) * D;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const int d = l16 + 16 * e;
                    xv[u][e] = (p < p1 && d < D) ? xr[d] : 0.f;
                    cv[u][e] = (p < p1 && d < D) ? cr[d] : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float sq = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float e0 = xv[u][e] - cv[u][e];
                    sq = fmaf(e0, e0, sq);
                }
                acc += (double)sq;
            }
        }
    acc = wave_sum_d(acc);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        double r = red[0];
        for (int w = 1; w < kWaves; ++w) r += red[w];
        a.partJ[c] = r;
    }
}

// One workgroup per search: the chunk partials are summed in a fixed order
// (thread t takes chunks t, t + 256, ...; then a fixed tree).
__global__ void __launch_bounds__(kThreads) big_objsum(BigArgs a) {
    __shared__ double red[kWaves];
    const int g = blockIdx.x, tid = threadIdx.x;
    if (g >= a.G) return;
    if (!a.needfull[g]) return;
    if (a.guard || a.mixed) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (ng > 0 && skipped(a, ng, K)) return;   // (uniform over the workgroup) objective left as it is
    }
    double J = 0.0;
    for (int c = a.chunk_off[g] + tid; c < a.chunk_off[g + 1]; c += kThreads) J += a.partJ[c];
    J = wave_sum_d(J);
    if ((tid & 63) == 0) red[tid >> 6] = J;
    __syncthreads();
    if (tid == 0) {
        double r = red[0];
        for (int w = 1; w < kWaves; ++w) r += red[w];
        a.objective[g] = (float)r;
    }
}

}  // namespace

static size_t al256(size_t v) { return (v + 255) & ~(size_t)255; }

BigWs big_ws_layout(const kb_batch& b, size_t base) {
    BigWs w;
    const size_t kpad = (size_t)((b.Kmax > 0 ? b.Kmax : 1) + 31) / 32 * 32;
    const size_t ds = (size_t)(b.D + 15) / 16;
    size_t off = base;
    w.kpad = (int)kpad;
    w.max_chunks = (size_t)(b.N / 32 + b.G) / kTilesPerChunk + (size_t)b.G + 1;
    w.chunk_off = off; off += al256(sizeof(int32_t) * ((size_t)b.G + 1));
    w.sums = off;      off += al256(sizeof(long long) * (size_t)(b.Ksum > 0 ? b.Ksum : 1) * b.D);
    w.cnpad = off;     off += al256(sizeof(float) * (size_t)b.G * kpad);
    w.centT = off;     off += al256(sizeof(float) * (size_t)b.G * kpad * b.D);
    w.aop = off;       off += al256((size_t)b.G * (kpad / 32) * ds * 2 * 64 * 16);
    w.dirty = off;     off += al256(sizeof(int) * (size_t)(b.Ksum > 0 ? b.Ksum : 1));
    w.amax = off;      off += al256(sizeof(unsigned) * (size_t)b.G);
    w.cnmax = off;     off += al256(sizeof(unsigned) * 2 * (size_t)b.G);
    w.nflag = off;     off += 256;
    w.few = off;       off += al256(sizeof(int4) * (size_t)(b.N > 0 ? b.N : 1));
    w.partJ = off;     off += al256(sizeof(double) * w.max_chunks);
    w.prop = off;      off += al256(sizeof(int32_t) * (size_t)(b.N > 0 ? b.N : 1));
    w.tsq = off;       off += al256(sizeof(double) * ((size_t)(b.N / 32) + (size_t)b.G));
    w.needfull = off;  off += al256(sizeof(int) * (size_t)b.G);
    w.end = off;
    return w;
}

hipError_t launch_cluster_big(const kb_batch& b, const ClusterCall& c, const BigWs& w, char* ws,
                              hipStream_t st) {
    BigArgs a;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.Kmax = b.Kmax > 0 ? b.Kmax : 1; a.Kpad = w.kpad;
    a.it = 0; a.final_pass = 0; a.guard = c.guard; a.mixed = c.mixed; a.limit_n = one_wg_limit_n(b); a.N = b.N; a.max_tiles = c.max_tiles;
    a.seg_off = b.seg_off; a.koff = b.koff; a.X = c.X; a.cent_init = c.cent_init;
    a.assign = c.assign; a.cent = c.cent_out; a.counts = c.counts; a.objective = c.objective;
    a.tile_off = c.tile_off; a.chunk_off = reinterpret_cast<const int32_t*>(ws + w.chunk_off);
    a.xn = c.xn; a.split = reinterpret_cast<bf16x8*>(c.split);
    a.sums = reinterpret_cast<long long*>(ws + w.sums);
    a.cnpad = reinterpret_cast<float*>(ws + w.cnpad);
    a.centT = reinterpret_cast<float*>(ws + w.centT);
    a.aop = reinterpret_cast<bf16x8*>(ws + w.aop);
    a.dirty = reinterpret_cast<int*>(ws + w.dirty);
    a.amax_bits = reinterpret_cast<unsigned*>(ws + w.amax);
    a.cnmax_bits = reinterpret_cast<unsigned*>(ws + w.cnmax);
    a.nflag = reinterpret_cast<int*>(ws + w.nflag);
    a.flist = c.a_new;
    a.few = reinterpret_cast<int4*>(ws + w.few);
    int32_t* const other = reinterpret_cast<int32_t*>(ws + w.prop);
    a.prev = other; a.next = c.assign;
    a.partJ = reinterpret_cast<double*>(ws + w.partJ);
    a.tsq_part = reinterpret_cast<double*>(ws + w.tsq);
    a.needfull = reinterpret_cast<int*>(ws + w.needfull);

    const int ds = (b.D + 15) / 16;
    const size_t init_items = (size_t)(b.N > (int64_t)b.Ksum * b.D ? b.N : (int64_t)b.Ksum * b.D);
    unsigned init_blocks = (unsigned)((init_items + kThreads - 1) / kThreads);
    if (init_blocks > 65536u) init_blocks = 65536u;
    if (init_blocks == 0) init_blocks = 1;
    if (c.iters == 0) a.it = -1;
    hipLaunchKernelGGL(big_init, dim3(init_blocks), dim3(kThreads), 0, st, a);
    if (c.iters == 0) return hipGetLastError();
    a.it = 0;

    const unsigned tile_blocks = (unsigned)((c.max_tiles + kWaves - 1) / kWaves);
    const unsigned row_blocks = (unsigned)(((size_t)b.G * w.kpad + kWaves - 1) / kWaves);
    const unsigned chunk_blocks = (unsigned)w.max_chunks;
    const size_t lds = (size_t)kGroupTiles * ds * 2 * 64 * 16 + (size_t)4 * kGroupTiles * 64 * 8 +
                       (size_t)kListCap * (16 + 4) + 16;
    // the vector-ALU scorer stages a search's centroids in LDS instead
    const size_t lds_valu = (size_t)w.kpad * (16 * ds + 1) * 4 + (size_t)kTilesPerChunk * 32 * 4 + 16;
    if (lds > 160 * 1024 || lds_valu > 160 * 1024) return hipErrorInvalidValue;
    const bool valu = c.scorer == KB_SCORER_VECTOR_ALU;
    const dim3 upd_grid((unsigned)((b.N + kUpdateRange - 1) / kUpdateRange),
                        (unsigned)((a.Kmax + kRowsPerGroup - 1) / kRowsPerGroup));

#define KB_BIG(DS_)                                                                              \
    do {                                                                                         \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(big_score<DS_>),        \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                           \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(big_score_valu<DS_>),              \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_valu);      \
        if (e != hipSuccess) return e;                                                           \
        if (tile_blocks) hipLaunchKernelGGL(big_presplit<DS_>, dim3(tile_blocks), dim3(kThreads), 0, st, a); \
        for (int it = 0; it < c.iters; ++it) {                                                   \
            a.it = it;                                                                           \
            /* the two assignment buffers swap roles; the last step writes the caller's */       \
            const bool mine = ((c.iters - 1 - it) & 1) == 0;                                     \
            a.next = mine ? c.assign : other;                                                    \
            a.prev = mine ? other : c.assign;                                                    \
            hipLaunchKernelGGL(big_renew<DS_>, dim3(row_blocks), dim3(kThreads), 0, st, a);      \
            if (valu)                                                                            \
                hipLaunchKernelGGL(big_score_valu<DS_>, dim3(chunk_blocks), dim3(kThreads),      \
                                   lds_valu, st, a);                                             \
            else                                                                                 \
                hipLaunchKernelGGL(big_score<DS_>, dim3(chunk_blocks), dim3(kThreads), lds, st, a); \
            hipLaunchKernelGGL(big_exact, dim3(kFewBlocks + kFullBlocks), dim3(kThreads), 0, st, a); \
            hipLaunchKernelGGL(big_update, upd_grid, dim3(kThreads), 0, st, a);                  \
        }                                                                                        \
        hipLaunchKernelGGL(big_objfast, dim3((unsigned)b.G), dim3(kObjThreads), 0, st, a);       \
        hipLaunchKernelGGL(big_objective, dim3(chunk_blocks), dim3(kThreads), 0, st, a);         \
        hipLaunchKernelGGL(big_objsum, dim3((unsigned)b.G), dim3(kThreads), 0, st, a);           \
        a.final_pass = 1;                                                                        \
        hipLaunchKernelGGL(big_renew<DS_>, dim3(row_blocks), dim3(kThreads), 0, st, a);          \
    } while (0)
    switch (ds) {
        case 1: KB_BIG(1); break;
        case 2: KB_BIG(2); break;
        case 3: KB_BIG(3); break;
        default: KB_BIG(4); break;
    }
#undef KB_BIG
    return hipGetLastError();
}

}  // namespace kb
