// K-Means (Lloyd) clustering of the behavioural feature vectors (Sec. 3.3;
// L2 norm of Assumption 2 / Eq. 3): one workgroup owns one search and runs all
// of its Lloyd steps, so the search's rows stay in L2 / Infinity Cache between
// steps and the centroids never leave LDS.
//
// Every scoring splits the fp32 feature rows it fetches into bf16 (hi, mid) pieces
// on the fly; |x|^2, the cluster and the drift limit of every candidate share one
// workspace array of 8 bytes per candidate.  (Batches of very short searches run
// one wave per search instead: cluster_wave_kernel at the end of this file.)
//
// One step:
//
//   bounds     (default mode) every scored candidate leaves a limit: the
//              cumulative drift of its cluster (its centroid's moves plus the
//              largest move of another centroid) at that time plus the gap
//              between the distance to its centroid and to the nearest other
//              one.  While that drift stays below the limit the candidate
//              provably keeps its cluster and is not scored; the others are
//              packed into dense tiles of 32.
//   A  score   fast scores s_j = |c_j|^2 - 2 x.c_j for every centroid, the best
//              and second-best per candidate, and a proved error bound E.
//              If second - best > 2E the winner is certain; otherwise the
//              candidate is listed for exact re-evaluation.  Two scorers:
//              matrix cores (bf16 x 3 split products, fp32 accumulate) for
//              K <= 64, a vector-ALU fp32 FMA chain otherwise.
//   R  refine  listed candidates get their squared distances in fp64, direct
//              difference form, summed over the features in index order with
//              separate multiply and add - exactly the plain definition - and
//              the lowest index attaining the minimum wins.
//   B  update  only candidates whose cluster changed touch the running sums:
//              their features are converted to 64-bit fixed point and moved
//              from the old to the new cluster with integer LDS atomics.
//              Integer addition commutes, so the sums (and with them the new
//              centroids) do not depend on the order the waves run in: results
//              are bit-identical from run to run without any sorting.  The
//              matrix-core scorer does this itself for the candidates it is
//              certain about.
//
// New centroid = (fixed-point sum / 2^shift) / count in fp64, rounded once to
// fp32; an empty cluster keeps its centroid.
#include "kb_cluster_dev.h"
#include "kb_ucb_dev.h"

namespace kb {

namespace {

struct ClusterArgs {
    int G, D, Ksum, Kmax, Nmax;
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
    int use_bounds;
    int guard;         // leave searches with N_g < 2 K_g as they are (re-clustering rule of Alg. 1)
    int mixed;         // leave searches of the multi-workgroup path (K_g > 64 or N_g > limit_n) alone
    int limit_n;       // most candidates of a search this kernel takes in this batch
    float2* lim;       // [N] state of every candidate: .x its drift limit (drift at its last scoring + its
                       //     slack) with its cluster + 1 in the 7 lowest bits, .y its |x|^2
};

// Threads per workgroup (a template parameter NT of the kernel and of the device
// functions that stride by it): 256, three workgroups per compute unit, is the
// shape of large batches; a batch with fewer searches than compute units runs 768,
// so that a lone search still fills the unit it is on.
constexpr int kThreadsNarrow = 256, kThreadsWide = 768;
constexpr int kWideMaxG = 256;     // most searches of a batch that takes the wide shape
constexpr int kFlagCap = 256;      // LDS list of candidates waiting for the exact pass
constexpr int kMoverBatch = 8;     // movers whose rows are requested together
constexpr int kQueue = 128;        // per wave: candidates waiting to be scored (at most 31 + 64 at a time)

// Cross-lane steps inside rows of 16 lanes (data-parallel primitives: no LDS
// traffic): lanes 1,0,3,2 and 2,3,0,1 of every four, then mirrors inside every
// eight and every sixteen.  After the four steps every lane of a row holds the
// row's result; rows are combined through scalar registers.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
    const long long b = __double_as_longlong(v);
    const int lo = (int)(unsigned)b, hi = (int)(b >> 32);
    const unsigned lo2 = (unsigned)__builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
    const unsigned hi2 = (unsigned)__builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
    return __longlong_as_double((long long)(((unsigned long long)hi2 << 32) | lo2));
}
__device__ __forceinline__ float row_max_f(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
__device__ __forceinline__ float row_min_f(float v) {
    v = fminf(v, dpp_f<0xB1>(v));
    v = fminf(v, dpp_f<0x4E>(v));
    v = fminf(v, dpp_f<0x141>(v));
    v = fminf(v, dpp_f<0x140>(v));
    return v;
}
// sum over the 16 lanes of a row, in a fixed order, delivered to all 16
__device__ __forceinline__ double row_sum_d(double v) {
    v += dpp_d<0xB1>(v);
    v += dpp_d<0x4E>(v);
    v += dpp_d<0x141>(v);
    v += dpp_d<0x140>(v);
    return v;
}
__device__ __forceinline__ float lane_f(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ double lane_d(double v, int l) {
    const long long b = __double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, l);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(b >> 32), l);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ float wave_max_f(float v) {
    v = row_max_f(v);
    return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ __forceinline__ float wave_min_f(float v) {
    v = row_min_f(v);
    return fminf(fminf(lane_f(v, 0), lane_f(v, 16)), fminf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ __forceinline__ double wave_sum_d(double v) {
    v = row_sum_d(v);
    return (lane_d(v, 0) + lane_d(v, 16)) + (lane_d(v, 32) + lane_d(v, 48));
}

// Block-wide reductions over the NW waves of a workgroup.  `red` is LDS scratch of
// 2 * NW doubles used as two alternating slots (`phase` counts the calls,
// identically in every thread), so one barrier per reduction is enough: a slot
// is rewritten only after another reduction's barrier has passed.  Every thread
// gets the result; per-wave values are combined in a fixed order.
template <int NW>
__device__ __forceinline__ float block_max_f(float v, double* red, int& phase) {
    float* slot = reinterpret_cast<float*>(red + (phase++ & 1) * NW);
    v = wave_max_f(v);
    if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = slot[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = fmaxf(r, slot[w]);
    return r;
}
template <int NW>
__device__ __forceinline__ double block_sum_d(double v, double* red, int& phase) {
    double* slot = red + (phase++ & 1) * NW;
    v = wave_sum_d(v);
    if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = slot[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r += slot[w];
    return r;
}
// bitwise OR of the two low bits of v over the block
template <int NW>
__device__ __forceinline__ int block_or_i(int v, double* red, int& phase) {
    int* slot = reinterpret_cast<int*>(red + (phase++ & 1) * NW);
    v = (__any(v & 1) ? 1 : 0) | (__any(v & 2) ? 2 : 0);
    if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) r |= slot[w];
    return r;
}

__device__ __forceinline__ void lds_add(long long* p, long long q) {
    atomicAdd(reinterpret_cast<unsigned long long*>(p), (unsigned long long)q);
}

// ---- phase A, vector-ALU scorer ---------------------------------------------
// One candidate per lane with its (zero-padded) feature row in registers; the
// centroids are broadcast from LDS.  Error bound of a score, with u = 2^-24,
// dot accumulated by a chain of D fused multiply-adds and s = fma(-2, dot, cn):
//   |s' - s| <= (D + 3) u (1 + o(1)) (|x|^2 + max_j |c_j|^2)
// (2 gamma_D |x||c| <= gamma_D (|x|^2+|c|^2) for the dot, u(|c|^2 + 2|x||c|) for
// the final rounding, u |c|^2 for the rounded norm).  kappa = (D + 4) u leaves
// room for the rounding of |x|^2, of E itself and of the gap.
template <int DV4, int NT>
__device__ __forceinline__ void score_valu(const ClusterArgs& a, const float* __restrict__ Xg,
                                           int n0, int ng, int K, int D, int DP,
                                           const float* cent, const float* cn, float cnmax) {
    const float kappa = (float)(D + 4) * 5.9604644775390625e-08f;
    const bool vec = (D & 3) == 0;
    for (int p = threadIdx.x; p < ng; p += NT) {
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

// ---- phase A, matrix-core scorer --------------------------------------------
// v_mfma_f32_32x32x16_bf16 computes a 32 x 32 tile of scores: rows = centroids,
// columns = candidates, contraction over 16 features.  Lane l supplies, for row
// or column l%32, the 8 features 8*(l/32) .. +7 of the K-step, and receives the
// 16 scores of column l%32 in rows 8*(r/4) + 4*(l/32) + r%4.
//
// fp32 operands are split into bf16 pieces v = hi + mid + rest (hi = bf16(v),
// mid = bf16(v - hi), both round-to-nearest-even, |rest| <= 2^-16 |v|) and the
// three leading products hi*hi + hi*mid + mid*hi are accumulated in fp32 on top
// of |c_j|^2, with the factor -2 folded into the centroid operand (exact).
// Error of a score against the real s_j = |c_j|^2 - 2 x.c_j:
//   dropped products  mid*mid, rest*x, c*rest   <= 3.05 * 2^-16 * 2 sum|c_d x_d|
//   fp32 accumulation of 3*Dpad products + |c|^2 <= (3 Dpad + 4) 2^-23 * (|c|^2 + 2 sum|c_d x_d|)(1+2^-7)
// and 2 sum|c_d x_d| <= |x|^2 + |c|^2, so
//   |s' - s| <= [3.1 * 2^-16 + (3 Dpad + 4) 2^-22] (|x|^2 + max_j |c_j|^2) = E.
// (One ulp, 2^-23, per accumulated term is assumed for the matrix core's
// internal summation, twice what round-to-nearest would give.)
//
// The centroid operands and |c_j|^2 (in accumulator layout) are read from LDS;
// a wave walks over tiles of 32 candidates.  Candidates the scorer is certain
// about and whose cluster changed are moved between the fixed-point sums right
// here (their fp32 row is read again; rare after the first steps).
// No bf16 copy of the features is kept: a later step fetches a candidate's fp32 row
// again (its D * 4 bytes are contiguous, so a packed tile of candidates from all over
// the search moves the bytes of those candidates only) and splits it in registers.
// An operand-ordered copy - the pieces of 32 neighbours interleaved, as the matrix
// cores read them - made a tile in which a few candidates are at risk pull in most of
// its cache lines (9.2 GB of HBM traffic on the largest benchmark against 7.1 GB for a
// candidate-major copy), and writing any copy costs more than converting again.
// Everything that follows a change of a centroid, four lanes per row: the new centroid (fixed-point sum / 2^shift) / count in
// fp64, rounded once to fp32; how far it moved (rounded up); |c_j|^2 in fp64; and
// the matrix cores' operands -2 c_j split into bf16 (hi, mid), stored in LDS in
// operand order [tile of 32 rows][16-feature step][hi|mid][lane] x 16 bytes so the
// scorer reads them with conflict-free 16-byte loads.  Only rows whose membership
// changed are touched (`init`: every row, nothing renewed; rows >= K get zero
// operands).  Returns this thread's view of max_j |c_j|^2.
// fp32 rounding of the correctly rounded fp64 quotient t / c, from one reciprocal
// rc = 1 / c shared by a row's features.  t * rc lies within 2^-52 (relative) of
// t / c, and so does the rounded quotient; the two round to the same fp32 unless
// an fp32 rounding boundary - a 1 followed by 28 zeros in the low 29 mantissa
// bits - lies within 2^-51 (at most 4 units of the last place) of t * rc.  Then,
// and for results near the subnormal fp32 range where the boundaries sit
// elsewhere, the quotient itself is formed.
__device__ __forceinline__ float mean_f32(double t, double c, double rc) {
    const double q = t * rc;
    const unsigned low = (unsigned)__double_as_longlong(q) & 0x1fffffffu;
    const unsigned off = low - 0x10000000u + 8u;
    if (off <= 16u || (fabs(q) < 0x1p-100 && t != 0.0)) return (float)(t / c);
    return (float)q;
}

// (Four lanes per row, lane q owning the 4-feature chunks q, q + 4, ...: all 64 rows of a
// search are renewed in one pass, so a step pays this dependent chain - reciprocal,
// means, fp64 sums across the four lanes, square root, operand conversion - once and
// not once per group of sixteen rows.)
__device__ __forceinline__ double quad_sum_d(double v) {
    v += dpp_d<0xB1>(v);
    v += dpp_d<0x4E>(v);
    return v;
}

template <int DS, bool OPERANDS, int NT>
__device__ __forceinline__ float renew_rows(float* cent, float* cn, bf16x8* aop, const long long* sums,
                                            const int* cnt, unsigned char* dirty, float* delta, int K, int D,
                                            int SP, double inv, bool init, bool need_scores,
                                            int tid_in = -1) {
    constexpr int DP = 16 * DS + 4;
    // (the caller's number among the NT threads that share the rows: the thread number in
    // the workgroup unless a single wave works on rows of its own)
    const int tid = tid_in >= 0 ? tid_in : (int)threadIdx.x, q = tid & 3;
    const int rows = init && OPERANDS ? ((K + 31) & ~31) : K;
    float cm = 0.f;
    for (int j0 = 0; j0 < rows; j0 += NT / 4) {
        const int j = j0 + (tid >> 2);
        const bool real = j < K;
        const int c = real ? cnt[j] : 0;
        const bool renew = !init && real && c > 0 && dirty[j] != 0;
        const bool fresh = renew || (init && j < rows);
        float4 v[DS];
#pragma unroll
        for (int i = 0; i < DS; ++i) {
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (real) v[i] = *reinterpret_cast<const float4*>(cent + (size_t)j * DP + 4 * (q + 4 * i));
        }
        double mv = 0.0;
        if (renew) {
            const double cd = (double)c, rc = 1.0 / cd;
#pragma unroll
            for (int i = 0; i < DS; ++i) {
                const int d0 = 4 * (q + 4 * i);
                float* vp = &v[i].x;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (d0 + e < D) {
                        const float cnew = mean_f32((double)sums[(size_t)j * SP + d0 + e] * inv, cd, rc);
                        const double df = (double)cnew - (double)vp[e];
                        mv += df * df;
                        vp[e] = cnew;
                    }
                }
                *reinterpret_cast<float4*>(cent + (size_t)j * DP + d0) = v[i];
            }
        }
        // uniform over the four lanes of a row from here on
        if (!init) {
            mv = quad_sum_d(mv);
            if (real && q == 0) {
                // rounded up: the fp32 square root is within 2^-23 of the true one
                delta[j] = !renew ? 0.f
                           : mv < 1.0e-30 ? (float)sqrt(mv) * 1.0000005f
                                          : sqrtf((float)mv) * 1.0000005f;
                dirty[j] = 0;
            }
        }
        float f = 0.f;
        if (need_scores) {
            if (fresh) {
                double sq = 0.0;
#pragma unroll
                for (int i = 0; i < DS; ++i)
                    sq += (double)v[i].x * (double)v[i].x + (double)v[i].y * (double)v[i].y +
                          (double)v[i].z * (double)v[i].z + (double)v[i].w * (double)v[i].w;
                sq = quad_sum_d(sq);
                f = (float)sq;
                if (real && q == 0) cn[j] = f;
                if constexpr (OPERANDS) {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    const int mt = j >> 5;
#pragma unroll
                    for (int i = 0; i < DS; ++i) {
                        // chunk ch holds features 4 ch .. 4 ch + 3: half of the 8-feature piece ch / 2
                        const int ch = q + 4 * i;
                        const float w[4] = {-2.f * v[i].x, -2.f * v[i].y, -2.f * v[i].z, -2.f * v[i].w};
                        bf16x4 hi, mid;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const __bf16 hb = (__bf16)w[e];
                            hi[e] = hb;
                            mid[e] = (__bf16)(w[e] - (float)hb);
                        }
                        const int piece = ch >> 1, st = piece >> 1, hh = piece & 1;
                        const int ln = (j & 31) + 32 * hh;
                        bf16x4* e2 = reinterpret_cast<bf16x4*>(aop + ((mt * DS + st) * 2 + 0) * 64 + ln) + (ch & 1);
                        e2[0] = hi;
                        e2[64 * 2] = mid;           // the mid block follows 64 entries of 16 bytes later
                    }
                }
            } else if (real) {
                f = cn[j];
            }
            if (real) cm = fmaxf(cm, f);
        }
    }
    return cm;
}

// Distance bounds.  When a candidate is scored, ub >= distance to its nearest
// centroid b and lb <= distance to every other centroid are known; its slack is
// lb - ub.  If afterwards the centroids move, b gets at most sum delta_b farther
// and any other centroid at most sum (largest move of a centroid other than b)
// closer.  So while
//     slack > T_b = sum over the steps since scoring of
//                   (delta_b + largest move of another centroid)
// the candidate's nearest centroid is unchanged and strictly nearest.  Two clocks
// are kept, both rounded up at every step: the drift of every cluster, T_j, and
// the drift of the search, sum of (largest + second largest move), which no T_j
// outruns.  A candidate's limit is T_b at its scoring + its slack, rounded down,
// and is tested against T_b; a tile of 32 candidates keeps one number in LDS in
// the search's clock - the smallest of (drift + what a candidate has left) - so a
// tile whose number still exceeds the drift is not scored, not fetched and its
// limits not even read.
__device__ __forceinline__ float slack_of(float best, float second, float xn, float E) {
    // A >= d_best^2 and B <= d_other^2 (room for the rounding of |x|^2 included), and
    // sqrt(B) - sqrt(A) = (B - A) / (sqrt(B) + sqrt(A)): two square roots and a
    // reciprocal, each good to an ulp, the result rounded down by far more than their
    // errors add up to.  (The cheaper (B - A) / (2 sqrt(B)) is a lower bound too, but up
    // to half as large: 3 % more candidates were scored with it.)
    const float Eb = E + 4.0e-6f * xn;
    const float A = fmaxf(best + xn + Eb, 0.f);
    const float B = second + xn - Eb;
    const float sl = (B - A) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(B) + __builtin_amdgcn_sqrtf(A)) * 0.999998f;
    return B > A ? sl : 0.f;
}
// minimum over lanes 0..31, delivered to every lane of the wave
__device__ __forceinline__ float half_wave_min_f(float v) {
    v = row_min_f(v);
    return fminf(lane_f(v, 0), lane_f(v, 16));
}
// drift + slack, rounded down (both non-negative)
__device__ __forceinline__ float tile_limit(float drift, float slack) {
    return (drift + slack) * 0.9999995f;
}
// A candidate's limit shares its word with the candidate's cluster: cluster + 1 in the 7
// lowest mantissa bits (0: none yet), which rounds the non-negative limit down by less
// than 2^-16 of itself.  The wave that finds a tile at risk reads the tile's words in one
// coalesced piece; the lane that scores a candidate then finds cluster and |x|^2 next
// to a limit that is already in the caches, instead of two gathers of their own.
__device__ __forceinline__ float pack_limit(float L, int cluster) {
    return __uint_as_float((__float_as_uint(L) & ~127u) | (unsigned)(cluster + 1));
}
__device__ __forceinline__ float limit_of(float v) { return __uint_as_float(__float_as_uint(v) & ~127u); }
__device__ __forceinline__ int cluster_of(float v) { return (int)(__float_as_uint(v) & 127u) - 1; }

// Scores of one tile of 32 candidates (operands Bh, Bm) against the K <= 64
// centroids: best score, second best and the row of the best, the same in both
// half-waves.
template <int DS, int MT>
__device__ __forceinline__ void tile_scores(const bf16x8 (&Bh)[DS], const bf16x8 (&Bm)[DS],
                                            const float* cn, const bf16x8* aop, int mtiles,
                                            int lane, float& best, float& second, int& bi) {
    const int h = lane >> 5;
    // Accumulators start at |c_j|^2 (padded with a huge value for rows >= K),
    // read from LDS in accumulator layout.  Two accumulators are always in
    // flight so that consecutive matrix instructions never depend on each
    // other: the two centroid tiles when there are two, otherwise the
    // hi*mid products are summed apart and added at the end.
    constexpr int NA = 2;
    f32x16 acc[NA];
    const bool two = MT == 2 && mtiles == 2;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
        const float4 c4 = *reinterpret_cast<const float4*>(cn + 8 * g4 + 4 * h);
        acc[0][4 * g4 + 0] = c4.x; acc[0][4 * g4 + 1] = c4.y;
        acc[0][4 * g4 + 2] = c4.z; acc[0][4 * g4 + 3] = c4.w;
    }
    if (two) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const float4 c4 = *reinterpret_cast<const float4*>(cn + 32 + 8 * g4 + 4 * h);
            acc[1][4 * g4 + 0] = c4.x; acc[1][4 * g4 + 1] = c4.y;
            acc[1][4 * g4 + 2] = c4.z; acc[1][4 * g4 + 3] = c4.w;
        }
        // the first tile of centroids is finished before the second one is started, so
        // that the vector unit can take its minimum while the matrix cores work on
        // the second
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            // centroid operands of this K-step, straight from LDS (operand order)
            const bf16x8 a0h = aop[((0 * DS + s) * 2 + 0) * 64 + lane];
            const bf16x8 a0m = aop[((0 * DS + s) * 2 + 1) * 64 + lane];
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, Bh[s], acc[0], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, Bm[s], acc[0], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0m, Bh[s], acc[0], 0, 0, 0);
        }
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            const bf16x8 a1h = aop[((1 * DS + s) * 2 + 0) * 64 + lane];
            const bf16x8 a1m = aop[((1 * DS + s) * 2 + 1) * 64 + lane];
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, Bh[s], acc[1], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, Bm[s], acc[1], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1m, Bh[s], acc[1], 0, 0, 0);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[1][r] = 0.f;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            const bf16x8 a0h = aop[((0 * DS + s) * 2 + 0) * 64 + lane];
            const bf16x8 a0m = aop[((0 * DS + s) * 2 + 1) * 64 + lane];
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, Bh[s], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, Bm[s], acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0m, Bh[s], acc[0], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] += acc[1][r];
    }
    // Best and second best among this lane's rows with three vector instructions per
    // score: the score's position replaces its 5 lowest mantissa bits (which moves
    // it by less than 2^-18 of itself - part of the error bound), then a
    // median-of-three and a minimum; the row of the best is read back from those
    // bits.  Two independent chains; the lane-dependent part of the row number
    // (4h) is added afterwards.
    float cb[2] = {kBig * 8.f, kBig * 8.f}, cs[2] = {kBig * 8.f, kBig * 8.f};
    if (two) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v = __uint_as_float((__float_as_uint(acc[t][r]) & 0xffffffe0u) | (unsigned)(16 * t + r));
                cs[t] = __builtin_amdgcn_fmed3f(cb[t], cs[t], v);
                cb[t] = vmin(cb[t], v);
            }
            if (t == 0) {
                // one matrix instruction of the second tile to five vector instructions of
                // the first tile's minimum
#pragma unroll
                for (int q = 0; q < 3 * DS; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                }
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = r & 1;
            const float v = __uint_as_float((__float_as_uint(acc[0][r]) & 0xffffffe0u) | (unsigned)r);
            cs[c] = __builtin_amdgcn_fmed3f(cb[c], cs[c], v);
            cb[c] = vmin(cb[c], v);
        }
    }
    auto merge = [](float& b1, float& s1, int& i1, float b2, float s2, int i2) {
        const bool take = b2 < b1;
        const float hi2 = take ? b1 : b2;        // the larger of the two bests
        const float sm = s2 < s1 ? s2 : s1;
        s1 = sm < hi2 ? sm : hi2;
        i1 = take ? i2 : i1;
        b1 = take ? b2 : b1;
    };
    best = vmin(cb[0], cb[1]);
    second = vmin(vmin(cs[0], cs[1]), vmax(cb[0], cb[1]));
    {
        const int code = (int)(__float_as_uint(best) & 31u);
        bi = (code >> 4) * 32 + 8 * ((code & 15) >> 2) + (code & 3) + 4 * h;
    }
    // the two half-waves hold complementary centroid rows of the same
    // candidate: one lane-swap per value hands both halves both results
    {
        const auto rb = __builtin_amdgcn_permlane32_swap(__float_as_uint(best), __float_as_uint(best), false, false);
        const auto rs = __builtin_amdgcn_permlane32_swap(__float_as_uint(second), __float_as_uint(second), false, false);
        const auto ri = __builtin_amdgcn_permlane32_swap((unsigned)bi, (unsigned)bi, false, false);
        float b0 = __uint_as_float(rb[0]), s0 = __uint_as_float(rs[0]);
        int i0 = (int)ri[0];
        merge(b0, s0, i0, __uint_as_float(rb[1]), __uint_as_float(rs[1]), (int)ri[1]);
        best = b0; second = s0; bi = i0;
    }
}

// A later step on the matrix-core path, with the candidates that have to be
// scored packed into dense tiles.  Every candidate carries its own limit (drift at scoring time + slack)
// in `lim`; a tile's number in `thr` is the smallest limit of its candidates.  A
// wave walks its tiles whose number the drift has reached, two at a time (one
// per half-wave), reads their candidates' limits, and appends those the drift has
// reached to a small queue in LDS; whenever 32 are waiting they are scored as one
// tile of the matrix instruction, each lane fetching its own candidate's fp32 row
// (in 16-byte pieces when D is a multiple of 4) and splitting it into the bf16
// operands in registers.  A tile in which a third of the candidates are at risk
// thus costs a third of a scoring instead of a whole one.
template <int DS, int MT, int NT, bool VEC>
__device__ __forceinline__ int score_packed(const ClusterArgs& a, const float* __restrict__ Xg,
                                            int n0, int ng, int K, int D, int DP, int SP,
                                            const float* cent, const float* cn, float cnmax,
                                            int fsh, long long* sums, int* cnt,
                                            int* nflag, unsigned short* flist, const bf16x8* aop, unsigned char* dirty,
                                            float* thr, float2* __restrict__ lim,
                                            unsigned short* queue, float drift, float T) {
    const int lane = threadIdx.x & 63, wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform)
    const int m = lane & 31, h = lane >> 5;
    const int mtiles = (K + 31) >> 5;
    const float kappa = mfma_kappa(DS);
    constexpr int kWaves = NT / kWave;
    const int ntiles = (ng + 31) >> 5;
    const int ntw = ntiles > wid ? (ntiles - wid + kWaves - 1) / kWaves : 0;   // tiles of this wave
    unsigned short* q = queue + wid * kQueue;
    unsigned head = 0, tail = 0;       // (uniform) the queue holds entries head .. tail - 1, modulo kQueue
    int any = 0;

    // Candidates that change cluster are moved between the fixed-point sums eight at
    // a time, lanes over features: their fp32 rows are read again (all requests
    // first), converted and moved.  An entry: candidate | new cluster << 16 |
    // (old cluster + 1) << 23.
    unsigned pend = 0;
    int ph = 0, pt = 0;                // (uniform) entries ph .. pt - 1 wait, in lanes (index & 63)
    const int lc = lane < D ? lane : 0;
    auto drain = [&](int n) __attribute__((always_inline)) {
        unsigned e[kMoverBatch];
        float xq[kMoverBatch];
#pragma unroll
        for (int u = 0; u < kMoverBatch; ++u)
            e[u] = (unsigned)__builtin_amdgcn_readlane((int)pend, (ph + (u < n ? u : 0)) & 63);
#pragma unroll
        for (int u = 0; u < kMoverBatch; ++u) xq[u] = Xg[(size_t)(e[u] & 0xffffu) * D + lc];
#pragma unroll
        for (int u = 0; u < kMoverBatch; ++u) {
            if (u < n) {                                   // uniform over the wave
                const int nb2 = (int)((e[u] >> 16) & 0x7fu);
                const int ob2 = (int)(e[u] >> 23) - 1;
                if (lane < D) {
                    const long long qf = to_fixed(xq[u], fsh);
                    lds_add(&sums[(size_t)nb2 * SP + lane], qf);
                    if (ob2 >= 0) lds_add(&sums[(size_t)ob2 * SP + lane], -qf);
                }
            }
        }
        ph += n;
    };

    // scores the first `count` (<= 32) candidates of the queue
    auto chunk = [&](int count) __attribute__((always_inline)) {
        const bool valid = m < count;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");      // the other lanes' queue entries
        const int p = q[(head + (valid ? m : 0)) & (kQueue - 1)];
        bf16x8 Bh[DS], Bm[DS];
        {
            // The operands are split from the candidate's fp32 row as it is fetched (all
            // requests first): a row is contiguous, so a packed chunk moves the bytes of
            // its own candidates only, and no bf16 copy of the features has to be written
            // and kept (it cost more HBM traffic than the conversions cost issue slots).
            const float* xr = Xg + (size_t)p * D;
            float4 r0[DS], r1[DS];
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                const int d0 = 16 * s + 8 * h;
                r0[s] = make_float4(0.f, 0.f, 0.f, 0.f);
                r1[s] = r0[s];
                if constexpr (VEC) {
                    if (d0 < D) r0[s] = *reinterpret_cast<const float4*>(xr + d0);
                    if (d0 + 4 < D) r1[s] = *reinterpret_cast<const float4*>(xr + d0 + 4);
                } else {
                    if (d0 + 0 < D) r0[s].x = xr[d0 + 0];
                    if (d0 + 1 < D) r0[s].y = xr[d0 + 1];
                    if (d0 + 2 < D) r0[s].z = xr[d0 + 2];
                    if (d0 + 3 < D) r0[s].w = xr[d0 + 3];
                    if (d0 + 4 < D) r1[s].x = xr[d0 + 4];
                    if (d0 + 5 < D) r1[s].y = xr[d0 + 5];
                    if (d0 + 6 < D) r1[s].z = xr[d0 + 6];
                    if (d0 + 7 < D) r1[s].w = xr[d0 + 7];
                }
            }
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                const float xv[8] = {r0[s].x, r0[s].y, r0[s].z, r0[s].w, r1[s].x, r1[s].y, r1[s].z, r1[s].w};
                split8(xv, Bh[s], Bm[s]);
            }
        }
        const float2 state = lim[p];
        const float xn = state.y;
        int old = cluster_of(state.x);
        old = (valid && old >= 0 && old < K) ? old : -1;

        float best, second;
        int bi;
        tile_scores<DS, MT>(Bh, Bm, cn, aop, mtiles, lane, best, second, bi);
        bi = bi < K ? bi : 0;
        const float E = kappa * (xn + cnmax);
        // (a best score next to zero may have lost its position bits to a flush of
        // subnormal numbers: that candidate goes to the exact pass)
        const bool certain = (K == 1) || (((second - best) > 2.f * E) && fabsf(best) > 1.0e-30f);
        const bool chg = valid && certain && (bi != old);
        unsigned rem = (unsigned)__ballot(chg && h == 0);
        if (rem) {
            any |= 1;
            if (chg && h == 0) {
                atomicAdd(&cnt[bi], 1);
                dirty[bi] = 1;
                if (old >= 0) { atomicSub(&cnt[old], 1); dirty[old] = 1; }
                a.assign[(size_t)n0 + p] = bi;
            }
            // the movers wait in a register queue (one entry per lane of `pend`) until
            // eight of them can fetch their rows together
            const unsigned info = (unsigned)p | ((unsigned)bi << 16) | ((unsigned)(old + 1) << 23);
            while (rem) {
                const int mb = __ffs((int)rem) - 1;
                rem &= rem - 1;
                const unsigned e = (unsigned)__builtin_amdgcn_readlane((int)info, mb);
                pend = lane == (pt & 63) ? e : pend;
                ++pt;
            }
            while (pt - ph >= kMoverBatch) drain(kMoverBatch);
        }
        // the candidate's limit counts in its own cluster's drift, the tile's number in
        // the search's (which grows at least as fast)
        const float Tb = __shfl(T, bi);
        if (valid && h == 0) {
            if (!certain) {
                // (the exact pass sets cluster and limit of the candidates it decides)
                a.a_new[(size_t)n0 + p] = bi | kFlagBit;
                const int pos = atomicAdd(nflag, 1);
                if (pos < kFlagCap) flist[pos] = (unsigned short)p;     // (N_g <= 65536 on this path)
            } else {
                const float sl = slack_of(best, second, xn, E);
                lim[p].x = pack_limit(a.use_bounds ? tile_limit(Tb, sl) : 0.f, bi);
                if (a.use_bounds)
                    atomicMin(reinterpret_cast<unsigned*>(&thr[p >> 5]), __float_as_uint(tile_limit(drift, sl)));
            }
        }
        if (__any(valid && !certain)) any |= 2;
    };

    for (int i0 = 0; i0 < ntw; i0 += 64) {
        const int nb = ntw - i0 < 64 ? ntw - i0 : 64;
        unsigned long long act = nb == 64 ? ~0ull : ((1ull << nb) - 1ull);
        if (a.use_bounds) {
            const int ti = wid + kWaves * (i0 + lane);
            act = __ballot(lane < nb && !(thr[ti] > drift));
        }
        act = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(act >> 32)) << 32) |
              (unsigned)__builtin_amdgcn_readfirstlane((int)act);
        // the next two tiles to look at, one for each half-wave, and this lane's
        // candidate in them; its limit is requested one pair ahead
        // (no branch around the request: with none left it reads the first limit again)
        auto take_pair = [&](bool& have, int& c0, int& c1, int& p, bool& in, float& lv) {   // lv: the raw state word
            have = act != 0;
            c0 = have ? __ffsll((long long)act) - 1 : 0;
            act &= act - 1;
            c1 = act ? __ffsll((long long)act) - 1 : -1;
            act &= act - 1;
            const int myc = h ? c1 : c0;
            const int tl = wid + kWaves * (i0 + (myc >= 0 ? myc : c0));
            p = tl * 32 + m;
            in = have && myc >= 0 && p < ng;
            lv = lim[in ? p : 0].x;
        };
        bool have, in;
        int c0, c1, p;
        float lv;
        take_pair(have, c0, c1, p, in, lv);
        while (have) {
            bool haven, inn;
            int c0n, c1n, pn;
            float lvn;
            take_pair(haven, c0n, c1n, pn, inn, lvn);
            bool active = in;
            if (a.use_bounds) {
                // at risk once the drift of the candidate's own cluster has reached its limit
                const int cl = cluster_of(lv);
                const float Ta = __shfl(T, cl < 0 ? 0 : cl);
                const float lc = limit_of(lv);
                active = in && !(lc > Ta);
                // what the tile's number becomes: the smallest of the limits of the
                // candidates that stay as they are, each restated in the search's drift
                // (drift now + what the candidate has left, rounded down; the scored ones
                // lower the number again)
                float keep = (in && !active) ? tile_limit(drift, (lc - Ta) * 0.9999995f) : INFINITY;
                keep = row_min_f(keep);
                const float k0 = vmin(lane_f(keep, 0), lane_f(keep, 16));
                const float k1 = vmin(lane_f(keep, 32), lane_f(keep, 48));
                if (lane == 0) thr[wid + kWaves * (i0 + c0)] = k0;
                if (lane == 32 && c1 >= 0) thr[wid + kWaves * (i0 + c1)] = k1;
            }
            const unsigned long long mask = __ballot(active);
            if (active) {
                const unsigned rank = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                          __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
                q[(tail + rank) & (kQueue - 1)] = (unsigned short)p;
            }
            tail += (unsigned)__popcll(mask);
            while (tail - head >= 32u) {
                chunk(32);
                head += 32u;
            }
            c0 = c0n; c1 = c1n; p = pn; in = inn; lv = lvn; have = haven;
        }
    }
    if (tail != head) chunk((int)(tail - head));
    if (pt != ph) drain(pt - ph);
    return any;   // bit 0: some candidate moved, bit 1: some candidate needs the exact pass
}

// First step of a call on the matrix-core path.  One pass over the fp32 rows:
// they are split into bf16 (hi, mid) operands, scored from the registers that
// hold them, and - every candidate joins a cluster in the first step - added to
// the fixed-point sums from the same registers; |x|^2 and the drift limit of every
// candidate go to the workspace for the steps that follow.  Returns max |x| over the rows this thread saw in
// `am_out`, which the caller checks against the estimate the scale was taken from.
template <int DS, int MT, int NT, bool VEC>
__device__ __forceinline__ int score_first(const ClusterArgs& a, const float* __restrict__ Xg,
                                           int n0, int ng, int K, int D,
                                           int SP, const float* cn, float cnmax, int fsh,
                                           long long* sums, int* cnt, int* nflag, unsigned short* flist,
                                           const bf16x8* aop, unsigned char* dirty, float* thr,
                                           float2* __restrict__ lim, float& am_out, double& sq_out) {
    const int lane = threadIdx.x & 63, wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform)
    const int m = lane & 31, h = lane >> 5;
    const int mtiles = (K + 31) >> 5;
    const float kappa = mfma_kappa(DS);
    constexpr int kWaves = NT / kWave;
    const int ntiles = (ng + 31) >> 5;
    // |x|^2 and the limits serve the steps that follow: a call of one step
    // (kb_cluster_step) stores none of them
    const bool later = a.iters > 1;

    // this lane's 8 features of every 16-feature step of row `tile * 32 + m`
    auto load_rows = [&](int tile, float4 (&r)[DS][2]) {
        const int p = tile * 32 + m;
        const bool valid = p < ng;
        const float* xr = Xg + (size_t)(valid ? p : 0) * D;
        if (VEC && D == 16 * DS && tile * 32 + 32 <= ng) {
            // (uniform) a whole tile of rows without padding: nothing to guard
#pragma unroll
            for (int s = 0; s < DS; ++s) {
                r[s][0] = *reinterpret_cast<const float4*>(xr + 16 * s + 8 * h);
                r[s][1] = *reinterpret_cast<const float4*>(xr + 16 * s + 8 * h + 4);
            }
            return;
        }
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            const int d0 = 16 * s + 8 * h;
            r[s][0] = make_float4(0.f, 0.f, 0.f, 0.f);
            r[s][1] = r[s][0];
            if constexpr (VEC) {
                if (valid && d0 < D) r[s][0] = *reinterpret_cast<const float4*>(xr + d0);
                if (valid && d0 + 4 < D) r[s][1] = *reinterpret_cast<const float4*>(xr + d0 + 4);
            } else if (valid) {
                if (d0 + 0 < D) r[s][0].x = xr[d0 + 0];
                if (d0 + 1 < D) r[s][0].y = xr[d0 + 1];
                if (d0 + 2 < D) r[s][0].z = xr[d0 + 2];
                if (d0 + 3 < D) r[s][0].w = xr[d0 + 3];
                if (d0 + 4 < D) r[s][1].x = xr[d0 + 4];
                if (d0 + 5 < D) r[s][1].y = xr[d0 + 5];
                if (d0 + 6 < D) r[s][1].z = xr[d0 + 6];
                if (d0 + 7 < D) r[s][1].w = xr[d0 + 7];
            }
        }
    };

    float am = 0.f;
    double sq = 0.0;          // sum of x^2 over this lane's features, exact products
    int any = 0;
    float4 cur[DS][2];
    for (int tile = wid; tile < ntiles; tile += kWaves) {
        load_rows(tile, cur);
        const int p = tile * 32 + m;
        const bool valid = p < ng;
        float xv[DS][8];
        bf16x8 Bh[DS], Bm[DS];
        float xn = 0.f;
#pragma unroll
        for (int s = 0; s < DS; ++s) {
            xv[s][0] = cur[s][0].x; xv[s][1] = cur[s][0].y; xv[s][2] = cur[s][0].z; xv[s][3] = cur[s][0].w;
            xv[s][4] = cur[s][1].x; xv[s][5] = cur[s][1].y; xv[s][6] = cur[s][1].z; xv[s][7] = cur[s][1].w;
            split8(xv[s], Bh[s], Bm[s]);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                xn = fmaf(xv[s][i], xv[s][i], xn);
                am = fmaxf(am, fabsf(xv[s][i]));
                sq = fma((double)xv[s][i], (double)xv[s][i], sq);
            }
        }
        xn += __shfl_xor(xn, 32);

        float best, second;
        int bi;
        tile_scores<DS, MT>(Bh, Bm, cn, aop, mtiles, lane, best, second, bi);
        bi = bi < K ? bi : 0;
        const float E = kappa * (xn + cnmax);
        // (a best score next to zero may have lost its position bits to a flush of
        // subnormal numbers: that candidate goes to the exact pass)
        const bool certain = (K == 1) || (((second - best) > 2.f * E) && fabsf(best) > 1.0e-30f);
        const bool chg = valid && certain;
        const unsigned long long cmask = __ballot(chg && h == 0);
        if (cmask) {
            any |= 1;
            if (chg) {
                long long* srow = sums + (size_t)bi * SP + 8 * h;
                if (D == 16 * DS) {         // (uniform) no feature is padding
#pragma unroll
                    for (int s = 0; s < DS; ++s) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) lds_add(srow + 16 * s + i, to_fixed(xv[s][i], fsh));
                    }
                } else {
#pragma unroll
                    for (int s = 0; s < DS; ++s) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            if (16 * s + 8 * h + i < D) lds_add(srow + 16 * s + i, to_fixed(xv[s][i], fsh));
                        }
                    }
                }
                if (h == 0) {
                    atomicAdd(&cnt[bi], 1);
                    dirty[bi] = 1;
                    a.assign[(size_t)n0 + p] = bi;
                }
            }
        }
        if (valid && h == 0) {
            a.a_new[(size_t)n0 + p] = certain ? bi : (bi | kFlagBit);
            if (!certain) {
                // left to the exact pass: no cluster yet
                a.assign[(size_t)n0 + p] = -1;
                const int pos = atomicAdd(nflag, 1);
                if (pos < kFlagCap) flist[pos] = (unsigned short)p;     // (N_g <= 65536 on this path)
            }
        }
        if (__any(valid && !certain)) any |= 2;
        if (later) {
            // state of the candidate for the later steps (no cluster yet for the ones left
            // to the exact pass, which then sets it)
            const float own = (valid && certain && a.use_bounds) ? slack_of(best, second, xn, E) : INFINITY;
            if (valid && h == 0)
                lim[p] = make_float2(certain ? pack_limit(a.use_bounds ? tile_limit(0.f, own) : 0.f, bi)
                                             : pack_limit(0.f, -1), xn);
            if (a.use_bounds) {
                const float sl = half_wave_min_f(own);
                if (lane == 0) thr[tile] = limit_of(tile_limit(0.f, sl));
            }
        }
    }
    am_out = am;
    sq_out = sq;
    return any;
}

// ---- phase R -----------------------------------------------------------------
// Exact nearest centroid of the marked candidates: lanes take centroids, each
// lane sums (x_d - c_d)^2 over d in index order in fp64 with separate multiply
// and add; the wave then reduces to the minimum, lowest index on ties.
template <int NT>
__device__ __forceinline__ void refine(const ClusterArgs& a, const float* __restrict__ Xg, int n0,
                                       int ng, int K, int D, int DP, const float* cent, bool mark) {
    const int lane = threadIdx.x & 63, wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform)
    for (int base = wid * kWave; base < ng; base += NT) {
        const int p = base + lane;
        const int v = p < ng ? a.a_new[(size_t)n0 + p] : 0;
        unsigned long long mask = __ballot(v < 0);
        while (mask) {
            const int b = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const float* xr = Xg + (size_t)(base + b) * D;
            // D <= 64: lane d holds feature d, broadcast by lane index below
            const float xv = lane < D ? xr[lane] : 0.f;
            double bd = INFINITY;
            int bj = 0x7fffffff;
            for (int j0 = 0; j0 < K; j0 += kWave) {
                const int j = j0 + lane;
                const float* cr = cent + (size_t)(j < K ? j : 0) * DP;
                // rows are zero-padded to a multiple of 4 features (and xv is 0 beyond
                // D), so whole float4 chunks can be summed: the extra terms are +0.0
                double acc = 0.0;
                for (int d = 0; d < D; d += 4) {
                    const float4 cv = *reinterpret_cast<const float4*>(cr + d);
                    double diff = __dsub_rn((double)__shfl(xv, d), (double)cv.x);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    diff = __dsub_rn((double)__shfl(xv, d + 1), (double)cv.y);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    diff = __dsub_rn((double)__shfl(xv, d + 2), (double)cv.z);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    diff = __dsub_rn((double)__shfl(xv, d + 3), (double)cv.w);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                }
                if (j < K && acc < bd) { bd = acc; bj = j; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double od = __shfl_xor(bd, o);
                const int oj = __shfl_xor(bj, o);
                if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
            }
            // (mark: only the entries decided here are fresh, and `update` must tell them apart)
            if (lane == 0) a.a_new[(size_t)n0 + base + b] = (bj < K ? bj : 0) | (mark ? kRefinedBit : 0);
        }
    }
}

// ---- phases R + B over the list of marked candidates ----------------------------
// One wave per listed candidate, lanes over centroids; the next candidate's row
// is requested before the current one is worked on.  First every squared
// distance in fp32, direct differences: a sum of non-negative terms, so its
// relative error is at most (D + 2) 2^-24.  If the two smallest are further apart
// than twice that bound allows, the smallest is the unique nearest centroid.
// Otherwise the distances are formed exactly as the plain definition does - fp64,
// summed over the features in index order with separate multiply and add - and the
// lowest index attaining the minimum wins.  Then, if the nearest centroid differs
// from the recorded cluster, the row moves between the running sums.
template <int DS, int NT>
__device__ __forceinline__ int refine_listed(const ClusterArgs& a, const float* __restrict__ Xg,
                                             int n0, int n, const unsigned short* flist, int K, int D, int DP,
                                             int SP, const float* cent, int fsh,
                                             long long* sums, int* cnt, unsigned char* dirty, float* thr,
                                             float2* __restrict__ lim, float drift, float T) {
    const int lane = threadIdx.x & 63, wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform)
    const int lc = lane < D ? lane : 0;
    const float eps = 2.f * (float)(D + 2) * 5.9604644775390625e-08f;
    int any = 0;
    if (wid >= n) return 0;
    constexpr int W = NT / kWave;
    // the rows of this wave's next two candidates are always in flight (a row is one
    // register: lanes over features), so a step's few candidates cost one trip to
    // memory and not one each
    int p_n = flist[wid];
    float xv_n = Xg[(size_t)p_n * D + lc];
    int old_n = a.assign[(size_t)n0 + p_n];
    int p_m = flist[wid + W < n ? wid + W : wid];
    float xv_m = Xg[(size_t)p_m * D + lc];
    int old_m = a.assign[(size_t)n0 + p_m];
    for (int i = wid; i < n; i += W) {
        const int p = p_n;
        const float xv = lane < D ? xv_n : 0.f;
        int old = old_n;
        p_n = p_m; xv_n = xv_m; old_n = old_m;
        {
            // no branch around the loads (the last candidates request their own row again)
            const int i2 = i + 2 * W < n ? i + 2 * W : i;
            p_m = flist[i2];
            xv_m = Xg[(size_t)p_m * D + lc];
            old_m = a.assign[(size_t)n0 + p_m];
        }
        // rows are zero-padded to a multiple of 4 features (and xv is 0 beyond D), so
        // whole float4 chunks can be summed: the extra terms are +0.0
        float lb = INFINITY, ls = INFINITY;       // this lane's smallest and second smallest
        int lj = 0x7fffffff;
        for (int j0 = 0; j0 < K; j0 += kWave) {
            const int j = j0 + lane;
            const float* cr = cent + (size_t)(j < K ? j : 0) * DP;
            float acc0 = 0.f, acc1 = 0.f;
            // (feature numbers known at compile time: the row's values are read out of
            // their lanes into scalar registers, no cross-lane traffic through LDS)
#pragma unroll
            for (int d = 0; d < 16 * DS; d += 4) {
                if (d < D) {
                    const float4 cv = *reinterpret_cast<const float4*>(cr + d);
                    const float e0 = lane_f(xv, d) - cv.x, e1 = lane_f(xv, d + 1) - cv.y;
                    const float e2 = lane_f(xv, d + 2) - cv.z, e3 = lane_f(xv, d + 3) - cv.w;
                    acc0 = fmaf(e0, e0, acc0);
                    acc1 = fmaf(e1, e1, acc1);
                    acc0 = fmaf(e2, e2, acc0);
                    acc1 = fmaf(e3, e3, acc1);
                }
            }
            const float acc = acc0 + acc1;
            if (j < K) {
                if (acc < lb) { ls = lb; lb = acc; lj = j; }
                else if (acc < ls) ls = acc;
            }
        }
        const float b32 = wave_min_f(lb);
        const int fl = __ffsll((long long)__ballot(lb == b32)) - 1;
        const float s32 = wave_min_f(lane == fl ? ls : lb);
        int bj = __shfl(lj, fl);
        float ub, lbd;      // upper bound on the nearest distance, lower bound on all others
        if (s32 * (1.f - eps) > b32 * (1.f + eps) + 1.0e-35f) {     // uniform over the wave
            ub = sqrtf(b32 * (1.f + eps)) * 1.0000005f;
            lbd = sqrtf(s32 * (1.f - eps)) * 0.9999995f;
        } else {
            double bd = INFINITY, sd = INFINITY;
            bj = 0x7fffffff;
            for (int j0 = 0; j0 < K; j0 += kWave) {
                const int j = j0 + lane;
                const float* cr = cent + (size_t)(j < K ? j : 0) * DP;
                double acc = 0.0;
#pragma unroll
                for (int d = 0; d < 16 * DS; d += 4) {
                    if (d < D) {
                        const float4 cv = *reinterpret_cast<const float4*>(cr + d);
                        double diff = __dsub_rn((double)lane_f(xv, d), (double)cv.x);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)lane_f(xv, d + 1), (double)cv.y);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)lane_f(xv, d + 2), (double)cv.z);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)lane_f(xv, d + 3), (double)cv.w);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    }
                }
                if (j < K) {
                    if (acc < bd) { sd = bd; bd = acc; bj = j; }
                    else if (acc < sd) sd = acc;
                }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double od = __shfl_xor(bd, o);
                const double os = __shfl_xor(sd, o);
                const int oj = __shfl_xor(bj, o);
                const bool take = od < bd || (od == bd && oj < bj);
                const double hi2 = take ? bd : od;        // the larger of the two bests
                const double sm = os < sd ? os : sd;
                sd = sm < hi2 ? sm : hi2;
                if (take) { bd = od; bj = oj; }
            }
            ub = (float)sqrt(bd) * 1.0000005f;
            lbd = (float)sqrt(sd) * 0.9999995f;
        }
        bj = bj < K ? bj : 0;
        const float Tb = __shfl(T, bj);
        if (lane == 0) {
            // the slack is the difference of the bounds, rounded down; limits are
            // non-negative floats, which order like their bit patterns
            const float sl = fmaxf((lbd - ub) * 0.9999995f, 0.f);
            lim[p].x = pack_limit(a.use_bounds ? tile_limit(Tb, sl) : 0.f, bj);
            if (a.use_bounds)
                atomicMin(reinterpret_cast<unsigned*>(&thr[p >> 5]), __float_as_uint(tile_limit(drift, sl)));
            a.a_new[(size_t)n0 + p] = bj;          // no longer waiting for the exact pass
        }
        old = (old >= 0 && old < K) ? old : -1;
        if (bj != old) {
            any = 1;
            if (lane < D) {
                const long long q = to_fixed(xv, fsh);
                lds_add(&sums[(size_t)bj * SP + lane], q);
                if (old >= 0) lds_add(&sums[(size_t)old * SP + lane], -q);
            }
            if (lane == 0) {
                atomicAdd(&cnt[bj], 1);
                dirty[bj] = 1;
                if (old >= 0) { atomicSub(&cnt[old], 1); dirty[old] = 1; }
                a.assign[(size_t)n0 + p] = bj;
            }
        }
    }
    return any;
}

// ---- phase B -----------------------------------------------------------------
// Move every candidate whose proposed cluster differs from its recorded one:
// lanes take features, one candidate at a time, so the atomics of one
// instruction hit consecutive LDS addresses.  Returns whether this thread's
// wave saw any change.
template <int NT>
__device__ __forceinline__ int update(const ClusterArgs& a, const float* __restrict__ Xg, int n0,
                                      int ng, int K, int D, int SP, bool first, int fsh,
                                      long long* sums, int* cnt, unsigned char* dirty, bool marked) {
    const int lane = threadIdx.x & 63, wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform)
    int any = 0;
    for (int base = wid * kWave; base < ng; base += NT) {
        const int p = base + lane;
        int na = 0, oa = -1;
        bool chg = false;
        if (p < ng) {
            na = a.a_new[(size_t)n0 + p];
            // (after the matrix-core scorer only the entries the scan has just decided count;
            // the others may date from earlier steps)
            const bool fresh = !marked || (na >= 0 && (na & kRefinedBit));
            if (marked && fresh) {
                na &= ~kRefinedBit;
                a.a_new[(size_t)n0 + p] = na;
            }
            na = (na >= 0 && na < K) ? na : 0;
            oa = first ? -1 : a.assign[(size_t)n0 + p];
            oa = (oa >= 0 && oa < K) ? oa : -1;
            chg = fresh && na != oa;
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
                const long long q = to_fixed(xr[d], fsh);
                lds_add(&sums[(size_t)nb * SP + d], q);
                if (ob >= 0) lds_add(&sums[(size_t)ob * SP + d], -q);
            }
            if (lane == 0) {
                atomicAdd(&cnt[nb], 1);
                dirty[nb] = 1;
                if (ob >= 0) { atomicSub(&cnt[ob], 1); dirty[ob] = 1; }
            }
        }
    }
    return any;
}

// LDS layout shared by the kernel and the host-side size computation.
struct Lds {
    size_t sums, cent, cn, cnt, dirty, delta, flist, aop, thr, queue, total;
};
__host__ __device__ inline Lds lds_layout(int Kmax, int D, int DP, int Nmax, int waves) {
    const int SP = D | 1;   // odd row stride: clusters spread over the LDS banks
    Lds l;
    // reduction scratch: two slots of one double per wave, then the count of listed candidates
    size_t off = (size_t)waves * 16 + 64;
    l.sums = off; off += (size_t)Kmax * SP * 8;
    off = (off + 15) & ~(size_t)15;
    l.cent = off; off += (size_t)Kmax * DP * 4;
    l.cn = off;   off += (size_t)((Kmax + 31) & ~31) * 4;   // padded to whole centroid tiles
    l.cnt = off;  off += (size_t)Kmax * 4;
    l.dirty = off; off += ((size_t)Kmax + 15) & ~(size_t)15;   // "membership changed" flags, one byte each
    l.delta = off; off += (size_t)Kmax * 4;         // how far each centroid moved in the last renewal
    l.flist = off; off += (size_t)kFlagCap * 2;          // 16-bit candidate numbers
    off = (off + 15) & ~(size_t)15;
    // centroid operands of the matrix-core scorer (only when Kmax <= 64)
    l.aop = off;  if (Kmax <= 64) off += (size_t)((Kmax + 31) / 32) * ((DP - 4) / 16) * 2 * 64 * 16;
    // one drift limit per tile of 32 candidates
    l.thr = off; if (Kmax <= 64) off += ((((size_t)Nmax + 31) / 32) * 4 + 15) & ~(size_t)15;
    // per wave: the candidates waiting to be scored
    l.queue = off; if (Kmax <= 64) off += (size_t)waves * kQueue * 2;
    l.total = off;
    return l;
}

// DS = feature K-steps of 16 (D <= 16*DS); MT = centroid tiles of 32 held in
// registers by the matrix-core scorer, MT = 0 selects the vector-ALU scorer.
// VEC: D is a multiple of 4, so the matrix-core scorers fetch rows in 16-byte pieces;
// otherwise (a compile-time choice, so the loops hold one form only) feature by feature.
// Workgroups per compute unit in the 256-thread shape: three, and four (128 registers,
// a few of them spilled) where at most 32 clusters and 48 features leave room for it -
// batches of many short searches gain 10-17 % from the fourth resident search
// (measured; five cost more in spills than they gain, and with two centroid tiles in
// registers four were 4 % slower).
constexpr int narrow_workgroups_per_cu(int DS, int MT) { return (MT == 1 && DS <= 3) ? 4 : 3; }

template <int DS, int MT, int NT, bool VEC = true>
__global__ void __launch_bounds__(NT, NT == kThreadsNarrow ? narrow_workgroups_per_cu(DS, MT) : 1)
cluster_fused_kernel(ClusterArgs a) {
    constexpr int kThreads = NT, kWaves = NT / kWave;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int D = a.D;
    constexpr int DP = 16 * DS + 4;
    const int SP = D | 1;

    int g = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;
    g = clampi(g, 0, a.G - 1);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (a.mixed && search_is_big(ng, K, a.limit_n)) return;      // the multi-workgroup kernels take this search
    if (K > a.Kmax) K = a.Kmax;   // LDS is sized from the host copy of Kmax
    if (ng > a.Nmax) ng = a.Nmax; // (and of Nmax; a consistent batch never gets here)
    if (MT > 0 && K > 32 * MT) K = 32 * MT;
    if (ng <= 0 || K <= 0) {
        if (tid == 0 && a.iters > 0 && a.objective) a.objective[g] = 0.f;
        return;
    }
    if (a.guard && ng < 2 * K) return;      // too few candidates to re-cluster: nothing is touched

    const Lds L = lds_layout(a.Kmax, D, DP, a.Nmax, kWaves);
    double* red = reinterpret_cast<double*>(smem);
    long long* sums = reinterpret_cast<long long*>(smem + L.sums);   // [Kmax][SP]
    float* cent = reinterpret_cast<float*>(smem + L.cent);           // [Kmax][DP]
    float* cn = reinterpret_cast<float*>(smem + L.cn);               // [Kmax]
    int* cnt = reinterpret_cast<int*>(smem + L.cnt);                 // [Kmax]
    unsigned short* flist = reinterpret_cast<unsigned short*>(smem + L.flist);   // [kFlagCap]
    unsigned char* dirty = reinterpret_cast<unsigned char*>(smem + L.dirty);             // [Kmax]
    float* delta = reinterpret_cast<float*>(smem + L.delta);         // [Kmax]
    float* thr = reinterpret_cast<float*>(smem + L.thr);             // [tiles]
    unsigned short* queue = reinterpret_cast<unsigned short*>(smem + L.queue);   // [kWaves][kQueue]
    float2* lim = a.lim + n0;                                        // [N_g], global
    int* nflag = reinterpret_cast<int*>(smem + kWaves * 16);         // behind the two reduction slots
    bf16x8* aop = reinterpret_cast<bf16x8*>(smem + L.aop);

    const float* Xg = a.X + (size_t)n0 * D;

    // requested together with the initial centroids so that the latencies overlap:
    // (matrix-core path) the largest |x| among the first rows, from which the
    // fixed-point scale is estimated
    float am = 0.f;
    if constexpr (MT > 0) {
        const int srows = ng < 64 ? ng : 64;
        if constexpr (VEC) {
            const int quads = srows * (D >> 2);
            for (int i = tid; i < quads; i += kThreads) {
                const float4 v = reinterpret_cast<const float4*>(Xg)[i];
                am = fmaxf(fmaxf(am, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
            }
        } else {
            for (int i = tid; i < srows * D; i += kThreads) am = fmaxf(am, fabsf(Xg[i]));
        }
    }
    for (int idx = tid; idx < K * DP; idx += kThreads) {
        const int j = idx / DP, d = idx - j * DP;
        float v = 0.f;
        if (d < D)
            v = a.cent_init ? a.cent_init[(size_t)(k0 + j) * D + d]
                            : Xg[(size_t)(j < ng ? j : ng - 1) * D + d];
        cent[idx] = v;
    }
    for (int idx = tid; idx < K * SP; idx += kThreads) sums[idx] = 0;
    for (int j = tid; j < K; j += kThreads) { cnt[j] = 0; dirty[j] = 0; delta[j] = 0.f; }
    for (int j = K + tid; j < ((a.Kmax + 31) & ~31); j += kThreads) cn[j] = kBig;
    if (tid == 0) *nflag = 0;
    __syncthreads();

    if (a.iters == 0) {
        for (int idx = tid; idx < K * D; idx += kThreads) {
            const int j = idx / D, d = idx - j * D;
            a.cent_out[(size_t)(k0 + j) * D + d] = cent[(size_t)j * DP + d];
        }
        return;
    }

    // Fixed-point scale of the sums, from max |x| of the search (fixed_shift rounds
    // the exponent up to a multiple of 4).  The vector-ALU path reads all rows for
    // it.  The matrix-core path estimates it from the first rows, since its first
    // step reads, scores and sums the rows in a single pass; that pass also finds
    // the true maximum, and in the rare case that the estimate's exponent class
    // was too small the sums are rebuilt with the right scale.
    double tsq = 0.0;           // sum of x^2 over the search (exact products, fp64 sums), for the objective
    if constexpr (MT == 0) {
        const size_t total = (size_t)ng * D;
        if ((D & 3) == 0) {
            const size_t quads = total >> 2;
            for (size_t i = tid; i < quads; i += kThreads) {
                const float4 v = reinterpret_cast<const float4*>(Xg)[i];
                am = fmaxf(fmaxf(am, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
                tsq = fma((double)v.x, (double)v.x, tsq);
                tsq = fma((double)v.y, (double)v.y, tsq);
                tsq = fma((double)v.z, (double)v.z, tsq);
                tsq = fma((double)v.w, (double)v.w, tsq);
            }
        } else {
            for (size_t i = tid; i < total; i += kThreads) {
                const float v = Xg[i];
                am = fmaxf(am, fabsf(v));
                tsq = fma((double)v, (double)v, tsq);
            }
        }
    }
    int phase = 0;
    am = block_max_f<kWaves>(am, red, phase);
    if constexpr (MT == 0) tsq = block_sum_d<kWaves>(tsq, red, phase);
    int sh = fixed_shift(am, ng);
    int fsh = sh - 32;          // what to_fixed takes
    double inv = ldexp(1.0, -sh);

    // |c_j|^2, their maximum and the matrix-core operands of the initial centroids
    float cm = renew_rows<DS, (MT > 0), NT>(cent, cn, aop, sums, cnt, dirty, delta, K, D, SP, inv, true, true);
    cm = block_max_f<kWaves>(cm, red, phase);

    bool first = true;
    float drift = 0.f;          // cumulative (largest + second largest) centroid move, rounded up
    float Tc = 0.f;             // lane j: cumulative (move of centroid j + largest move of another), rounded up
    for (int it = 0; it < a.iters; ++it) {
        if constexpr (MT > 0) {
            if (a.use_bounds && it > 0) {
                const int lane = tid & 63;
                const float dj = lane < K ? delta[lane] : 0.f;     // K <= 64 on this path
                const float d1 = wave_max_f(dj);
                const int jm = __ffsll((long long)__ballot(dj == d1)) - 1;
                const float d2 = wave_max_f(lane == jm ? 0.f : dj);
                drift = (drift + (d1 + d2) * 1.0000005f) * 1.0000005f;
                Tc = (Tc + (dj + (lane == jm ? d2 : d1)) * 1.0000005f) * 1.0000005f;
            }
        }
        unsigned char* dw = dirty;        // rows touched in this step, for the renewal at its end

        int st;
        if constexpr (MT > 0) {
            if (first) {
                float am_seen;
                st = score_first<DS, MT, NT, VEC>(a, Xg, n0, ng, K, D, SP, cn, cm, fsh, sums, cnt, nflag,
                                         flist, aop, dw, thr, lim, am_seen, tsq);
                am_seen = block_max_f<kWaves>(am_seen, red, phase);
                tsq = block_sum_d<kWaves>(tsq, red, phase);
                const int sh_true = fixed_shift(am_seen, ng);
                if (sh_true != sh) {
                    // the rows beyond the estimate's sample were larger: rebuild the
                    // sums of the candidates placed so far with the right scale
                    sh = sh_true;
                    fsh = sh - 32;
                    inv = ldexp(1.0, -sh);
                    for (int idx = tid; idx < K * SP; idx += kThreads) sums[idx] = 0;
                    for (int j = tid; j < K; j += kThreads) cnt[j] = 0;
                    __syncthreads();
                    const int lane = tid & 63;
                    for (int p = tid >> 6; p < ng; p += kWaves) {
                        int v = a.a_new[(size_t)n0 + p];      // uniform over the wave
                        if (v < 0) continue;                    // waits for the exact pass
                        v = v < K ? v : 0;
                        for (int d = lane; d < D; d += kWave)
                            lds_add(&sums[(size_t)v * SP + d], to_fixed(Xg[(size_t)p * D + d], fsh));
                        if (lane == 0) atomicAdd(&cnt[v], 1);
                    }
                    __syncthreads();
                }
            } else
            st = score_packed<DS, MT, NT, VEC>(a, Xg, n0, ng, K, D, DP, SP, cent, cn, cm, fsh, sums, cnt,
                                      nflag, flist, aop, dw, thr, lim, queue, drift, Tc);
        } else {
            score_valu<4 * DS, NT>(a, Xg, n0, ng, K, D, DP, cent, cn, cm);
            st = 2;
        }
        st = block_or_i<kWaves>(st, red, phase);
        if (st & 2) {
            int moved;
            const int nf = MT > 0 ? *nflag : kFlagCap + 1;
            if (nf <= kFlagCap) {
                moved = refine_listed<DS, NT>(a, Xg, n0, nf, flist, K, D, DP, SP, cent, fsh, sums, cnt, dw,
                                      thr, lim, drift, Tc);
            } else {
                // the list overflowed (or the vector-ALU scorer ran): scan every candidate;
                // no slack is known for the refined ones, so every tile is scored next time
                refine<NT>(a, Xg, n0, ng, K, D, DP, cent, MT > 0);
                __syncthreads();
                // after the matrix-core scorer only refined candidates are left to move,
                // and it has already recorded an assignment for every other candidate
                moved = update<NT>(a, Xg, n0, ng, K, D, SP, first && MT == 0, fsh, sums, cnt, dw, MT > 0);
                if (MT > 0 && a.iters > 1) {
                    // every candidate's state: its cluster as it stands now, limit 0
                    __syncthreads();
                    for (int q = tid; q < ng; q += kThreads) {
                        const int c = a.assign[(size_t)n0 + q];
                        lim[q].x = pack_limit(0.f, (c >= 0 && c < K) ? c : -1);
                    }
                    if (a.use_bounds)
                        for (int t = tid; t < ((ng + 31) >> 5); t += kThreads) thr[t] = 0.f;
                }
            }
            st |= block_or_i<kWaves>(moved, red, phase);
            // every thread has read the counter before that barrier, and the barriers of
            // the renewal below separate this reset from the next step's additions
            if (tid == 0) *nflag = 0;
        }
        const int changed = st & 1;
        first = false;

        const bool last = (it == a.iters - 1) || (a.early_exit && !changed);
        if (last) {
            // Objective relative to the centroids c_j that entered this step.  With
            // S_j the (exact, fixed-point) sum and n_j the size of cluster j,
            //   sum_k |x_k - c_a(k)|^2 = sum_k |x_k|^2 - sum_j c_j . (2 S_j - n_j c_j),
            // everything in fp64.  The subtraction cancels; when less than 1e-7 of the
            // first term is left the members are summed one by one instead.
            double part = 0.0;
            for (int j0 = 0; j0 < K; j0 += kThreads / 16) {
                const int j = j0 + (tid >> 4), l16 = tid & 15;
                if (j < K) {
                    const double nj = (double)cnt[j];
                    for (int d = l16; d < D; d += 16) {
                        const double cj = (double)cent[(size_t)j * DP + d];
                        const double Sj = (double)sums[(size_t)j * SP + d] * inv;
                        part += cj * (2.0 * Sj - nj * cj);
                    }
                }
            }
            part = block_sum_d<kWaves>(part, red, phase);
            const double Jfast = tsq - part;
            if (Jfast >= 1.0e-7 * tsq) {
                if (tid == 0) a.objective[g] = (float)Jfast;
            } else {
            // 16 lanes per candidate (4 features each), per-lane fp64 partial sums in a
            // fixed candidate order, then a fixed-order reduction
            double acc = 0.0;
            {
                const int sub = tid >> 4, l16 = tid & 15;
                const bool vec4 = (D & 3) == 0;
                constexpr int U = 4, GR = kThreads / 16;
                for (int p0 = sub; p0 < ng; p0 += GR * U) {
                    int jj[U];
                    float4 xq[U];
#pragma unroll
                    for (int q = 0; q < U; ++q) {
                        const int p = p0 + q * GR;
                        jj[q] = p < ng ? a.assign[(size_t)n0 + p] : 0;
                    }
#pragma unroll
                    for (int q = 0; q < U; ++q) {
                        const int p = p0 + q * GR;
                        xq[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (p < ng) {
                            const float* xr = Xg + (size_t)p * D;
                            if (vec4) {
                                if (4 * l16 < D) xq[q] = *reinterpret_cast<const float4*>(xr + 4 * l16);
                            } else {
                                const int d = 4 * l16;
                                if (d < D) xq[q].x = xr[d];
                                if (d + 1 < D) xq[q].y = xr[d + 1];
                                if (d + 2 < D) xq[q].z = xr[d + 2];
                                if (d + 3 < D) xq[q].w = xr[d + 3];
                            }
                        }
                    }
#pragma unroll
                    for (int q = 0; q < U; ++q) {
                        const int p = p0 + q * GR;
                        if (p < ng && 4 * l16 < D) {
                            const int j = (jj[q] >= 0 && jj[q] < K) ? jj[q] : 0;
                            // centroid rows are zero-padded beyond D, like xq
                            const float4 cv = *reinterpret_cast<const float4*>(cent + (size_t)j * DP + 4 * l16);
                            const float e0 = xq[q].x - cv.x, e1 = xq[q].y - cv.y;
                            const float e2 = xq[q].z - cv.z, e3 = xq[q].w - cv.w;
                            acc += (double)fmaf(e0, e0, fmaf(e1, e1, fmaf(e2, e2, e3 * e3)));
                        }
                    }
                }
            }
            acc = block_sum_d<kWaves>(acc, red, phase);
            if (tid == 0) a.objective[g] = (float)acc;
            }
        }
        // new centroids, and what the next step needs from them
        cm = renew_rows<DS, (MT > 0), NT>(cent, cn, aop, sums, cnt, dirty, delta, K, D, SP, inv, false, !last);
        cm = block_max_f<kWaves>(cm, red, phase);
        if (last) break;
    }

    for (int idx = tid; idx < K * D; idx += kThreads) {
        const int j = idx / D, d = idx - j * D;
        a.cent_out[(size_t)(k0 + j) * D + d] = cent[(size_t)j * DP + d];
    }
    for (int j = tid; j < K; j += kThreads) a.counts[k0 + j] = cnt[j];
}

// ---- very short searches: one wave per search --------------------------------------
// A search of at most 64 candidates and 16 clusters - the size of a search in the
// paper's own runs (Sec. 3.6: a frontier of a few dozen kernels, K = 3) - is one
// wave's work: lane l keeps candidate l's row in registers for the whole call, the
// search's centroids and fixed-point sums sit in the wave's own piece of LDS, and
// since nothing is shared with another wave no step needs a workgroup barrier or a
// block-wide reduction (what a step of a short search mostly consists of in the
// kernel above).  Four searches per workgroup.
//
// A step: every lane decides its candidate exactly - fp32 direct-difference distances
// (relative error <= (D + 2) 2^-24, sums of non-negative terms); if the two smallest
// are further apart than twice that bound allows, the smallest is the unique nearest
// centroid; otherwise fp64, summed over the features in index order with separate
// multiply and add (the plain definition), lowest index on ties - and moves its row
// between the fixed-point sums if the cluster changed.  Between scorings a lane
// keeps an upper bound on the distance to its centroid and a lower bound on the
// distance to any other; the first grows by its centroid's move, the second shrinks
// by the largest move of another centroid, and while the first stays below the second
// the candidate is not scored.  Centroids from the sums exactly as in the kernel
// above (same grid, same rounding), so both give the same bytes.
constexpr int kWaveMaxN = 64, kWaveMaxK = 16;

struct WaveLds {
    size_t sums, cent, cnt, delta, dirty, armR, armkmin, armN, armalive, total;
};
// S > 0: with the cluster-arm tables of the selection step (the whole-round kernel)
__host__ __device__ inline WaveLds wave_lds_layout(int Kmax, int D, int DP, int S = 0) {
    const int SP = D | 1;
    WaveLds l;
    size_t off = 0;
    l.sums = off;  off += (size_t)Kmax * SP * 8;
    off = (off + 15) & ~(size_t)15;
    l.cent = off;  off += (size_t)Kmax * DP * 4;
    l.cnt = off;   off += (size_t)Kmax * 4;
    l.delta = off; off += (size_t)Kmax * 4;
    l.dirty = off; off += ((size_t)Kmax + 15) & ~(size_t)15;
    off = (off + 15) & ~(size_t)15;
    l.armR = off;     off += (size_t)Kmax * S * 8;
    l.armkmin = off;  off += S > 0 ? (size_t)Kmax * 8 : 0;
    l.armN = off;     off += (size_t)Kmax * S * 4;
    l.armalive = off; off += S > 0 ? (size_t)Kmax * 4 : 0;
    l.total = (off + 15) & ~(size_t)15;
    return l;
}

// What the whole-round kernel needs beyond the clustering arguments: the pruning
// step's inputs and outputs (Eq. 2 and the mask of Eq. 5) and the selection call.
struct WaveRound {
    const float* flops;
    const float* bytes;
    const float* incumbent;
    float peak_flops, peak_bw;
    float* bound;
    uint8_t* alive;
    UcbArgs u;
};

// ROUND: the whole round of the search in this one wave - the roofline bound and the
// mask of every candidate first (the same correctly rounded divisions and strict
// compare as the pruning kernel), the clustering, then the cluster-arm statistics
// from the lanes' own clusters (integer LDS atomics, as in the selection kernel, so
// the same tables), scores and selection.  (The host takes this path with a.iters >= 1
// and a.guard = 0.)
template <int DS, bool ROUND>
__device__ __forceinline__ void wave_search(const ClusterArgs& a, const WaveRound* rd, unsigned char* smem) {
    constexpr int DP = 16 * DS + 4;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = (int)blockIdx.x * 4 + wv;
    if (g >= a.G) return;                 // (a whole wave leaves: nothing in this kernel waits for another wave)
    const int D = a.D, SP = D | 1;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (ng > kWaveMaxN) ng = kWaveMaxN;   // (the host launches this kernel only for such batches)
    bool live = true;                     // this lane's candidate passed the pruning step
    float rbound = 0.f;
    if constexpr (ROUND) {
        if (lane < ng) {
            const float t_compute = rd->flops[(size_t)n0 + lane] / rd->peak_flops;
            const float t_memory = rd->bytes[(size_t)n0 + lane] / rd->peak_bw;
            rbound = t_compute > t_memory ? t_compute : t_memory;
            live = rbound < rd->incumbent[g];
            rd->bound[(size_t)n0 + lane] = rbound;
            rd->alive[(size_t)n0 + lane] = live ? 1 : 0;
        }
    }
    if (ng <= 0 || K <= 0) {
        if (lane == 0 && a.iters > 0 && a.objective) a.objective[g] = 0.f;
        if constexpr (ROUND) {
            if (lane < 3) rd->u.sel[(size_t)g * 3 + lane] = -1;
        }
        return;
    }
    if (a.guard && ng < 2 * K) return;

    const WaveLds L = wave_lds_layout(a.Kmax, D, DP, ROUND ? rd->u.S : 0);
    unsigned char* base = smem + (size_t)wv * L.total;
    long long* sums = reinterpret_cast<long long*>(base + L.sums);      // [Kmax][SP]
    float* cent = reinterpret_cast<float*>(base + L.cent);              // [Kmax][DP]
    int* cnt = reinterpret_cast<int*>(base + L.cnt);                    // [Kmax]
    float* delta = reinterpret_cast<float*>(base + L.delta);            // [Kmax]
    unsigned char* dirty = base + L.dirty;                              // [Kmax]
    const float* Xg = a.X + (size_t)n0 * D;
    const bool valid = lane < ng;

    // this lane's row, zero-padded to 16 * DS features (a lane without a candidate holds zeros)
    float x[16 * DS];
#pragma unroll
    for (int d = 0; d < 16 * DS; ++d) x[d] = 0.f;
    if (valid) {
        const float* xr = Xg + (size_t)lane * D;
        if ((D & 3) == 0) {
#pragma unroll
            for (int c = 0; c < 4 * DS; ++c) {
                if (4 * c < D) {
                    const float4 v = reinterpret_cast<const float4*>(xr)[c];
                    x[4 * c] = v.x; x[4 * c + 1] = v.y; x[4 * c + 2] = v.z; x[4 * c + 3] = v.w;
                }
            }
        } else {
#pragma unroll
            for (int d = 0; d < 16 * DS; ++d) if (d < D) x[d] = xr[d];
        }
    }
    float am = 0.f;
    double tsq = 0.0;
#pragma unroll
    for (int d = 0; d < 16 * DS; ++d) {
        am = fmaxf(am, fabsf(x[d]));
        tsq = fma((double)x[d], (double)x[d], tsq);
    }
    am = wave_max_f(am);
    tsq = wave_sum_d(tsq);

    for (int idx = lane; idx < K * DP; idx += kWave) {
        const int j = idx / DP, d = idx - j * DP;
        float v = 0.f;
        if (d < D)
            v = a.cent_init ? a.cent_init[(size_t)(k0 + j) * D + d]
                            : Xg[(size_t)(j < ng ? j : ng - 1) * D + d];
        cent[idx] = v;
    }
    for (int idx = lane; idx < K * SP; idx += kWave) sums[idx] = 0;
    if (lane < K) { cnt[lane] = 0; dirty[lane] = 0; delta[lane] = 0.f; }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");

    if (a.iters == 0) {
        for (int idx = lane; idx < K * D; idx += kWave) {
            const int j = idx / D, d = idx - j * D;
            a.cent_out[(size_t)(k0 + j) * D + d] = cent[(size_t)j * DP + d];
        }
        return;
    }
    const int sh = fixed_shift(am, ng);
    const int fsh = sh - 32;
    const double inv = ldexp(1.0, -sh);
    const float eps = 2.f * (float)(D + 2) * 5.9604644775390625e-08f;

    int mine = -1;
    float ub = 0.f, lb = 0.f;
    for (int it = 0; it < a.iters; ++it) {
        bool need = valid;
        if (it > 0) {
            const float dj = lane < K ? delta[lane] : 0.f;       // K <= 16 here
            const float d1 = wave_max_f(dj);
            const int jm = __ffsll((long long)__ballot(dj == d1)) - 1;
            const float d2 = wave_max_f(lane == jm ? 0.f : dj);
            if (valid) {
                ub = (ub + delta[mine]) * 1.0000005f;                           // rounded up
                const float t = lb - (mine == jm ? d2 : d1) * 1.0000005f;
                lb = t - fabsf(t) * 1.0e-6f;                                    // rounded down
                need = !(a.use_bounds && ub < lb);
            }
        }
        int moved = 0;
        if (need) {
            float b32 = INFINITY, s32 = INFINITY;
            int bj = 0;
            for (int j = 0; j < K; ++j) {
                const float4* cr = reinterpret_cast<const float4*>(cent + (size_t)j * DP);   // (one address for all lanes)
                float acc0 = 0.f, acc1 = 0.f;
                // rows and centroids are zero-padded to 16 * DS features: the extra terms are +0.0
#pragma unroll
                for (int c = 0; c < 4 * DS; ++c) {
                    const float4 cv = cr[c];
                    const float e0 = x[4 * c] - cv.x, e1 = x[4 * c + 1] - cv.y;
                    const float e2 = x[4 * c + 2] - cv.z, e3 = x[4 * c + 3] - cv.w;
                    acc0 = fmaf(e0, e0, acc0);
                    acc1 = fmaf(e1, e1, acc1);
                    acc0 = fmaf(e2, e2, acc0);
                    acc1 = fmaf(e3, e3, acc1);
                }
                const float acc = acc0 + acc1;
                if (acc < b32) { s32 = b32; b32 = acc; bj = j; }
                else if (acc < s32) s32 = acc;
            }
            if (s32 * (1.f - eps) > b32 * (1.f + eps) + 1.0e-35f) {
                ub = sqrtf(b32 * (1.f + eps)) * 1.0000005f;
                lb = sqrtf(s32 * (1.f - eps)) * 0.9999995f;
            } else {
                double bd = INFINITY, sd = INFINITY;
                bj = 0;
                for (int j = 0; j < K; ++j) {
                    const float* cr = cent + (size_t)j * DP;
                    double acc = 0.0;
#pragma unroll
                    for (int d = 0; d < 16 * DS; ++d) {
                        const double diff = __dsub_rn((double)x[d], (double)cr[d]);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    }
                    if (acc < bd) { sd = bd; bd = acc; bj = j; }
                    else if (acc < sd) sd = acc;
                }
                ub = (float)sqrt(bd) * 1.0000005f;
                lb = (float)sqrt(sd) * 0.9999995f;
            }
            if (bj != mine) {
#pragma unroll
                for (int d = 0; d < 16 * DS; ++d) {
                    if (d < D) {
                        const long long q = to_fixed(x[d], fsh);
                        lds_add(&sums[(size_t)bj * SP + d], q);
                        if (mine >= 0) lds_add(&sums[(size_t)mine * SP + d], -q);
                    }
                }
                atomicAdd(&cnt[bj], 1);
                dirty[bj] = 1;
                if (mine >= 0) { atomicSub(&cnt[mine], 1); dirty[mine] = 1; }
                a.assign[(size_t)n0 + lane] = bj;
                mine = bj;
                moved = 1;
            }
        }
        const bool changed = __any(moved) != 0;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");

        const bool last = (it == a.iters - 1) || (a.early_exit && !changed);
        if (last) {
            // objective relative to the centroids that entered this step, from the exact sums
            // (see the kernel above); member by member when the subtraction cancels
            double part = 0.0;
            for (int idx = lane; idx < K * D; idx += kWave) {
                const int j = idx / D, d = idx - j * D;
                const double cj = (double)cent[(size_t)j * DP + d];
                const double Sj = (double)sums[(size_t)j * SP + d] * inv;
                part += cj * (2.0 * Sj - (double)cnt[j] * cj);
            }
            part = wave_sum_d(part);
            double J = tsq - part;
            if (!(J >= 1.0e-7 * tsq)) {
                double acc = 0.0;
                if (valid) {
                    const float4* cr = reinterpret_cast<const float4*>(cent + (size_t)mine * DP);
#pragma unroll
                    for (int c = 0; c < 4 * DS; ++c) {
                        const float4 cv = cr[c];
                        const float e0 = x[4 * c] - cv.x, e1 = x[4 * c + 1] - cv.y;
                        const float e2 = x[4 * c + 2] - cv.z, e3 = x[4 * c + 3] - cv.w;
                        acc += (double)fmaf(e0, e0, fmaf(e1, e1, fmaf(e2, e2, e3 * e3)));
                    }
                }
                J = wave_sum_d(acc);
            }
            if (lane == 0) a.objective[g] = (float)J;
        }
        // new centroids (a wave of its own: the cross-lane steps of the renewal stay inside it)
        renew_rows<DS, false, kWave>(cent, nullptr, nullptr, sums, cnt, dirty, delta, K, D, SP, inv, false, false, lane);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        if (last) break;
    }

    for (int idx = lane; idx < K * D; idx += kWave) {
        const int j = idx / D, d = idx - j * D;
        a.cent_out[(size_t)(k0 + j) * D + d] = cent[(size_t)j * DP + d];
    }
    if (lane < K) a.counts[k0 + lane] = cnt[lane];

    if constexpr (ROUND) {
        const UcbArgs& u = rd->u;
        const int KS = K * u.S;
        unsigned long long* R = reinterpret_cast<unsigned long long*>(base + L.armR);        // [Kmax*S]
        unsigned long long* kmin = reinterpret_cast<unsigned long long*>(base + L.armkmin);  // [Kmax]
        unsigned* Ncnt = reinterpret_cast<unsigned*>(base + L.armN);                         // [Kmax*S]
        unsigned* nalive = reinterpret_cast<unsigned*>(base + L.armalive);                   // [Kmax]
        for (int i = lane; i < KS; i += kWave) { R[i] = 0ull; Ncnt[i] = 0u; }
        if (lane < K) { kmin[lane] = ~0ull; nalive[lane] = 0u; }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        if (valid && live)        // (iters >= 1: every candidate has a cluster)
            ucb_add_candidate(u, (size_t)n0 + lane, lane, mine >= 0 ? mine : 0, rbound, Ncnt, R, nalive, kmin);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        ucb_finish<kWave>(u, g, n0, k0, K, Ncnt, R, nalive, kmin, nullptr, nullptr, lane);
    }
}

template <int DS>
__global__ void __launch_bounds__(256) cluster_wave_kernel(ClusterArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    wave_search<DS, false>(a, nullptr, smem);
}

template <int DS>
__global__ void __launch_bounds__(256) round_wave_kernel(ClusterArgs a, WaveRound rd) {
    extern __shared__ __align__(16) unsigned char smem[];
    wave_search<DS, true>(a, &rd, smem);
}

constexpr size_t kMaxLds = 160 * 1024;

}  // namespace

// sizes the one-workgroup kernel is laid out for: the largest search it will take
static int one_wg_kmax(const kb_batch& b) { return b.Kmax > kOneWgMaxK ? kOneWgMaxK : (b.Kmax > 0 ? b.Kmax : 1); }
static int one_wg_nmax(const kb_batch& b) { return b.Nmax > one_wg_limit_n(b) ? one_wg_limit_n(b) : b.Nmax; }

bool cluster_supported(const kb_batch& b) {
    const int ds = (b.D + 15) / 16;
    return lds_layout(one_wg_kmax(b), b.D, 16 * ds + 4, one_wg_nmax(b), kThreadsNarrow / kWave).total <= kMaxLds;
}

static ClusterArgs cluster_args(const kb_batch& b, const ClusterCall& c) {
    ClusterArgs a;
    a.G = b.G; a.D = b.D; a.Ksum = b.Ksum; a.Kmax = one_wg_kmax(b); a.N = b.N;
    a.seg_off = b.seg_off; a.koff = b.koff; a.X = c.X; a.cent_init = c.cent_init;
    a.iters = c.iters; a.early_exit = c.stop_early ? 1 : 0; a.assign = c.assign; a.cent_out = c.cent_out;
    a.counts = c.counts; a.objective = c.objective; a.a_new = c.a_new;
    a.order = b.G > 1 ? c.order : nullptr;       // (one search: the order is the identity and was not computed)
    a.use_bounds = c.scorer != 2;
    a.guard = c.guard;
    a.mixed = c.mixed;
    a.limit_n = one_wg_limit_n(b);
    a.lim = reinterpret_cast<float2*>(c.lim);
    a.Nmax = one_wg_nmax(b);
    return a;
}

bool cluster_wave_per_search(const kb_batch& b, int scorer) {
    return scorer == KB_SCORER_DEFAULT && b.Nmax <= kWaveMaxN && b.Kmax <= kWaveMaxK;
}
static bool wave_per_search(const kb_batch& b, const ClusterCall& c) {
    return !c.mixed && cluster_wave_per_search(b, c.scorer);
}

// One wave per search, four searches per workgroup; rd: the whole round, else the
// clustering step only.
static hipError_t launch_wave(const kb_batch& b, const ClusterArgs& a_in, const WaveRound* rd, hipStream_t st) {
    // A search stops at its first step without a move: such a step leaves sums, sizes
    // and centroids as they were, so every later step would repeat it and every output
    // is the same bytes as after the full count of steps.
    ClusterArgs a = a_in;
    a.early_exit = 1;
    const int ds = (b.D + 15) / 16;
    const size_t wlds = 4 * wave_lds_layout(a.Kmax, b.D, 16 * ds + 4, rd ? b.S : 0).total;
    if (wlds > kMaxLds) return hipErrorInvalidValue;
    const dim3 wgrid((unsigned)((b.G + 3) / 4)), wblock(256);
#define KB_LAUNCH_WAVE(DS_)                                                                     \
    do {                                                                                        \
        if (rd) {                                                                               \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(round_wave_kernel<DS_>), \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)wlds); \
            if (e != hipSuccess) return e;                                                      \
            hipLaunchKernelGGL((round_wave_kernel<DS_>), wgrid, wblock, wlds, st, a, *rd);      \
        } else {                                                                                \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(cluster_wave_kernel<DS_>), \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)wlds); \
            if (e != hipSuccess) return e;                                                      \
            hipLaunchKernelGGL((cluster_wave_kernel<DS_>), wgrid, wblock, wlds, st, a);         \
        }                                                                                       \
    } while (0)
    switch (ds) {
        case 1: KB_LAUNCH_WAVE(1); break;
        case 2: KB_LAUNCH_WAVE(2); break;
        case 3: KB_LAUNCH_WAVE(3); break;
        default: KB_LAUNCH_WAVE(4); break;
    }
#undef KB_LAUNCH_WAVE
    return hipGetLastError();
}

// A batch of searches of at most 64 candidates and 16 clusters each, in the default
// mode: the whole round (Sec. 3.5: prune, cluster, select) is one launch, a wave per
// search.  (The selection tables share the wave's piece of LDS; strategy counts that
// would leave fewer than two workgroups per compute unit take the three-stage path.)
bool round_in_one_launch(const kb_batch& b, int scorer) {
    if (scorer != KB_SCORER_DEFAULT || b.Nmax > kWaveMaxN || b.Kmax > kWaveMaxK) return false;
    const int ds = (b.D + 15) / 16;
    const int kmax = b.Kmax > 0 ? b.Kmax : 1;
    return 4 * wave_lds_layout(kmax, b.D, 16 * ds + 4, b.S).total <= 64 * 1024;
}

hipError_t launch_round_wave(const kb_batch& b, const ClusterCall& c, const UcbCall& uc,
                             const float* flops, const float* bytes, const float* incumbent,
                             float peak_flops, float peak_bw, float* bound, uint8_t* alive,
                             hipStream_t st) {
    if (!round_in_one_launch(b, c.scorer) || c.mixed || c.guard || c.iters < 1 || c.cent_init)
        return hipErrorInvalidValue;
    const ClusterArgs a = cluster_args(b, c);
    WaveRound rd;
    rd.flops = flops; rd.bytes = bytes; rd.incumbent = incumbent;
    rd.peak_flops = peak_flops; rd.peak_bw = peak_bw; rd.bound = bound; rd.alive = alive;
    rd.u = make_ucb_args(b, uc);
    return launch_wave(b, a, &rd, st);
}

hipError_t launch_cluster(const kb_batch& b, const ClusterCall& c, hipStream_t st) {
    const ClusterArgs a = cluster_args(b, c);
    const int ds = (b.D + 15) / 16;   // 1..4 K-steps of 16 features
    int mt = a.Kmax <= 32 ? 1 : (a.Kmax <= 64 ? 2 : 0);
    if (c.scorer == 1) mt = 0;
    // the matrix-core kernels fetch rows in 16-byte pieces when D is a multiple of 4 and
    // feature by feature otherwise (own instantiations, in the 256-thread shape only)
    const bool vec = (b.D & 3) == 0;
    // few searches: every workgroup has a compute unit to itself and takes the wide shape
    const size_t lds_wide = lds_layout(a.Kmax, b.D, 16 * ds + 4, a.Nmax, kThreadsWide / kWave).total;
    // ... and so does a batch of long searches only (2048 candidates or more on average):
    // measured 13-20 % faster than three of them sharing a compute unit
    const bool wide = (vec || mt == 0) && (b.G <= kWideMaxG || b.N >= (int64_t)2048 * b.G) && lds_wide <= kMaxLds;
    const size_t lds = wide ? lds_wide
                            : lds_layout(a.Kmax, b.D, 16 * ds + 4, a.Nmax, kThreadsNarrow / kWave).total;
    if (lds > kMaxLds) return hipErrorInvalidValue;
    // a batch of very short searches, in the library's default mode: one wave per search
    if (wave_per_search(b, c)) return launch_wave(b, a, nullptr, st);
    const dim3 grid((unsigned)b.G), block(wide ? kThreadsWide : kThreadsNarrow);
#define KB_NARROW_SCALAR kThreadsNarrow, false
#define KB_LAUNCH_NT(DS_, MT_, NT_)                                                             \
    do {                                                                                        \
        hipError_t e = hipFuncSetAttribute(                                                     \
            reinterpret_cast<const void*>(cluster_fused_kernel<DS_, MT_, NT_>),                 \
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                              \
        if (e != hipSuccess) return e;                                                          \
        hipLaunchKernelGGL((cluster_fused_kernel<DS_, MT_, NT_>), grid, block, lds, st, a);     \
    } while (0)
#define KB_LAUNCH_MATRIX(DS_, MT_)                                                              \
    do {                                                                                        \
        if (wide) KB_LAUNCH_NT(DS_, MT_, kThreadsWide);                                         \
        else if (vec) KB_LAUNCH_NT(DS_, MT_, kThreadsNarrow);                                   \
        else KB_LAUNCH_NT(DS_, MT_, KB_NARROW_SCALAR);                                          \
    } while (0)
#define KB_LAUNCH_VECTOR_ALU(DS_)                                                               \
    do {                                                                                        \
        if (wide) KB_LAUNCH_NT(DS_, 0, kThreadsWide);                                           \
        else KB_LAUNCH_NT(DS_, 0, kThreadsNarrow);                                              \
    } while (0)
#define KB_LAUNCH_DS(DS_)                                                                       \
    do {                                                                                        \
        if (mt == 1) KB_LAUNCH_MATRIX(DS_, 1);                                                  \
        else if (mt == 2) KB_LAUNCH_MATRIX(DS_, 2);                                             \
        else KB_LAUNCH_VECTOR_ALU(DS_);                                                         \
    } while (0)
    switch (ds) {
        case 1: KB_LAUNCH_DS(1); break;
        case 2: KB_LAUNCH_DS(2); break;
        case 3: KB_LAUNCH_DS(3); break;
        default: KB_LAUNCH_DS(4); break;
    }
#undef KB_LAUNCH_DS
#undef KB_LAUNCH_VECTOR_ALU
#undef KB_LAUNCH_MATRIX
#undef KB_LAUNCH_NT
#undef KB_NARROW_SCALAR
    return hipGetLastError();
}

}  // namespace kb
