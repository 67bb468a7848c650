// Internal declarations shared by the translation units of libkernelband.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "kb.h"

namespace kb {

constexpr int kWave = 64;
constexpr int kGeoRange = 2048;      // candidates per workgroup of the representative / radius pass
constexpr int kSampleRange = 4096;   // candidates per workgroup of the in-cluster draw
constexpr int kShortSearch = 256;    // a batch whose longest search has at most this many candidates runs
                                     // the selection and the representative pass one wave per search
constexpr int kTilesPerChunk = 64;   // tiles of 32 candidates per workgroup of the multi-workgroup clustering path

// ---- workspace layout (all offsets 256-byte aligned) ------------------------
// extra buffers of the multi-workgroup clustering path
struct BigWs {
    int kpad;            // Kmax rounded up to whole centroid tiles of 32
    size_t max_chunks;   // upper bound of the number of tile chunks (grid size)
    size_t chunk_off, sums, cnpad, centT, aop, dirty, amax, cnmax, nflag, few, partJ, prop, tsq, needfull, end;
};
BigWs big_ws_layout(const kb_batch& b, size_t base);
// Searches with more than 64 clusters or more than 65536 candidates take the
// multi-workgroup path, the others the one-workgroup kernel.  The host sees only
// the largest K_g and N_g of a batch: when those say that the batch holds such a
// search, both paths are enqueued and each leaves the other's searches alone
// (decided on the device from every search's own K_g and N_g).
constexpr int kOneWgMaxK = 64;
constexpr int kOneWgMaxN = 65536;
// In a batch of few searches a long one does not leave its share of the chip to others
// by staying on one compute unit: there the multi-workgroup path takes over earlier
// (measured: a lone search of 32768 candidates 1.47 against 1.16 ms, eight of 30000 6.1
// against 1.7 ms; 32 searches of 16000 are as fast either way).
// The same holds for a few long searches among many short ones, which are done long
// before the long ones (2000 searches of 12-41 candidates and one of 30000: 1.67 ms,
// all of it the long one on its compute unit).  The host does not see the lengths, but
// a batch of at most 32 * 24576 candidates cannot hold more than 32 searches beyond 24576.
constexpr int kFewSearches = 32;
constexpr int kFewSearchesMaxN = 24576;
// most candidates of a search that the one-workgroup Lloyd kernel takes in this batch
inline int one_wg_limit_n(const kb_batch& b) {
    const bool few_long = b.G <= kFewSearches || b.N <= (int64_t)kFewSearches * kFewSearchesMaxN;
    return (few_long && b.Nmax > kFewSearchesMaxN) ? kFewSearchesMaxN : kOneWgMaxN;
}
inline bool cluster_uses_big(const kb_batch& b) { return b.Kmax > kOneWgMaxK || b.Nmax > one_wg_limit_n(b); }
// (limit_n: one_wg_limit_n of the batch)
__host__ __device__ inline bool search_is_big(int ng, int K, int limit_n) { return K > kOneWgMaxK || ng > limit_n; }

struct WsLayout {
    size_t a_new;   // int32 [N]     proposed assignment of the current step (bit 31: needs exact re-evaluation)
    size_t order;   // int32 [G]     searches sorted by decreasing work, for longest-first scheduling
    size_t misc;    // int32 [128]   histogram / cursors of the ordering kernel
    size_t tile_off;// int32 [G+1]   prefix sum of ceil(N_g / 32): first 32-candidate tile of each search
    size_t xn;      // float [N]     |x_k|^2 of every candidate (multi-workgroup path)
    size_t split;   // bf16          feature rows split into bf16 (hi, mid) pieces, 4 * Dpad bytes per
                    //               candidate: [candidate][16-feature step][half][hi|mid][8] on the
                    //               one-workgroup path, [tile][16-feature step][hi|mid][lane][8] (the
                    //               matrix cores' operand order) on the multi-workgroup path
    size_t max_tiles;   // capacity of `split` in tiles (not an offset)
    bool use_big;
    BigWs big;
    bool ucb_chunked;   // searches longer than 16384 candidates: partial tables per candidate range
    size_t ucb_R, ucb_N, ucb_kmin, ucb_nalive;
    size_t geo_d2;     // double [N]     squared distance of every candidate to its centroid
    size_t geo_min;    // uint64 [Ksum]  bit pattern of the smallest such distance per cluster
    size_t geo_max;    // uint64 [Ksum]  and of the largest
    size_t dia_off;    // int32 [Ksum + 1] first slot of every cluster in the grouped index list
    size_t dia_toff;   // int32 [Ksum + 1] first tile of every cluster in the global tile numbering
    size_t dia_bsum;   // int64 [2 * (Ksum / 4096 + 1)] block sums of the two prefix sums
    size_t samp_key;   // double [2*ranges]  partial best keys of searches that cross range borders
    size_t samp_idx;   // int32  [2*ranges]  their candidates
    size_t seed_key;   // double [4*ranges]  seeding of long searches: best key of every range, two
                       //                    slots, two alternating sets
    size_t seed_idx;   // int32  [4*ranges]  and its row
    size_t total;
};
WsLayout ws_layout(const kb_batch& b);

// ---- launchers (enqueue only; return hipGetLastError()) ---------------------
hipError_t launch_prune(const kb_batch& b, float peak_flops, float peak_bw,
                        const float* flops, const float* bytes,
                        const float* incumbent, float* bound, uint8_t* alive,
                        hipStream_t st);

hipError_t launch_order(const kb_batch& b, int32_t* order, int32_t* tile_off, int32_t* chunk_off,
                        hipStream_t st);

struct ClusterCall {
    const float* X;
    const float* cent_init;   // NULL: first K_g rows
    int32_t iters;
    int32_t* assign;
    float* cent_out;
    int32_t* counts;
    float* objective;
    int32_t* a_new;
    const int32_t* order;
    const int32_t* tile_off;
    float* xn;
    void* split;
    int64_t max_tiles;
    float* lim;               // float2 [N] scratch of the fused kernel (every candidate's drift limit | cluster, |x|^2)
    int guard;                // 1: searches with N_g < 2 K_g keep their clustering untouched
    int mixed;                // 1: the batch may hold searches of both paths; each kernel skips the other's
    int scorer;               // kb_params::scorer: 0 default, 1 vector ALU only, 2 matrix cores without bounds
    int stop_early;           // kb_params::stop_early (one-workgroup kernels only)
};
hipError_t launch_cluster(const kb_batch& b, const ClusterCall& c, hipStream_t st);
hipError_t launch_cluster_big(const kb_batch& b, const ClusterCall& c, const BigWs& w, char* ws,
                              hipStream_t st);
bool cluster_supported(const kb_batch& b);   // shape fits the compiled clustering kernels
bool cluster_wave_per_search(const kb_batch& b, int scorer);   // the batch runs one wave per search (no scheduling order needed)

struct UcbCall {
    const int32_t* assign;
    const uint8_t* alive;     // NULL: every candidate alive
    const float* bound;       // NULL: k* = lowest-index member
    const uint8_t* M;         // NULL or [Ksum,S] strategy mask
    const int32_t* visits;
    const float* rsum;
    const int64_t* t;
    float c, prior_n, prior_mu;
    int32_t* Ncs;
    float* mu;
    float* ucb;
    int32_t* sel;
    const int32_t* order;
    // cluster-arm tables in global memory: visit counts, reward sums in 2^-30 fixed
    // point, alive members and best member per cluster.  Searches of more than 16384
    // candidates are aggregated there (chunked != 0 says the batch has such a
    // search; the tables must then be given); the others only when keep_tables asks
    // for a copy of their LDS tables.  from_tables: no aggregation at all, scores
    // and selection come from the tables as they stand.
    unsigned* gN;
    unsigned long long* gR;
    unsigned* gnalive;
    unsigned long long* gkmin;
    int chunked, keep_tables, from_tables;
};
hipError_t launch_ucb(const kb_batch& b, const UcbCall& c, hipStream_t st);
bool ucb_wave_per_search(const kb_batch& b);   // a plain or table-keeping selection call runs one wave per search (no scheduling order needed)

// The whole round of a batch of very short searches in one launch (one wave per
// search): true if batch and mode allow it; the launch itself takes the three
// stages' arguments (no initial centroids, iters >= 1, no workspace arrays).
bool round_in_one_launch(const kb_batch& b, int scorer);
hipError_t launch_round_wave(const kb_batch& b, const ClusterCall& c, const UcbCall& uc,
                             const float* flops, const float* bytes, const float* incumbent,
                             float peak_flops, float peak_bw, float* bound, uint8_t* alive,
                             hipStream_t st);

struct SampleCall {
    const int32_t* assign;
    const uint8_t* alive;      // NULL: every candidate alive
    const float* bound;
    const float* incumbent;
    const int32_t* sel;
    const float* h;            // non-NULL selects the signature form of the headroom
    const int32_t* target;
    int R;
    float theta_sat;
    uint64_t seed, draw;
    float tau;
    int32_t* ksel;
    double* slot_key;
    int32_t* slot_idx;
};
hipError_t launch_sample(const kb_batch& b, const SampleCall& c, hipStream_t st);

struct GeoCall {
    const float* X;
    const float* cent;
    const int32_t* assign;
    int32_t* rep;
    float* radius;
    double* d2;
    unsigned long long* gmin;
    unsigned long long* gmax;
};
hipError_t launch_geometry(const kb_batch& b, const GeoCall& c, hipStream_t st);
size_t geometry_lds_bytes(int Kmax, int D);

struct DiameterCall {
    const float* X;
    const int32_t* assign;
    float* diam;
    int32_t* cnt;     // [Ksum]
    int32_t* off;     // [Ksum + 1]
    int32_t* toff;    // [Ksum + 1]
    long long* bsum;  // [2 * (Ksum / 4096 + 1)]
    int32_t* perm;    // [N]
};
hipError_t launch_diameter(const kb_batch& b, const DiameterCall& c, hipStream_t st);

// number of candidate ranges of the launch-per-centroid seeding (sizes skey / sidx: 4 per range)
size_t seed_ranges(const kb_batch& b);
hipError_t launch_seed(const kb_batch& b, const float* X, float* cent, int32_t* pick, double* mind,
                       double* skey, int32_t* sidx, const int32_t* order, int dsquared,
                       uint64_t seed, uint64_t draw0, hipStream_t st);

hipError_t launch_strategy_mask(const kb_batch& b, int R, const float* h, const int32_t* target,
                                const int32_t* rep, float theta_sat, uint8_t* M, int32_t* nvalid,
                                hipStream_t st);
// gN / gR != NULL: the cluster-arm tables of UcbCall are advanced too (they then equal
// what an aggregation of the updated history under `assign` / `alive` would give).
hipError_t launch_update_stats(const kb_batch& b, float prior_n, const int32_t* sel,
                               const int32_t* ksel, const float* reward, const uint8_t* ok,
                               int32_t* visits, float* rsum, int32_t* Ncs, float* mu, int64_t* t,
                               hipStream_t st, const int32_t* assign = nullptr,
                               const uint8_t* alive = nullptr, unsigned* gN = nullptr,
                               unsigned long long* gR = nullptr);

// ---- device helpers ----------------------------------------------------------
// Reward sum in 2^-30 fixed point, rounded to nearest (ties to even), with exact
// fp32 steps only: the integer part of r and its fraction are converted apart.
// r is non-negative and below 2^31 (a reward sum never exceeds its visit count).
__device__ __forceinline__ unsigned long long reward_fixed(float r) {
    const float hi = floorf(r);
    const float lo = rintf(ldexpf(r - hi, 30));       // r - hi is exact, in [0, 1)
    return ((unsigned long long)(unsigned)hi << 30) + (unsigned)lo;
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) {
    return v < lo ? lo : (v > hi ? hi : v);
}

// Bounds of search g, clamped so that a malformed offset array cannot index
// outside [0, N] / [0, Ksum].
__device__ __forceinline__ void search_bounds(const int32_t* seg_off, const int32_t* koff,
                                              int g, int64_t N, int Ksum,
                                              int& n0, int& ng, int& k0, int& K) {
    int a = clampi(seg_off[g], 0, (int)N);
    int b = clampi(seg_off[g + 1], a, (int)N);
    int c = clampi(koff[g], 0, Ksum);
    int d = clampi(koff[g + 1], c, Ksum);
    n0 = a; ng = b - a; k0 = c; K = d - c;
}

// The first search g' >= g whose bounds satisfy take(n0, ng, k0, K), or G.  For kernels
// whose workgroups walk the searches of a candidate range but handle only some of them
// (a batch of a few long searches among thousands of short ones: a walk that looks at
// one search at a time spends 0.25 us of dependent loads on every search it skips).
// The 64 lanes of a wave test 64 searches at once; every wave of a workgroup gets the
// same answer on its own, so no barrier is involved.  `take` must also hold for the
// first search beyond the range, where the walk ends.
template <class F>
__device__ __forceinline__ int next_search(const int32_t* seg_off, const int32_t* koff, int g, int G,
                                           int64_t N, int Ksum, F take) {
    const int lane = threadIdx.x & 63;
    while (g < G) {
        const int gi = g + lane;
        bool hit = false;
        if (gi < G) {
            int n0, ng, k0, K;
            search_bounds(seg_off, koff, gi, N, Ksum, n0, ng, k0, K);
            hit = take(n0, ng, k0, K);
        }
        const unsigned long long m = __ballot(hit);
        if (m) return g + __ffsll((long long)m) - 1;
        g += 64;
    }
    return G;
}

}  // namespace kb
