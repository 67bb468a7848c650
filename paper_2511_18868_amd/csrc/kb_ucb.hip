// Cluster-arm statistics, masked UCB index and arm selection (Eq. 6, Sec. 3.4).
//
// One workgroup per search streams the search's visits / reward-sum rows once
// (flat, coalesced 16-byte loads) and scatters them into K x S accumulators in
// LDS keyed by the candidate's cluster.  All accumulators are integers - visit
// counts as they are, reward sums in 2^-30 fixed point (a cluster's reward sum
// is below its visit count, which is below 2^31) - so the LDS atomics commute
// and the statistics are bit-identical from run to run.  The per-cluster "most
// headroom" candidate is a 64-bit atomic min over (ordered bound bits, index).
// Scores are formed in fp64 from the accumulators, compared in fp64, and
// rounded to fp32 on output.
#include "kb_internal.h"
#include "kb_ucb_dev.h"

namespace kb {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kUcbLong = 16384;     // searches longer than this are cut into candidate ranges

// Scatter the visits / reward sums of the alive candidates [q0, q1) of a search
// (indices local to the search) into K x S tables keyed by cluster.
//
// A candidate's two rows are cut into pieces of E values - 16 bytes when S is a
// multiple of 4, 8 bytes when it is even, single values otherwise (the rows start at
// multiples of 4 S bytes, so that is the alignment they have) - and T threads, the
// next power of two at or above the number of pieces, share a candidate: the
// thread-to-piece mapping is fixed, so no index arithmetic per step (with S = 6, the
// paper's own count, a loop over single values that divides every index by S ran at a
// quarter of the rate of S = 8).  Four candidates per thread are in flight: mask and
// cluster first, then the rows of the alive ones, then the atomics.
// EXACT: the pieces of a row are a power of two in number, one per thread of its group
// (no idle threads and no loop over pieces).
template <int E, bool EXACT>
__device__ __forceinline__ void ucb_accumulate_pieces(const UcbArgs& a, int n0, int K, int q0, int q1,
                                                      unsigned* Ncnt, unsigned long long* R,
                                                      unsigned* nalive, unsigned long long* kmin) {
    const int tid = threadIdx.x;
    const int S = a.S;
    const int pieces = S / E;
    int T = 1;
    while (T < pieces && T < kThreads) T <<= 1;
    const int rpp = kThreads / T;             // candidates per pass of the workgroup
    const int sq = tid & (T - 1), row = tid / T;
    constexpr int U = 4;
    for (int pb = q0 + row; pb < q1; pb += rpp * U) {
        bool al[U];
        int jj[U];
        float bd[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = pb + u * rpp;
            const int pc = p < q1 ? p : q1 - 1;
            al[u] = (a.alive ? a.alive[(size_t)n0 + pc] != 0 : true) && p < q1;
            jj[u] = a.assign[(size_t)n0 + pc];
            bd[u] = a.bound ? a.bound[(size_t)n0 + pc] : 0.f;
        }
        const auto piece = [&](int c) {
            int v[U][E];
            float r[U][E];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = pb + u * rpp;
#pragma unroll
                for (int e = 0; e < E; ++e) { v[u][e] = 0; r[u][e] = 0.f; }
                if (al[u]) {
                    const size_t at = ((size_t)n0 + p) * pieces + c;
                    if constexpr (E == 4) {
                        const int4 vv = reinterpret_cast<const int4*>(a.visits)[at];
                        const float4 rv = reinterpret_cast<const float4*>(a.rsum)[at];
                        v[u][0] = vv.x; v[u][1] = vv.y; v[u][2] = vv.z; v[u][3] = vv.w;
                        r[u][0] = rv.x; r[u][1] = rv.y; r[u][2] = rv.z; r[u][3] = rv.w;
                    } else if constexpr (E == 2) {
                        const int2 vv = reinterpret_cast<const int2*>(a.visits)[at];
                        const float2 rv = reinterpret_cast<const float2*>(a.rsum)[at];
                        v[u][0] = vv.x; v[u][1] = vv.y;
                        r[u][0] = rv.x; r[u][1] = rv.y;
                    } else {
                        v[u][0] = a.visits[at];
                        r[u][0] = a.rsum[at];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!al[u]) continue;
                const int j = (jj[u] >= 0 && jj[u] < K) ? jj[u] : 0;
                unsigned* nc = Ncnt + (size_t)j * S + c * E;
                unsigned long long* rr = R + (size_t)j * S + c * E;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    atomicAdd(nc + e, (unsigned)v[u][e]);
                    atomicAdd(rr + e, reward_fixed(r[u][e]));
                }
                if (c == 0) {         // the thread with a row's first piece also counts the candidate
                    atomicAdd(&nalive[j], 1u);
                    const unsigned long long key =
                        ((unsigned long long)ordered_bits(bd[u]) << 32) | (unsigned)(pb + u * rpp);
                    atomicMin(&kmin[j], key);
                }
            }
        };
        if constexpr (EXACT) {
            piece(sq);
        } else {
            for (int c = sq; c < pieces; c += T) piece(c);     // (one round unless a row has more than 256 pieces)
        }
    }
}


// E, EXACT: how the rows are cut (ucb_accumulate_pieces); instantiations of their own,
// so that each form has the registers it needs and no more (in one kernel the forms for
// odd strategy counts raised the count from 64 to 99 and halved the resident waves of all)
template <int E, bool EXACT>
__global__ void __launch_bounds__(kThreads) ucb_kernel(UcbArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int S = a.S;

    int g = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;
    g = clampi(g, 0, a.G - 1);
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (ng <= 0 || K <= 0) {
        if (tid < 3) a.sel[(size_t)g * 3 + tid] = -1;
        return;
    }
    if (a.mixed && ng > kUcbLong) return;     // the range kernels take this search
    const int KS = K * S;

    double* redv = reinterpret_cast<double*>(smem);                                      // [kWaves]
    int* redi = reinterpret_cast<int*>(smem + 32);                                       // [kWaves]
    unsigned long long* R = reinterpret_cast<unsigned long long*>(smem + 64);            // [Kmax*S]
    unsigned long long* kmin = R + (size_t)a.Kmax * S;                                   // [Kmax]
    unsigned* Ncnt = reinterpret_cast<unsigned*>(kmin + a.Kmax);                         // [Kmax*S]
    unsigned* nalive = Ncnt + (size_t)a.Kmax * S;                                        // [Kmax]

    for (int i = tid; i < KS; i += kThreads) { R[i] = 0ull; Ncnt[i] = 0u; }
    for (int i = tid; i < K; i += kThreads) { kmin[i] = ~0ull; nalive[i] = 0u; }
    __syncthreads();

    ucb_accumulate_pieces<E, EXACT>(a, n0, K, 0, ng, Ncnt, R, nalive, kmin);
    __syncthreads();

    if (a.keep) {
        // (a search is owned by this workgroup: plain stores)
        for (int i = tid; i < KS; i += kThreads) {
            a.gN[(size_t)k0 * S + i] = Ncnt[i];
            a.gR[(size_t)k0 * S + i] = R[i];
        }
        for (int i = tid; i < K; i += kThreads) { a.gnalive[k0 + i] = nalive[i]; a.gkmin[k0 + i] = kmin[i]; }
    }
    ucb_finish<kThreads>(a, g, n0, k0, K, Ncnt, R, nalive, kmin, redv, redi, tid);
}


// ---- short searches: a wave per search, four searches per workgroup, no barrier.
// A lane owns a candidate and adds its two rows to the wave's own tables; the same
// integer tables as above, so the same scores and the same selection.
__global__ void __launch_bounds__(kThreads) ucb_wave(UcbArgs a, int per) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = (int)blockIdx.x * kWaves + wv;
    if (g >= a.G) return;                 // (a whole wave leaves: no wave waits for another in this kernel)
    const int S = a.S;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (ng <= 0 || K <= 0) {
        if (lane < 3) a.sel[(size_t)g * 3 + lane] = -1;
        return;
    }
    const int KS = K * S;
    unsigned char* base = smem + (size_t)wv * per;
    unsigned long long* R = reinterpret_cast<unsigned long long*>(base);                 // [Kmax*S]
    unsigned long long* kmin = R + (size_t)a.Kmax * S;                                   // [Kmax]
    unsigned* Ncnt = reinterpret_cast<unsigned*>(kmin + a.Kmax);                         // [Kmax*S]
    unsigned* nalive = Ncnt + (size_t)a.Kmax * S;                                        // [Kmax]
    for (int i = lane; i < KS; i += kWave) { R[i] = 0ull; Ncnt[i] = 0u; }
    for (int i = lane; i < K; i += kWave) { kmin[i] = ~0ull; nalive[i] = 0u; }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    for (int p = lane; p < ng; p += kWave) {
        if (a.alive && !a.alive[(size_t)n0 + p]) continue;
        int j = a.assign[(size_t)n0 + p];
        j = (j >= 0 && j < K) ? j : 0;
        ucb_add_candidate(a, (size_t)n0 + p, p, j, a.bound ? a.bound[(size_t)n0 + p] : 0.f, Ncnt, R, nalive, kmin);
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    if (a.keep) {
        for (int i = lane; i < KS; i += kWave) {
            a.gN[(size_t)k0 * S + i] = Ncnt[i];
            a.gR[(size_t)k0 * S + i] = R[i];
        }
        for (int i = lane; i < K; i += kWave) { a.gnalive[k0 + i] = nalive[i]; a.gkmin[k0 + i] = kmin[i]; }
    }
    ucb_finish<kWave>(a, g, n0, k0, K, Ncnt, R, nalive, kmin, nullptr, nullptr, lane);
}


// ---- searches too long for one workgroup: partial tables per candidate range,
// ---- merged in global memory with integer atomics (still order-independent)
constexpr int kUcbRange = 8192;

__global__ void __launch_bounds__(kThreads) ucb_zero(UcbArgs a) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t0; i < (int64_t)a.Ksum * a.S; i += stride) { a.gN[i] = 0u; a.gR[i] = 0ull; }
    for (int64_t i = t0; i < a.Ksum; i += stride) { a.gnalive[i] = 0u; a.gkmin[i] = ~0ull; }
}

template <int E, bool EXACT>
__global__ void __launch_bounds__(kThreads) ucb_partial(UcbArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int S = a.S;
    const int64_t r0 = (int64_t)blockIdx.x * kUcbRange;
    if (r0 >= a.N) return;
    const int64_t r1 = r0 + kUcbRange < a.N ? r0 + kUcbRange : a.N;
    unsigned long long* R = reinterpret_cast<unsigned long long*>(smem + 64);
    unsigned long long* kmin = R + (size_t)a.Kmax * S;
    unsigned* Ncnt = reinterpret_cast<unsigned*>(kmin + a.Kmax);
    unsigned* nalive = Ncnt + (size_t)a.Kmax * S;
    // largest g with seg_off[g] <= r0
    int lo = 0, hi = a.G;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.seg_off[mid] <= r0) lo = mid; else hi = mid;
    }
    const auto mine = [&](int n0, int ng, int k0, int K) {
        return n0 >= r1 || (ng > 0 && K > 0 && !(a.mixed && ng <= kUcbLong));
    };
    for (int g = lo; (g = next_search(a.seg_off, a.koff, g, a.G, a.N, a.Ksum, mine)) < a.G; ++g) {
        int n0, ng, k0, K;
        search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
        if (K > a.Kmax) K = a.Kmax;
        if (n0 >= r1) break;
        if (ng <= 0 || K <= 0) continue;
        if (a.mixed && ng <= kUcbLong) continue;     // one workgroup takes this search whole
        const int64_t q0 = r0 > n0 ? r0 : n0;
        const int64_t q1 = r1 < (int64_t)n0 + ng ? r1 : (int64_t)n0 + ng;
        if (q0 >= q1) continue;
        const int KS = K * S;
        for (int i = tid; i < KS; i += kThreads) { R[i] = 0ull; Ncnt[i] = 0u; }
        for (int i = tid; i < K; i += kThreads) { kmin[i] = ~0ull; nalive[i] = 0u; }
        __syncthreads();
        ucb_accumulate_pieces<E, EXACT>(a, n0, K, (int)(q0 - n0), (int)(q1 - n0), Ncnt, R, nalive, kmin);
        __syncthreads();
        for (int i = tid; i < KS; i += kThreads) {
            if (Ncnt[i]) atomicAdd(&a.gN[(size_t)k0 * S + i], Ncnt[i]);
            if (R[i]) atomicAdd(&a.gR[(size_t)k0 * S + i], R[i]);
        }
        for (int i = tid; i < K; i += kThreads) {
            if (nalive[i]) {
                atomicAdd(&a.gnalive[k0 + i], nalive[i]);
                atomicMin(&a.gkmin[k0 + i], kmin[i]);
            }
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(kThreads) ucb_final(UcbArgs a) {
    __shared__ double redv[kWaves];
    __shared__ int redi[kWaves];
    const int g = blockIdx.x;
    int n0, ng, k0, K;
    search_bounds(a.seg_off, a.koff, g, a.N, a.Ksum, n0, ng, k0, K);
    if (K > a.Kmax) K = a.Kmax;
    if (a.mixed && ng <= kUcbLong) return;       // (uniform) done by ucb_kernel, empty searches included
    if (ng <= 0 || K <= 0) {
        if (threadIdx.x < 3) a.sel[(size_t)g * 3 + threadIdx.x] = -1;
        return;
    }
    ucb_finish<kThreads>(a, g, n0, k0, K, a.gN + (size_t)k0 * a.S, a.gR + (size_t)k0 * a.S,
                         a.gnalive + k0, a.gkmin + k0, redv, redi, (int)threadIdx.x);
}

}  // namespace

// bytes of one search's tables in ucb_wave
static int wave_table_bytes(const kb_batch& b) {
    const size_t kmax = b.Kmax > 0 ? b.Kmax : 1;
    return (int)(((kmax * b.S * 12 + kmax * 12) + 15) & ~(size_t)15);
}

bool ucb_wave_per_search(const kb_batch& b) {
    return b.G > 0 && b.Nmax <= kShortSearch && (size_t)wave_table_bytes(b) * kWaves <= 64 * 1024;
}

namespace {

// the aggregation kernels in the form that fits the strategy count (see ucb_accumulate_pieces)
template <int E, bool EXACT>
hipError_t launch_search_kernel(const UcbArgs& a, size_t lds, hipStream_t st) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ucb_kernel<E, EXACT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((ucb_kernel<E, EXACT>), dim3((unsigned)a.G), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}
template <int E, bool EXACT>
hipError_t launch_range_kernel(const UcbArgs& a, unsigned ranges, size_t lds, hipStream_t st) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ucb_partial<E, EXACT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((ucb_partial<E, EXACT>), dim3(ranges), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}
// form 0: 16-byte pieces, a power of two of them per row; 1: 16-byte pieces; 2: 8-byte; 3: single values
int row_form(int S) {
    if ((S & 3) == 0) {
        const int pieces = S >> 2;
        return ((pieces & (pieces - 1)) == 0 && pieces <= kThreads) ? 0 : 1;
    }
    return (S & 1) == 0 ? 2 : 3;
}
hipError_t launch_search_kernel(const UcbArgs& a, size_t lds, hipStream_t st) {
    switch (row_form(a.S)) {
        case 0: return launch_search_kernel<4, true>(a, lds, st);
        case 1: return launch_search_kernel<4, false>(a, lds, st);
        case 2: return launch_search_kernel<2, false>(a, lds, st);
        default: return launch_search_kernel<1, false>(a, lds, st);
    }
}
hipError_t launch_range_kernel(const UcbArgs& a, unsigned ranges, size_t lds, hipStream_t st) {
    switch (row_form(a.S)) {
        case 0: return launch_range_kernel<4, true>(a, ranges, lds, st);
        case 1: return launch_range_kernel<4, false>(a, ranges, lds, st);
        case 2: return launch_range_kernel<2, false>(a, ranges, lds, st);
        default: return launch_range_kernel<1, false>(a, ranges, lds, st);
    }
}

}  // namespace

hipError_t launch_ucb(const kb_batch& b, const UcbCall& c, hipStream_t st) {
    UcbArgs a = make_ucb_args(b, c);
    const size_t lds = 64 + (size_t)a.Kmax * b.S * 12 + (size_t)a.Kmax * 12;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (c.from_tables) {
        if (!c.gN) return hipErrorInvalidValue;
        hipLaunchKernelGGL(ucb_final, dim3((unsigned)b.G), dim3(kThreads), 0, st, a);
        return hipGetLastError();
    }
    if (c.keep_tables && !c.gN) return hipErrorInvalidValue;
    a.keep = c.keep_tables ? 1 : 0;
    if (c.chunked) {
        if (!c.gN) return hipErrorInvalidValue;
        // long searches: candidate ranges -> partial tables -> global tables -> scores;
        // in a batch of several searches the short ones get a workgroup each as usual
        const size_t items = (size_t)b.Ksum * b.S;
        unsigned zb = (unsigned)((items + kThreads - 1) / kThreads);
        if (zb > 4096u) zb = 4096u;
        if (zb == 0) zb = 1;
        hipLaunchKernelGGL(ucb_zero, dim3(zb), dim3(kThreads), 0, st, a);
        if (b.G > 1) {
            a.mixed = 1;
            const hipError_t e = launch_search_kernel(a, lds, st);
            if (e != hipSuccess) return e;
        }
        const unsigned ranges = (unsigned)((b.N + kUcbRange - 1) / kUcbRange);
        if (ranges) {
            const hipError_t e = launch_range_kernel(a, ranges, lds, st);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(ucb_final, dim3((unsigned)b.G), dim3(kThreads), 0, st, a);
        return hipGetLastError();
    }
    // a batch of short searches only: a wave per search (if four searches' tables fit the
    // 64 KB of LDS a kernel gets without asking); needs no scheduling order
    if (ucb_wave_per_search(b)) {
        const int per = wave_table_bytes(b);
        hipLaunchKernelGGL(ucb_wave, dim3((unsigned)((b.G + kWaves - 1) / kWaves)), dim3(kThreads),
                           (size_t)per * kWaves, st, a, per);
        return hipGetLastError();
    }
    return launch_search_kernel(a, lds, st);
}

}  // namespace kb
