// Hardware-aware pruning (Assumption 1 / Eq. 2, mask of Eq. 5) and the
// longest-first ordering of searches used by the per-search kernels.
#include "kb_internal.h"

namespace kb {

// Each thread owns 4 consecutive candidates: one 16-byte load per input array,
// one 16-byte store of the bound and one 4-byte store of the mask.  The search
// a candidate belongs to is found by a binary search over seg_off for the
// thread's first candidate and a forward walk for the other three.
//
// The divisions are IEEE-754 correctly rounded (no fast-math, no reciprocal):
// the incumbent is typically one of the bounds themselves, so the equality case
// of the strict compare must round exactly as on any other implementation.
__global__ void __launch_bounds__(256)
prune_kernel(int G, int64_t N, const int32_t* __restrict__ seg_off,
             const float* __restrict__ flops, const float* __restrict__ bytes,
             float peak_flops, float peak_bw, const float* __restrict__ incumbent,
             float* __restrict__ bound, uint8_t* __restrict__ alive, int alive_vec) {
    const int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i0 >= N) return;
    // largest g with seg_off[g] <= i0 (skips empty searches)
    int lo = 0, hi = G;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((int64_t)seg_off[mid] <= i0) lo = mid; else hi = mid;
    }
    int g = lo;
    int64_t end = seg_off[g + 1];
    float inc = incumbent[g];

    float f[4], b[4];
    const bool full = i0 + 3 < N;
    if (full) {
        const float4 fv = *reinterpret_cast<const float4*>(flops + i0);
        const float4 bv = *reinterpret_cast<const float4*>(bytes + i0);
        f[0] = fv.x; f[1] = fv.y; f[2] = fv.z; f[3] = fv.w;
        b[0] = bv.x; b[1] = bv.y; b[2] = bv.z; b[3] = bv.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool ok = i0 + e < N;
            f[e] = ok ? flops[i0 + e] : 0.0f;
            b[e] = ok ? bytes[i0 + e] : 0.0f;
        }
    }
    float r[4];
    uint8_t m[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t k = i0 + e;
        while (k >= end && g + 1 < G) {
            ++g;
            end = seg_off[g + 1];
            inc = incumbent[g];
        }
        const float t_compute = f[e] / peak_flops;
        const float t_memory = b[e] / peak_bw;
        r[e] = t_compute > t_memory ? t_compute : t_memory;
        m[e] = r[e] < inc ? 1 : 0;
    }
    if (full) {
        if (bound) *reinterpret_cast<float4*>(bound + i0) = make_float4(r[0], r[1], r[2], r[3]);
        if (alive_vec) {
            *reinterpret_cast<uchar4*>(alive + i0) = make_uchar4(m[0], m[1], m[2], m[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) alive[i0 + e] = m[e];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (i0 + e < N) {
                if (bound) bound[i0 + e] = r[e];
                alive[i0 + e] = m[e];
            }
        }
    }
}

hipError_t launch_prune(const kb_batch& b, float peak_flops, float peak_bw, const float* flops,
                        const float* bytes, const float* incumbent, float* bound, uint8_t* alive,
                        hipStream_t st) {
    const int64_t quads = (b.N + 3) / 4;
    const unsigned blocks = (unsigned)((quads + 255) / 256);
    const int alive_vec = ((uintptr_t)alive % 4) == 0;
    hipLaunchKernelGGL(prune_kernel, dim3(blocks), dim3(256), 0, st, b.G, b.N, b.seg_off, flops,
                       bytes, peak_flops, peak_bw, incumbent, bound, alive, alive_vec);
    return hipGetLastError();
}

// Per-search scheduling data, computed by one workgroup: the first tile of every
// search in the split-feature workspace, and the
// searches sorted by decreasing floor(log2(N_g * K_g)): a counting sort over 64
// buckets done by one workgroup.  The per-search kernels map blockIdx -> order[]
// so the hardware dispatcher starts the long searches first and fills the tail
// with short ones.  The order inside a bucket depends on atomics and may differ
// between runs; it only affects scheduling, never results.
__global__ void __launch_bounds__(1024)
order_kernel(int G, int64_t N, int Ksum, const int32_t* __restrict__ seg_off,
             const int32_t* __restrict__ koff, int32_t* __restrict__ order,
             int32_t* __restrict__ tile_off, int32_t* __restrict__ chunk_off) {
    __shared__ int hist[64];
    __shared__ int start[64];
    __shared__ long long part[32];
    const int tid = threadIdx.x;
    // tile_off = exclusive prefix sum of ceil(N_g / 32): each thread owns a
    // contiguous chunk of searches
    {
        const int chunk = (G + (int)blockDim.x - 1) / (int)blockDim.x;
        const int lo = tid * chunk < G ? tid * chunk : G;
        const int hi = lo + chunk < G ? lo + chunk : G;
        // two prefix sums at once: tiles of 32 candidates, and chunks of
        // kTilesPerChunk tiles (packed as low / high 32 bits while scanning)
        long long local = 0;
        for (int g = lo; g < hi; ++g) {
            int n0, ng, k0, K;
            search_bounds(seg_off, koff, g, N, Ksum, n0, ng, k0, K);
            const int tiles = (ng + 31) >> 5;
            local += (long long)tiles + ((long long)((tiles + kTilesPerChunk - 1) / kTilesPerChunk) << 32);
        }
        // exclusive prefix sum over the 1024 threads: shuffles inside each wave, then
        // the 16 wave totals
        const int lane = tid & 63, wv = tid >> 6;
        long long incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const long long t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) part[wv] = incl;
        __syncthreads();
        if (wv == 0) {
            const long long tot = lane < 16 ? part[lane] : 0;
            long long w = tot;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) {
                const long long t = __shfl_up(w, o);
                if (lane >= o) w += t;
            }
            if (lane < 16) part[16 + lane] = w - tot;
        }
        __syncthreads();
        long long acc = part[16 + wv] + incl - local;
        for (int g = lo; g < hi; ++g) {
            int n0, ng, k0, K;
            search_bounds(seg_off, koff, g, N, Ksum, n0, ng, k0, K);
            const int tiles = (ng + 31) >> 5;
            tile_off[g] = (int)(acc & 0xffffffffll);
            if (chunk_off) chunk_off[g] = (int)(acc >> 32);
            acc += (long long)tiles + ((long long)((tiles + kTilesPerChunk - 1) / kTilesPerChunk) << 32);
        }
        if (hi == G && lo < G) {
            tile_off[G] = (int)(acc & 0xffffffffll);
            if (chunk_off) chunk_off[G] = (int)(acc >> 32);
        }
        if (G == 0 && tid == 0) tile_off[0] = 0;
    }
    if (tid < 64) hist[tid] = 0;
    __syncthreads();
    for (int g = tid; g < G; g += blockDim.x) {
        int n0, ng, k0, K;
        search_bounds(seg_off, koff, g, N, Ksum, n0, ng, k0, K);
        const unsigned long long cost = (unsigned long long)ng * (unsigned long long)(K > 0 ? K : 1);
        const int bkt = cost ? 63 - __clzll((long long)cost) : 0;
        atomicAdd(&hist[63 - bkt], 1);   // bucket 0 = largest
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int i = 0; i < 64; ++i) { start[i] = acc; acc += hist[i]; }
    }
    __syncthreads();
    for (int g = tid; g < G; g += blockDim.x) {
        int n0, ng, k0, K;
        search_bounds(seg_off, koff, g, N, Ksum, n0, ng, k0, K);
        const unsigned long long cost = (unsigned long long)ng * (unsigned long long)(K > 0 ? K : 1);
        const int bkt = cost ? 63 - __clzll((long long)cost) : 0;
        const int pos = atomicAdd(&start[63 - bkt], 1);
        if (pos < G) order[pos] = g;
    }
}

hipError_t launch_order(const kb_batch& b, int32_t* order, int32_t* tile_off, int32_t* chunk_off,
                        hipStream_t st) {
    hipLaunchKernelGGL(order_kernel, dim3(1), dim3(1024), 0, st, b.G, b.N, b.Ksum, b.seg_off,
                       b.koff, order, tile_off, chunk_off);
    return hipGetLastError();
}

}  // namespace kb
