// C-ABI entry points: host-side validation, workspace layout and dispatch.
// Nothing here synchronises with the device or allocates memory.
#include "kb_internal.h"
#include <mutex>

namespace kb {

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

WsLayout ws_layout(const kb_batch& b) {
    WsLayout w;
    size_t off = 0;
    w.a_new = off;  off += align256(sizeof(int32_t) * (size_t)(b.N > 0 ? b.N : 1));
    w.order = off;  off += align256(sizeof(int32_t) * (size_t)b.G);
    w.misc = off;   off += align256(sizeof(int32_t) * 128);
    w.tile_off = off; off += align256(sizeof(int32_t) * ((size_t)b.G + 1));
    // every search rounds its candidates up to whole tiles of 32
    w.max_tiles = (size_t)(b.N / 32) + (size_t)b.G;
    w.use_big = cluster_uses_big(b);
    w.xn = w.split = off;
    if (w.use_big) {
        // only the multi-workgroup clustering path keeps |x|^2 and a bf16 copy of the features
        const size_t steps = (size_t)(b.D + 15) / 16;
        w.xn = off;     off += align256(sizeof(float) * (size_t)(b.N > 0 ? b.N : 1));
        w.split = off;  off += align256(w.max_tiles * steps * 2 * 64 * 16);
        w.big = big_ws_layout(b, off);
        off = w.big.end;
    }
    // cluster-arm tables of the selection step in global memory: searches of more than
    // 16384 candidates are aggregated there, and kb_iterate carries them from round to
    // round
    w.ucb_chunked = b.Nmax > 16384;
    {
        const size_t ks = (size_t)(b.Ksum > 0 ? b.Ksum : 1) * b.S, k = (size_t)(b.Ksum > 0 ? b.Ksum : 1);
        w.ucb_R = off;      off += align256(8 * ks);
        w.ucb_kmin = off;   off += align256(8 * k);
        w.ucb_N = off;      off += align256(4 * ks);
        w.ucb_nalive = off; off += align256(4 * k);
    }
    {
        const size_t k = (size_t)(b.Ksum > 0 ? b.Ksum : 1);
        w.geo_d2 = off;  off += align256(8 * (size_t)(b.N > 0 ? b.N : 1));
        w.geo_min = off; off += align256(8 * k);
        w.geo_max = off; off += align256(8 * k);
        w.dia_off = off; off += align256(4 * (k + 1));
        w.dia_toff = off; off += align256(4 * (k + 1));
        w.dia_bsum = off; off += align256(16 * (k / 4096 + 1));
    }
    {
        const size_t ranges = (size_t)((b.N + kSampleRange - 1) / kSampleRange) + 1;
        w.samp_key = off; off += align256(8 * 2 * ranges);
        w.samp_idx = off; off += align256(4 * 2 * ranges);
    }
    {
        const size_t ranges = seed_ranges(b);
        w.seed_key = off; off += align256(8 * 4 * ranges);
        w.seed_idx = off; off += align256(4 * 4 * ranges);
    }
    w.total = off;
    return w;
}

static bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

static kb_status check_batch(const kb_batch* b) {
    if (!b) return KB_EINVAL;
    if (b->G <= 0 || b->D <= 0 || b->S <= 0) return KB_EINVAL;
    if (b->N < 0 || b->Ksum < 0 || b->Kmax < 0 || b->Nmax < 0) return KB_EINVAL;
    if (!b->seg_off || !b->koff) return KB_EINVAL;
    if (b->Kmax > b->Nmax) return KB_EINVAL;
    if ((int64_t)b->Nmax > b->N || b->Kmax > b->Ksum) return KB_EINVAL;
    if (b->N > 0 && (b->Nmax == 0)) return KB_EINVAL;
    if (b->N >= ((int64_t)1 << 31)) return KB_EUNSUPPORTED;
    if (b->G > KB_MAX_G) return KB_EUNSUPPORTED;
    return KB_OK;
}

static kb_status check_cluster_shape(const kb_batch* b) {
    if (b->D > KB_MAX_D || b->Kmax > KB_MAX_K) return KB_EUNSUPPORTED;
    if (!cluster_supported(*b)) return KB_EUNSUPPORTED;
    return KB_OK;
}

static kb_status check_ws(const kb_batch* b, void* ws, size_t ws_bytes) {
    if (!ws || !aligned(ws, 256)) return KB_EWORKSPACE;
    if (ws_bytes < ws_layout(*b).total) return KB_EWORKSPACE;
    return KB_OK;
}

static kb_status dev(hipError_t e) { return e == hipSuccess ? KB_OK : KB_EDEVICE; }

static kb_status check_prune(const kb_params* p, const float* flops, const float* bytes,
                             const float* inc, const float* bound, const uint8_t* alive) {
    if (!p || !flops || !bytes || !inc || !alive) return KB_EINVAL;
    if (!(p->peak_flops > 0.0f) || !(p->peak_bw > 0.0f)) return KB_EINVAL;
    if (!aligned(flops, 16) || !aligned(bytes, 16) || (bound && !aligned(bound, 16)))
        return KB_EINVAL;
    return KB_OK;
}

static kb_status do_prune(const kb_batch* b, const kb_params* p, const float* flops,
                          const float* bytes, const float* inc, float* bound,
                          uint8_t* alive, hipStream_t st) {
    kb_status s = check_prune(p, flops, bytes, inc, bound, alive);
    if (s != KB_OK) return s;
    if (b->N == 0) return KB_OK;
    return dev(launch_prune(*b, p->peak_flops, p->peak_bw, flops, bytes, inc, bound, alive, st));
}

static kb_status check_cluster(const kb_batch* b, const float* X, const float* cent_init,
                               int32_t iters, const int32_t* assign, const float* cent,
                               const int32_t* counts, const float* objective) {
    if (!X || !cent) return KB_EINVAL;
    if (iters < 0) return KB_EINVAL;
    if (iters > 0 && (!assign || !counts || !objective)) return KB_EINVAL;
    if (!aligned(X, 16) || !aligned(cent, 16) || (cent_init && !aligned(cent_init, 16)))
        return KB_EINVAL;
    if (cent_init) {
        // the two centroid arrays must not overlap
        const char* a = (const char*)cent_init;
        const char* c = (const char*)cent;
        size_t bytes = sizeof(float) * (size_t)b->Ksum * b->D;
        if (a < c + bytes && c < a + bytes) return KB_EINVAL;
    }
    return check_cluster_shape(b);
}

static kb_status do_cluster(const kb_batch* b, const float* X, const float* cent_init,
                            int32_t iters, int scorer, int stop_early, int32_t* assign, float* cent,
                            int32_t* counts, float* objective, void* ws, hipStream_t st,
                            bool reclustering = false, bool* ordered = nullptr) {
    if (scorer < KB_SCORER_DEFAULT || scorer > KB_SCORER_MATRIX_EVERY) return KB_EINVAL;
    if (stop_early != 0 && stop_early != 1) return KB_EINVAL;
    // (a re-clustering may continue from the centroids it overwrites: every kernel
    // reads a search's initial centroids before it writes that search's new ones)
    kb_status s = check_cluster(b, X, reclustering ? nullptr : cent_init, iters, assign, cent,
                                counts, objective);
    if (s != KB_OK) return s;
    WsLayout w = ws_layout(*b);
    char* base = (char*)ws;
    int32_t* order = (int32_t*)(base + w.order);
    // (a lone search on the one-workgroup path needs neither a scheduling order nor
    // tile offsets, and neither does a batch that runs one wave per search: one launch less)
    const bool need_order = (b->G > 1 && !cluster_wave_per_search(*b, scorer)) || w.use_big;
    if (ordered) *ordered = need_order;
    if (need_order) {
        hipError_t e = launch_order(*b, order, (int32_t*)(base + w.tile_off),
                                    w.use_big ? (int32_t*)(base + w.big.chunk_off) : nullptr, st);
        if (e != hipSuccess) return KB_EDEVICE;
    }
    ClusterCall c;
    c.X = X; c.cent_init = cent_init; c.iters = iters; c.assign = assign;
    c.cent_out = cent; c.counts = counts; c.objective = objective;
    c.a_new = (int32_t*)(base + w.a_new); c.order = order;
    c.tile_off = (const int32_t*)(base + w.tile_off); c.xn = (float*)(base + w.xn);
    c.lim = (float*)(base + w.geo_d2);      // (the representative pass uses this array at other times)
    c.split = (void*)(base + w.split); c.max_tiles = (int64_t)w.max_tiles;
    c.scorer = scorer;
    c.stop_early = stop_early;
    c.guard = reclustering ? 1 : 0;
    c.mixed = 0;
    if (!w.use_big) return dev(launch_cluster(*b, c, st));
    // some search needs the multi-workgroup kernels; with more than one search in the
    // batch the others may not, and go to the one-workgroup kernel in the same call
    c.mixed = b->G > 1 ? 1 : 0;
    if (c.mixed) {
        hipError_t e = launch_cluster(*b, c, st);
        if (e != hipSuccess) return KB_EDEVICE;
    }
    return dev(launch_cluster_big(*b, c, w.big, base, st));
}

static kb_status check_ucb(const kb_batch* b, const kb_params* p, const int32_t* assign,
                           const uint8_t* alive, const float* bound, const int32_t* visits,
                           const float* rsum, const int64_t* t, const int32_t* Ncs,
                           const float* mu, const float* ucb, const int32_t* sel,
                           bool optional_mask_inputs = false) {
    if (!p || !assign || !visits || !rsum || !t || !Ncs || !mu || !ucb || !sel) return KB_EINVAL;
    if (!optional_mask_inputs && (!alive || !bound)) return KB_EINVAL;
    if (!(p->prior_n >= 0.0f) || !(p->c == p->c) || !(p->prior_mu == p->prior_mu)) return KB_EINVAL;
    if (!aligned(visits, 16) || !aligned(rsum, 16)) return KB_EINVAL;
    if (b->Kmax > KB_MAX_K || (int64_t)b->Kmax * b->S > KB_MAX_KS) return KB_EUNSUPPORTED;
    return KB_OK;
}

// device scratch of the selection step
struct UcbScratch {
    int32_t* order;                 // [G]
    int32_t* tile_off;              // [G + 1] (written by the ordering kernel, not read here)
    unsigned* gN;                   // cluster-arm tables in global memory (NULL: none; then no search
    unsigned long long* gR;         // may be longer than 16384 candidates)
    unsigned* gnalive;
    unsigned long long* gkmin;
    bool chunked;                   // the batch has a search that is aggregated in those tables
};

static UcbScratch ucb_scratch_in_ws(const kb_batch* b, void* ws) {
    const WsLayout w = ws_layout(*b);
    char* base = (char*)ws;
    UcbScratch u;
    u.order = (int32_t*)(base + w.order);
    u.tile_off = (int32_t*)(base + w.tile_off);
    u.gN = (unsigned*)(base + w.ucb_N); u.gR = (unsigned long long*)(base + w.ucb_R);
    u.gnalive = (unsigned*)(base + w.ucb_nalive); u.gkmin = (unsigned long long*)(base + w.ucb_kmin);
    u.chunked = w.ucb_chunked;
    return u;
}

static kb_status do_ucb(const kb_batch* b, const kb_params* p, const int32_t* assign,
                        const uint8_t* alive, const float* bound, const int32_t* visits,
                        const float* rsum, const int64_t* t, int32_t* Ncs, float* mu,
                        float* ucb, int32_t* sel, const UcbScratch& u, bool have_order,
                        hipStream_t st, const uint8_t* M = nullptr,
                        bool optional_mask_inputs = false, int tables = 0) {
    // tables: 0 = plain call; 1 = aggregate and leave every search's tables in u's global
    // arrays; 2 = no aggregation, scores and selection from those arrays as they stand
    kb_status s = check_ucb(b, p, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel,
                            optional_mask_inputs);
    if (s != KB_OK) return s;
    if (!have_order && b->G > 1 && !ucb_wave_per_search(*b)) {
        hipError_t e = launch_order(*b, u.order, u.tile_off, nullptr, st);
        if (e != hipSuccess) return KB_EDEVICE;
    }
    UcbCall c;
    c.assign = assign; c.alive = alive; c.bound = bound; c.M = M; c.visits = visits; c.rsum = rsum;
    c.t = t; c.c = p->c; c.prior_n = p->prior_n; c.prior_mu = p->prior_mu;
    c.Ncs = Ncs; c.mu = mu; c.ucb = ucb; c.sel = sel; c.order = u.order;
    c.gN = u.gN; c.gR = u.gR; c.gnalive = u.gnalive; c.gkmin = u.gkmin;
    c.chunked = u.chunked ? 1 : 0;
    c.keep_tables = tables == 1; c.from_tables = tables == 2;
    return dev(launch_ucb(*b, c, st));
}

// ---- selection step without a caller workspace ---------------------------------
// The scratch of kb_ucb_select_static: a file-scope device array, one copy per GPU
// the library runs on, held until the process ends.  Layout (all blocks 256-byte
// aligned): order [G], tile_off [G + 1], then the tables of the chunked path gR
// [Ksum * S] (8 bytes), gkmin [Ksum] (8), gN [Ksum * S] (4), gnalive [Ksum] (4).
constexpr size_t kStaticOrder = 0;
constexpr size_t kStaticTileOff = kStaticOrder + 4 * (size_t)KB_STATIC_MAX_G;
constexpr size_t kStaticR = kStaticTileOff + 4 * ((size_t)KB_STATIC_MAX_G + 64);
constexpr size_t kStaticKmin = kStaticR + 8 * (size_t)KB_STATIC_MAX_KS;
constexpr size_t kStaticN = kStaticKmin + 8 * (size_t)KB_STATIC_MAX_KSUM;
constexpr size_t kStaticNalive = kStaticN + 4 * (size_t)KB_STATIC_MAX_KS;
constexpr size_t kStaticBytes = kStaticNalive + 4 * (size_t)KB_STATIC_MAX_KSUM;
static_assert(kStaticTileOff % 256 == 0 && kStaticR % 256 == 0 && kStaticKmin % 256 == 0 &&
              kStaticN % 256 == 0 && kStaticNalive % 256 == 0, "blocks stay 256-byte aligned");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// Device address of `scratch` on the current device.  In host code the array's
// name is only a handle for the runtime, not an address a kernel can use, so the
// address is looked up once per device (every GPU has its own copy at its own
// address) and kept.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[kMaxDevices];     // zero-initialised: not looked up yet

static kb_status static_scratch(unsigned char** out) {
    int devno = -1;
    if (hipGetDevice(&devno) != hipSuccess || devno < 0 || devno >= kMaxDevices) return KB_EDEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[devno]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KB_EDEVICE;
        g_scratch_ptr[devno] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[devno];
    return KB_OK;
}

}  // namespace kb

using namespace kb;

extern "C" {

size_t kb_workspace_bytes(const kb_batch* batch, const kb_params* /*params*/) {
    if (check_batch(batch) != KB_OK) return 0;
    return ws_layout(*batch).total;
}

kb_status kb_prune(const kb_batch* batch, const kb_params* params, const float* flops,
                   const float* bytes, const float* incumbent, float* bound, uint8_t* alive,
                   void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    return do_prune(batch, params, flops, bytes, incumbent, bound, alive, (hipStream_t)stream);
}

kb_status kb_cluster_step(const kb_batch* batch, const float* X, const float* cent_in,
                          int32_t* assign, float* cent_out, int32_t* counts, float* objective,
                          void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!cent_in) return KB_EINVAL;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    return do_cluster(batch, X, cent_in, 1, KB_SCORER_DEFAULT, 0, assign, cent_out, counts, objective, ws,
                      (hipStream_t)stream);
}

kb_status kb_cluster(const kb_batch* batch, const kb_params* params, const float* X,
                     const float* cent_init, int32_t* assign, float* cent, int32_t* counts,
                     float* objective, void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!params) return KB_EINVAL;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    return do_cluster(batch, X, cent_init, params->iters, params->scorer, params->stop_early, assign, cent, counts,
                      objective, ws,
                      (hipStream_t)stream);
}

kb_status kb_ucb_select(const kb_batch* batch, const kb_params* params, const int32_t* assign,
                        const uint8_t* alive, const float* bound, const int32_t* visits,
                        const float* rsum, const int64_t* t, int32_t* Ncs, float* mu, float* ucb,
                        int32_t* sel, void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    // (arguments and shape limits before the workspace, whose size depends on the shape)
    s = check_ucb(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel);
    if (s != KB_OK) return s;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    return do_ucb(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel,
                  ucb_scratch_in_ws(batch, ws), false, (hipStream_t)stream);
}

kb_status kb_ucb_select_masked(const kb_batch* batch, const kb_params* params,
                               const int32_t* assign, const uint8_t* alive, const float* bound,
                               const uint8_t* M, const int32_t* visits, const float* rsum,
                               const int64_t* t, int32_t* Ncs, float* mu, float* ucb, int32_t* sel,
                               void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    s = check_ucb(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel, true);
    if (s != KB_OK) return s;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    return do_ucb(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel,
                  ucb_scratch_in_ws(batch, ws), false, (hipStream_t)stream, M, true);
}

kb_status kb_ucb_select_static(const kb_batch* batch, const kb_params* params,
                               const int32_t* assign, const uint8_t* alive, const float* bound,
                               const int32_t* visits, const float* rsum, const int64_t* t,
                               int32_t* Ncs, float* mu, float* ucb, int32_t* sel, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    // sizes beyond the static scratch
    const bool chunked = batch->Nmax > 16384;
    if (batch->G > KB_STATIC_MAX_G) return KB_EUNSUPPORTED;
    if (chunked && (batch->Ksum > KB_STATIC_MAX_KSUM ||
                    (int64_t)batch->Ksum * batch->S > KB_STATIC_MAX_KS))
        return KB_EUNSUPPORTED;
    s = check_ucb(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel);
    if (s != KB_OK) return s;
    unsigned char* base = nullptr;
    s = static_scratch(&base);
    if (s != KB_OK) return s;
    UcbScratch u;
    u.order = (int32_t*)(base + kStaticOrder);
    u.tile_off = (int32_t*)(base + kStaticTileOff);
    u.gN = nullptr; u.gR = nullptr; u.gnalive = nullptr; u.gkmin = nullptr;
    u.chunked = chunked;
    if (chunked) {
        u.gR = (unsigned long long*)(base + kStaticR);
        u.gkmin = (unsigned long long*)(base + kStaticKmin);
        u.gN = (unsigned*)(base + kStaticN);
        u.gnalive = (unsigned*)(base + kStaticNalive);
    }
    return do_ucb(batch, params, assign, alive, bound, visits, rsum, t, Ncs, mu, ucb, sel, u, false,
                  (hipStream_t)stream);
}

kb_status kb_cluster_geometry(const kb_batch* batch, const float* X, const float* cent,
                              const int32_t* assign, int32_t* rep, float* radius, void* ws,
                              size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!X || !cent || !assign || !rep || !radius) return KB_EINVAL;
    if (!aligned(X, 16) || !aligned(cent, 16)) return KB_EINVAL;
    if (batch->D > KB_MAX_D || batch->Kmax > KB_MAX_K) return KB_EUNSUPPORTED;
    if (geometry_lds_bytes(batch->Kmax > 0 ? batch->Kmax : 1, batch->D) > 160 * 1024)
        return KB_EUNSUPPORTED;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    WsLayout w = ws_layout(*batch);
    char* base = (char*)ws;
    GeoCall c;
    c.X = X; c.cent = cent; c.assign = assign; c.rep = rep; c.radius = radius;
    c.d2 = (double*)(base + w.geo_d2);
    c.gmin = (unsigned long long*)(base + w.geo_min);
    c.gmax = (unsigned long long*)(base + w.geo_max);
    return dev(launch_geometry(*batch, c, (hipStream_t)stream));
}

kb_status kb_cluster_diameter(const kb_batch* batch, const float* X, const int32_t* assign,
                              float* diam, void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!X || !assign || !diam) return KB_EINVAL;
    if (!aligned(X, 16)) return KB_EINVAL;
    if (batch->D > KB_MAX_D || batch->Kmax > KB_MAX_K) return KB_EUNSUPPORTED;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    WsLayout w = ws_layout(*batch);
    char* base = (char*)ws;
    DiameterCall c;
    c.X = X; c.assign = assign; c.diam = diam;
    // the grouped index list and the per-cluster counters live in buffers the
    // clustering and the representative pass use at other times
    c.perm = (int32_t*)(base + w.a_new);
    c.cnt = (int32_t*)(base + w.geo_min);
    c.off = (int32_t*)(base + w.dia_off);
    c.toff = (int32_t*)(base + w.dia_toff);
    c.bsum = (long long*)(base + w.dia_bsum);
    return dev(launch_diameter(*batch, c, (hipStream_t)stream));
}

static kb_status do_seed(const kb_batch* batch, const float* X, float* cent, int32_t* pick,
                         void* ws, size_t ws_bytes, void* stream, int dsquared, uint64_t seed,
                         uint64_t draw0) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!X || !cent) return KB_EINVAL;
    if (!aligned(X, 16) || !aligned(cent, 16)) return KB_EINVAL;
    if (batch->D > KB_MAX_D) return KB_EUNSUPPORTED;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    WsLayout w = ws_layout(*batch);
    char* base = (char*)ws;
    int32_t* order = (int32_t*)(base + w.order);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = launch_order(*batch, order, (int32_t*)(base + w.tile_off), nullptr, st);
    if (e != hipSuccess) return KB_EDEVICE;
    return dev(launch_seed(*batch, X, cent, pick, (double*)(base + w.geo_d2),
                           (double*)(base + w.seed_key), (int32_t*)(base + w.seed_idx), order,
                           dsquared, seed, draw0, st));
}

kb_status kb_seed_farthest(const kb_batch* batch, const float* X, float* cent, int32_t* pick,
                           void* ws, size_t ws_bytes, void* stream) {
    return do_seed(batch, X, cent, pick, ws, ws_bytes, stream, 0, 0, 0);
}

kb_status kb_seed_dsquared(const kb_batch* batch, const float* X, uint64_t seed, uint64_t draw0,
                           float* cent, int32_t* pick, void* ws, size_t ws_bytes, void* stream) {
    return do_seed(batch, X, cent, pick, ws, ws_bytes, stream, 1, seed, draw0);
}

kb_status kb_strategy_mask(const kb_batch* batch, int32_t R, const float* h, const int32_t* target,
                           const int32_t* rep, float theta_sat, uint8_t* M, int32_t* nvalid,
                           void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (R <= 0 || !h || !target || !rep || !M || !nvalid) return KB_EINVAL;
    if (!(theta_sat == theta_sat)) return KB_EINVAL;
    return dev(launch_strategy_mask(*batch, R, h, target, rep, theta_sat, M, nvalid,
                                    (hipStream_t)stream));
}

kb_status kb_update_stats(const kb_batch* batch, const kb_params* params, const int32_t* sel,
                          const int32_t* ksel, const float* reward, const uint8_t* ok,
                          int32_t* visits, float* rsum, int32_t* Ncs, float* mu, int64_t* t,
                          void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!params || !sel || !ksel || !reward || !ok || !visits || !rsum || !Ncs || !mu || !t)
        return KB_EINVAL;
    if (!(params->prior_n >= 0.0f)) return KB_EINVAL;
    return dev(launch_update_stats(*batch, params->prior_n, sel, ksel, reward, ok, visits, rsum,
                                   Ncs, mu, t, (hipStream_t)stream));
}

kb_status kb_sample_signature(const kb_batch* batch, const kb_sample_params* sp,
                              const int32_t* assign, const uint8_t* alive, int32_t R,
                              const float* h, const int32_t* target, float theta_sat,
                              const int32_t* sel, int32_t* ksel, void* ws, size_t ws_bytes,
                              void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!sp || !assign || R <= 0 || !h || !target || !sel || !ksel) return KB_EINVAL;
    if (!(sp->tau > 0.0f) || !(sp->tau < INFINITY) || !(theta_sat == theta_sat)) return KB_EINVAL;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    WsLayout w = ws_layout(*batch);
    char* base = (char*)ws;
    SampleCall c;
    c.assign = assign; c.alive = alive; c.bound = nullptr; c.incumbent = nullptr; c.sel = sel;
    c.h = h; c.target = target; c.R = R; c.theta_sat = theta_sat;
    c.seed = sp->seed; c.draw = sp->draw; c.tau = sp->tau; c.ksel = ksel;
    c.slot_key = (double*)(base + w.samp_key); c.slot_idx = (int32_t*)(base + w.samp_idx);
    return dev(launch_sample(*batch, c, (hipStream_t)stream));
}

kb_status kb_sample(const kb_batch* batch, const kb_sample_params* sp, const int32_t* assign,
                    const uint8_t* alive, const float* bound, const float* incumbent,
                    const int32_t* sel, int32_t* ksel, void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!sp || !assign || !bound || !incumbent || !sel || !ksel) return KB_EINVAL;
    if (!(sp->tau > 0.0f) || !(sp->tau < INFINITY)) return KB_EINVAL;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    WsLayout w = ws_layout(*batch);
    char* base = (char*)ws;
    SampleCall c;
    c.assign = assign; c.alive = alive; c.bound = bound; c.incumbent = incumbent; c.sel = sel;
    c.h = nullptr; c.target = nullptr; c.R = 1; c.theta_sat = 0.0f;
    c.seed = sp->seed; c.draw = sp->draw; c.tau = sp->tau; c.ksel = ksel;
    c.slot_key = (double*)(base + w.samp_key); c.slot_idx = (int32_t*)(base + w.samp_idx);
    return dev(launch_sample(*batch, c, (hipStream_t)stream));
}

kb_status kb_round(const kb_batch* batch, const kb_params* params, const kb_round_io* io,
                   void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!params || !io) return KB_EINVAL;
    if (params->iters < 1) return KB_EINVAL;
    if (params->scorer < KB_SCORER_DEFAULT || params->scorer > KB_SCORER_MATRIX_EVERY) return KB_EINVAL;
    if (params->stop_early != 0 && params->stop_early != 1) return KB_EINVAL;
    if (!io->bound) return KB_EINVAL;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    // validate every stage before enqueueing anything
    s = check_prune(params, io->flops, io->bytes, io->incumbent, io->bound, io->alive);
    if (s != KB_OK) return s;
    s = check_cluster(batch, io->X, nullptr, params->iters, io->assign, io->cent, io->counts,
                      io->objective);
    if (s != KB_OK) return s;
    s = check_ucb(batch, params, io->assign, io->alive, io->bound, io->visits, io->rsum, io->t,
                  io->Ncs, io->mu, io->ucb, io->sel);
    if (s != KB_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if (batch->G > 0 && round_in_one_launch(*batch, params->scorer)) {
        // very short searches only: the three stages of every search in one wave, one launch
        ClusterCall c{};
        c.X = io->X; c.iters = params->iters; c.assign = io->assign; c.cent_out = io->cent;
        c.counts = io->counts; c.objective = io->objective; c.scorer = params->scorer;
        UcbCall u{};
        u.assign = io->assign; u.alive = io->alive; u.bound = io->bound; u.visits = io->visits;
        u.rsum = io->rsum; u.t = io->t; u.c = params->c; u.prior_n = params->prior_n;
        u.prior_mu = params->prior_mu; u.Ncs = io->Ncs; u.mu = io->mu; u.ucb = io->ucb; u.sel = io->sel;
        return dev(launch_round_wave(*batch, c, u, io->flops, io->bytes, io->incumbent,
                                     params->peak_flops, params->peak_bw, io->bound, io->alive, st));
    }
    s = do_prune(batch, params, io->flops, io->bytes, io->incumbent, io->bound, io->alive, st);
    if (s != KB_OK) return s;
    s = do_cluster(batch, io->X, nullptr, params->iters, params->scorer, params->stop_early, io->assign, io->cent,
                   io->counts, io->objective, ws, st);
    if (s != KB_OK) return s;
    return do_ucb(batch, params, io->assign, io->alive, io->bound, io->visits, io->rsum, io->t,
                  io->Ncs, io->mu, io->ucb, io->sel, ucb_scratch_in_ws(batch, ws), true, st);
}

kb_status kb_iterate(const kb_batch* batch, const kb_params* params, const kb_iterate_params* ip,
                     const kb_iterate_io* io, void* ws, size_t ws_bytes, void* stream) {
    kb_status s = check_batch(batch);
    if (s != KB_OK) return s;
    if (!params || !ip || !io) return KB_EINVAL;
    if (ip->rounds < 1 || ip->t0 < 0 || ip->R <= 0) return KB_EINVAL;
    if (!(ip->theta_sat == ip->theta_sat)) return KB_EINVAL;
    if (!(ip->sample.tau > 0.0f) || !(ip->sample.tau < INFINITY)) return KB_EINVAL;
    if (!io->X || !io->h || !io->target || !io->reward || !io->ok || !io->visits || !io->rsum ||
        !io->t || !io->assign || !io->cent || !io->counts || !io->objective || !io->rep ||
        !io->radius || !io->M || !io->nvalid || !io->Ncs || !io->mu || !io->ucb || !io->sel_log ||
        !io->ksel_log)
        return KB_EINVAL;
    if (!aligned(io->X, 16) || !aligned(io->cent, 16)) return KB_EINVAL;
    const bool recluster = ip->tau_recluster > 0;
    if (recluster && params->iters < 1) return KB_EINVAL;
    if (params->scorer < KB_SCORER_DEFAULT || params->scorer > KB_SCORER_MATRIX_EVERY) return KB_EINVAL;
    if (params->stop_early != 0 && params->stop_early != 1) return KB_EINVAL;
    s = check_ws(batch, ws, ws_bytes);
    if (s != KB_OK) return s;
    // validate every stage before enqueueing anything
    s = check_ucb(batch, params, io->assign, io->alive, nullptr, io->visits, io->rsum, io->t, io->Ncs,
                  io->mu, io->ucb, io->sel_log, true);
    if (s != KB_OK) return s;
    if (recluster) {
        s = check_cluster(batch, io->X, nullptr, params->iters, io->assign, io->cent, io->counts,
                          io->objective);
        if (s != KB_OK) return s;
        if (geometry_lds_bytes(batch->Kmax > 0 ? batch->Kmax : 1, batch->D) > 160 * 1024)
            return KB_EUNSUPPORTED;
    }
    hipStream_t st = (hipStream_t)stream;
    const WsLayout w = ws_layout(*batch);
    char* base = (char*)ws;
    const size_t G = (size_t)batch->G;
    bool have_order = false;        // the scheduling order in ws, computed by the first stage that needs it
    bool ordered = false;
    // The cluster-arm tables (visit counts and fixed-point reward sums of the alive
    // members of every cluster) are aggregated from the per-candidate history in the
    // first round and after every re-clustering, kept in the workspace, and advanced by
    // the update step in between: integer tables, so the carried ones equal a fresh
    // aggregation bit for bit and a round without re-clustering reads K_g*S entries per
    // search instead of N_g*S.
    const UcbScratch us = ucb_scratch_in_ws(batch, ws);
    bool tables_valid = false;
    for (int32_t r = 0; r < ip->rounds; ++r) {
        const bool now = recluster && ((ip->t0 + r) % ip->tau_recluster) == 0;
        if (now) {
            // K-Means on the frontier wherever |P| >= 2K, then the cluster representatives
            // and the mask their hardware signatures give (Alg. 1; Eq. 5)
            s = do_cluster(batch, io->X, ip->warm_start ? io->cent : nullptr, params->iters,
                           params->scorer, params->stop_early, io->assign, io->cent, io->counts, io->objective, ws, st,
                           true, &ordered);
            if (s != KB_OK) return s;
            have_order = have_order || ordered;
            tables_valid = false;
            GeoCall gc;
            gc.X = io->X; gc.cent = io->cent; gc.assign = io->assign; gc.rep = io->rep;
            gc.radius = io->radius; gc.d2 = (double*)(base + w.geo_d2);
            gc.gmin = (unsigned long long*)(base + w.geo_min);
            gc.gmax = (unsigned long long*)(base + w.geo_max);
            if (launch_geometry(*batch, gc, st) != hipSuccess) return KB_EDEVICE;
            if (launch_strategy_mask(*batch, ip->R, io->h, io->target, io->rep, ip->theta_sat, io->M,
                                     io->nvalid, st) != hipSuccess)
                return KB_EDEVICE;
        }
        int32_t* sel = io->sel_log + (size_t)r * G * 3;
        int32_t* ksel = io->ksel_log + (size_t)r * G;
        // the cluster-arm tables are rebuilt from the per-candidate history, so they
        // follow every re-clustering; masked UCB argmax (Eq. 6)
        s = do_ucb(batch, params, io->assign, io->alive, nullptr, io->visits, io->rsum, io->t,
                   io->Ncs, io->mu, io->ucb, sel, us, have_order, st, io->M, true,
                   tables_valid ? 2 : 1);
        if (s != KB_OK) return s;
        have_order = true;
        tables_valid = true;
        // draw of k_t with the potential theta_sat - h (Sec. 3.4)
        SampleCall sc;
        sc.assign = io->assign; sc.alive = io->alive; sc.bound = nullptr; sc.incumbent = nullptr;
        sc.sel = sel; sc.h = io->h; sc.target = io->target; sc.R = ip->R; sc.theta_sat = ip->theta_sat;
        sc.seed = ip->sample.seed; sc.draw = ip->sample.draw + (uint64_t)r; sc.tau = ip->sample.tau;
        sc.ksel = ksel;
        sc.slot_key = (double*)(base + w.samp_key); sc.slot_idx = (int32_t*)(base + w.samp_idx);
        if (launch_sample(*batch, sc, st) != hipSuccess) return KB_EDEVICE;
        // reward of the generated kernel -> statistics (Alg. 1, last lines)
        if (launch_update_stats(*batch, params->prior_n, sel, ksel, io->reward + (size_t)r * G,
                                io->ok + (size_t)r * G, io->visits, io->rsum, io->Ncs, io->mu, io->t,
                                st, io->assign, io->alive, us.gN, us.gR) != hipSuccess)
            return KB_EDEVICE;
    }
    return KB_OK;
}

const char* kb_status_str(kb_status status) {
    switch (status) {
        case KB_OK: return "KB_OK";
        case KB_EINVAL: return "KB_EINVAL: invalid argument";
        case KB_EUNSUPPORTED: return "KB_EUNSUPPORTED: shape beyond the compiled kernel limits";
        case KB_EWORKSPACE: return "KB_EWORKSPACE: workspace missing, misaligned or too small";
        case KB_EDEVICE: return "KB_EDEVICE: HIP reported an error";
    }
    return "KB_E?: unknown status";
}

const char* kb_version(void) { return "0.6"; }

}  // extern "C"
