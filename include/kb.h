/*
 * kb.h - C ABI of the MI355X arm-scoring library (libkernelband.so).
 *
 * One call scores the arms of a batch of G independent KernelBand searches
 * (Alg. 1, the steps between "compute phi(k)" and "sample k_t"):
 *
 *   kb_prune         hardware-aware pruning: a roofline lower bound on the
 *                    runtime reachable from each candidate and the binary mask
 *                    of candidates whose bound still beats the incumbent
 *                    (Assumption 1 / Eq. 2; mask of Eq. 5, strict '<').
 *   kb_cluster_step  one K-Means (Lloyd) step on the behavioural feature
 *                    vectors phi(k) under the L2 norm (Sec. 3.3; Assumption 2 /
 *                    Eq. 3): nearest centroid, then centroid = mean of members.
 *   kb_cluster       a fixed number of Lloyd steps starting from the first K
 *                    rows of each search (or caller-supplied centroids).
 *   kb_ucb_select    per-cluster arm statistics N_{i,s}, mu_{i,s}, the masked
 *                    UCB index mu + c*sqrt(ln t / N) and its argmax (Eq. 6),
 *                    then the member of the chosen cluster with the largest
 *                    headroom (Sec. 3.4, zero-temperature limit of the softmax
 *                    over V_hw).
 *   kb_round         the three in sequence on one stream.
 *   kb_cluster_geometry, kb_strategy_mask, kb_ucb_select_masked,
 *   kb_sample_signature, kb_update_stats, kb_seed_farthest,
 *   kb_seed_dsquared, kb_cluster_diameter
 *                    the remaining device-side steps of an iteration of Alg. 1:
 *                    cluster representatives, the mask in the paper's own form,
 *                    selection under that mask, the draw with the paper's
 *                    potential, and the statistics update.
 *   kb_iterate       several whole iterations of Alg. 1 (re-clustering every tau
 *                    iterations where |P| >= 2K, mask, selection, draw, update)
 *                    in one call, rewards supplied up front.
 *   kb_sample        the draw of k_t inside the chosen cluster with probability
 *                    proportional to exp(headroom) (Sec. 3.4), reproducible from
 *                    (seed, draw).
 *
 * Data model.  Search g owns the candidates seg_off[g] .. seg_off[g+1]-1 (its
 * frontier P_t) and the clusters koff[g] .. koff[g+1]-1.  N = seg_off[G] is the
 * total number of candidates, Ksum = koff[G] the total number of clusters.
 * A search with no candidates is legal.  Every search with candidates needs
 * 1 <= K_g <= N_g.
 *
 * Pointers.  Unless a comment says "host", every pointer is a DEVICE pointer to
 * memory the caller allocated and keeps owning.  The library allocates nothing
 * and keeps no state between calls (kb_ucb_select_static aside, which says what
 * it keeps); all scratch comes from the caller's workspace `ws` (device,
 * >= kb_workspace_bytes(), 256-byte aligned, contents undefined before and
 * after a call).  The workspace holds, besides small tables, a proposal and an
 * 8-byte entry (drift limit, cluster, |x|^2; at other times an fp64 distance) per
 * candidate and 12 bytes per cluster arm (integer statistics tables of the
 * selection step): about 12 * N + 12 * Ksum * S bytes; a batch with a search of more than 64 clusters
 * or 65536 candidates adds a bf16 copy of the features and per-candidate lists,
 * about (4*Dpad + 28) * N bytes more with Dpad = D rounded up to 16.  Two calls
 * may run concurrently only on different workspaces.
 * Arrays are dense, row-major, with no padding.  X, cent*, flops, bytes, bound,
 * visits and rsum must be 16-byte aligned.
 *
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default
 * stream).  Every call only enqueues work on it and returns without waiting.
 *
 * Errors.  Only the return code.  Host-visible arguments are validated before
 * anything is enqueued; contents of device memory cannot be (that would need a
 * synchronisation), so these are preconditions: offsets non-decreasing and
 * starting at 0, 1 <= K_g <= N_g, t_g >= 1, 0 <= rsum[k,s] <= visits[k,s],
 * visits >= 0 with per-cluster totals below 2^31, finite inputs.  Offsets are
 * only ever used after clamping to [0, N] / [0, Ksum], so a violated
 * precondition gives wrong numbers but no out-of-bounds access.
 *
 * Scale of the features.  The centroid sums are exact 64-bit fixed-point sums on
 * ONE grid per search, 2^-37 of the search's largest |x| or finer (2^-45 for a
 * search of 4096 candidates): a centroid coordinate is the fp32 rounding of the
 * exact mean up to that absolute step.  Features are expected to be
 * commensurately scaled, as the normalised phi of Sec. 3.2 is.  A feature column
 * whose values lie more than a factor 2^13 below the largest |x| of its search
 * starts to lose low-order bits of an fp32 centroid (beyond 2^20 below, its
 * centroids are off by more than 1e-5 relative); no error is reported.
 *
 * Limits of the compiled kernels (KB_EUNSUPPORTED beyond):
 *   1 <= D <= 64, 1 <= S, Kmax <= 256, Kmax*S <= 8192, N < 2^31,
 *   and G <= 1048576.
 */
#ifndef KB_H_
#define KB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KB_OK = 0,
    KB_EINVAL = 1,       /* NULL/misaligned required pointer, non-positive size, bad parameter */
    KB_EUNSUPPORTED = 2, /* shape beyond the compiled kernel limits */
    KB_EWORKSPACE = 3,   /* ws is NULL, misaligned or smaller than kb_workspace_bytes() */
    KB_EDEVICE = 4       /* a HIP call or kernel launch reported an error */
} kb_status;

#define KB_MAX_D 64
#define KB_MAX_K 256
#define KB_MAX_KS 8192
#define KB_MAX_G 1048576

/* Shape of a batch.  The scalars are HOST copies used for grid sizing and
 * validation; they must agree with the device arrays. */
typedef struct {
    int32_t G;              /* number of searches, >= 1 */
    int32_t D;              /* features per candidate (dimension of phi) */
    int32_t S;              /* strategies |S| per candidate */
    int64_t N;              /* total candidates = seg_off[G] */
    int32_t Kmax;           /* max over searches of K_g */
    int32_t Ksum;           /* koff[G] */
    int32_t Nmax;           /* max over searches of N_g */
    const int32_t *seg_off; /* device [G+1] */
    const int32_t *koff;    /* device [G+1] */
} kb_batch;

typedef struct {
    float peak_flops; /* flop/s of the target hardware, > 0 */
    float peak_bw;    /* B/s of the target hardware, > 0 */
    float c;          /* UCB exploration constant (the paper uses 2.0) */
    float prior_n;    /* pseudo-visits added to every cluster arm (Alg. 1 starts at 1), >= 0 */
    float prior_mu;   /* mean reward of the pseudo-visits (Alg. 1 starts at 0.5) */
    int32_t iters;    /* Lloyd steps for kb_cluster / kb_round, >= 0 (>= 1 for kb_round) */
    int32_t scorer;   /* how kb_cluster / kb_round form the fast distance scores of a Lloyd
                       * step: one of KB_SCORER_*; 0 is the default.  Every mode gives
                       * identical results (doubtful candidates are re-evaluated exactly in
                       * every mode); only speed differs.  kb_cluster_step always runs the
                       * default. */
    int32_t stop_early; /* 0: every search runs all `iters` Lloyd steps.  1: a search stops at
                       * its first step in which no candidate changes cluster - such a step
                       * leaves sums, sizes and centroids as they were, so every later step
                       * would repeat it and all outputs are the same bytes as with 0.
                       * Honoured by the kernels that keep a search in one workgroup;
                       * searches on the multi-workgroup path run all steps either way.
                       * (Searches of at most 64 candidates and 16 clusters that run one
                       * wave each always stop there.) */
} kb_params;

/* kb_params::scorer */
enum {
    /* bf16 x 3 split products on the matrix cores.  Searches on the one-workgroup
     * path (K_g <= 64 and N_g <= 65536 - 24576 in a batch of at most 32 searches
     * or 786432 candidates -,
     * chosen search by search) also keep distance
     * bounds: a candidate whose nearest centroid provably cannot have changed
     * since it was last scored (triangle inequality on how far the centroids
     * moved) is not scored again, the others are packed into dense tiles.  (A
     * batch of searches of at most 64 candidates and 16 clusters runs one wave per
     * search with exact fp32 / fp64 distances instead, and a search stops at its
     * first step without a move, after which nothing could change: same results.)  Rows
     * are fetched in 16-byte pieces when D is a multiple of 4 and feature by
     * feature otherwise (about a third slower). */
    KB_SCORER_DEFAULT = 0,
    /* fp32 fused multiply-adds on the vector ALU, every candidate scored in every
     * step: the reference the matrix-core scorers are measured against. */
    KB_SCORER_VECTOR_ALU = 1,
    /* matrix cores, every candidate scored in every step (no distance bounds; on
     * the multi-workgroup path this is what the default does as well). */
    KB_SCORER_MATRIX_EVERY = 2
};

/* Inputs and outputs of kb_round: the union of the arguments of the three
 * stages, with the same meaning and layout as in their own entry points. */
typedef struct {
    const float *X;          /* [N, D]  feature vectors phi(k) */
    const float *flops;      /* [N]     floating-point operations of candidate k */
    const float *bytes;      /* [N]     bytes moved by candidate k */
    const float *incumbent;  /* [G]     best runtime found so far in search g, seconds */
    const int32_t *visits;   /* [N, S]  times strategy s was applied to candidate k */
    const float *rsum;       /* [N, S]  sum of the rewards of those applications */
    const int64_t *t;        /* [G]     iteration counter of search g, >= 1 */
    float *bound;            /* [N]     out: roofline lower-bound runtime */
    uint8_t *alive;          /* [N]     out: 1 = bound < incumbent */
    int32_t *assign;         /* [N]     out: cluster of k, local to its search */
    float *cent;             /* [Ksum, D] out: centroids after the last step */
    int32_t *counts;         /* [Ksum]  out: cluster sizes */
    float *objective;        /* [G]     out: sum of squared distances, last step */
    int32_t *Ncs;            /* [Ksum, S] out */
    float *mu;               /* [Ksum, S] out */
    float *ucb;              /* [Ksum, S] out */
    int32_t *sel;            /* [G, 3]  out: (I, S*, k*) */
} kb_round_io;

/* Bytes of device workspace any entry point needs for this batch.  Pure host
 * function; returns 0 for a NULL or invalid batch. */
size_t kb_workspace_bytes(const kb_batch *batch, const kb_params *params);

/* Pruning (Assumption 1, Eq. 5).
 *   bound[k] = max(flops[k]/peak_flops, bytes[k]/peak_bw)   seconds, IEEE fp32
 *   alive[k] = bound[k] < incumbent[g(k)]                    (equality => pruned)
 * A pruned candidate cannot beat the incumbent even at the hardware limit; all
 * |S| arms of it are masked.  incumbent = +inf keeps everything ("no pruning
 * initially", Alg. 1).  bound may be NULL.  Needs no workspace. */
kb_status kb_prune(const kb_batch *batch, const kb_params *params,
                   const float *flops, const float *bytes,
                   const float *incumbent, float *bound, uint8_t *alive,
                   void *stream);

/* One Lloyd step from cent_in (Sec. 3.3).
 *   assign[k]   = lowest j minimising ||x_k - cent_in[j]||^2 within k's search
 *   objective[g]= sum over the search of that minimal squared distance
 *   counts[j]   = members of cluster j
 *   cent_out[j] = mean of the members; an empty cluster keeps cent_in[j]
 * cent_in and cent_out must not overlap.  A search with no candidates gets
 * objective 0 and nothing else written. */
kb_status kb_cluster_step(const kb_batch *batch, const float *X,
                          const float *cent_in, int32_t *assign,
                          float *cent_out, int32_t *counts, float *objective,
                          void *ws, size_t ws_bytes, void *stream);

/* params->iters Lloyd steps.  Initial centroids are cent_init ([Ksum, D]) or,
 * when it is NULL, the first K_g rows of each search.  Outputs are those of the
 * last step: assign, counts and objective refer to the centroids entering it,
 * cent is its updated centroids; identical to iterating kb_cluster_step.
 * iters == 0 only writes cent = the initial centroids.  cent_init and cent must
 * not overlap. */
kb_status kb_cluster(const kb_batch *batch, const kb_params *params,
                     const float *X, const float *cent_init, int32_t *assign,
                     float *cent, int32_t *counts, float *objective, void *ws,
                     size_t ws_bytes, void *stream);

/* Cluster-arm statistics, masked UCB and selection (Eq. 6, Sec. 3.4).
 *   Ncs[i,s] = sum of visits[k,s] over alive members k of cluster i
 *   mu[i,s]  = (sum of rsum[k,s] + prior_n*prior_mu) / (Ncs[i,s] + prior_n)
 *              (NaN when the denominator is 0)
 *   ucb[i,s] = mu + c*sqrt(ln t_g / (Ncs+prior_n))  if cluster i has an alive member
 *            = +inf  if it has one and the denominator is 0 (untried arm first)
 *            = -inf  if it has none (masked)
 *   sel[g]   = (I, S*, k*): (I, S*) = lowest flat index I*S+S* attaining the
 *              maximal ucb among clusters with an alive member (scores are
 *              compared in fp64 before rounding to fp32); k* = the alive member
 *              of cluster I with the smallest bound, lowest index on ties, as
 *              a GLOBAL candidate index; (-1,-1,-1) if no candidate is alive.
 * assign must hold values in [0, K_g). */
kb_status kb_ucb_select(const kb_batch *batch, const kb_params *params,
                        const int32_t *assign, const uint8_t *alive,
                        const float *bound, const int32_t *visits,
                        const float *rsum, const int64_t *t, int32_t *Ncs,
                        float *mu, float *ucb, int32_t *sel, void *ws,
                        size_t ws_bytes, void *stream);

/* kb_prune, then kb_cluster on ALL candidates (pruned ones are clustered too:
 * the frontier is partitioned first and masked afterwards, Alg. 1), then
 * kb_ucb_select with the mask, bounds and assignment just computed.
 * Requires params->iters >= 1.  Same outputs, byte for byte, as the three calls
 * one after the other; a batch of searches of at most 64 candidates and 16
 * clusters each takes, in the default scorer mode, a single launch in which one
 * wave carries a search through all three stages. */
kb_status kb_round(const kb_batch *batch, const kb_params *params,
                   const kb_round_io *io, void *ws, size_t ws_bytes,
                   void *stream);

/* kb_ucb_select for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same inputs, outputs, results and errors as kb_ucb_select,
 * without ws: the scratch (the scheduling order of the searches and, for
 * searches of more than 16384 candidates, the partial cluster-arm tables) lives
 * in a static device array of 2.9 MB inside the library, one copy per GPU, held
 * until the process ends.  The call allocates and frees nothing.  Limits
 * (KB_EUNSUPPORTED beyond): G <= KB_STATIC_MAX_G; and when Nmax > 16384 also
 * Ksum <= KB_STATIC_MAX_KSUM and Ksum * S <= KB_STATIC_MAX_KS.  The scratch
 * belongs to the device that is current when the call is made, which must be
 * the device of `stream`.  All calls on one GPU share it and it keeps the last
 * call's contents (every call rewrites what it reads): two calls that overlap on
 * one GPU - different streams or host threads - race; calls on one stream are
 * ordered and safe.  The address of the array is looked up on the first call on
 * each device and kept for the life of the process. */
#define KB_STATIC_MAX_G 65536
#define KB_STATIC_MAX_KSUM 65536
#define KB_STATIC_MAX_KS 131072
kb_status kb_ucb_select_static(const kb_batch *batch, const kb_params *params,
                               const int32_t *assign, const uint8_t *alive,
                               const float *bound, const int32_t *visits,
                               const float *rsum, const int64_t *t, int32_t *Ncs,
                               float *mu, float *ucb, int32_t *sel, void *stream);

/* Parameters of the in-cluster draw. */
typedef struct {
    uint64_t seed; /* key of the counter-based generator */
    uint64_t draw; /* number of the draw (e.g. the round t); distinct draws are independent */
    float tau;     /* softmax temperature, > 0 and finite (the paper's form is tau = 1) */
} kb_sample_params;

/* Draw of k_t inside the chosen cluster (Sec. 3.4; Alg. 1 "Sample k_t"):
 *   P(k) proportional to exp(V(k)/tau) over the members k of cluster I = sel[g][0]
 *   with alive[k] != 0, where V(k) = 1 - bound[k]/incumbent[g] is the fraction of
 *   the incumbent's runtime candidate k could still gain (its headroom; +inf as
 *   incumbent makes the draw uniform).
 * The draw is reproducible: u_k = (m + 1/2) 2^-52 with m the first 52 bits of
 * Philox4x32-10 (counter (k, 0, draw low, draw high), key (seed low, seed high),
 * k the global candidate index), and
 *   ksel[g] = argmax_k ( V(k)/tau - ln(-ln u_k) )       (Gumbel-max identity)
 * evaluated in fp64, lowest k on exact ties; -1 when I < 0 or the cluster has
 * no alive member.  tau -> 0 tends to the k* of kb_ucb_select.
 * sel is the [G,3] output of kb_ucb_select (device); only its first column is
 * read.  alive may be NULL (every candidate alive).  Keys must be finite:
 * incumbent > 0, tau a normal positive number. */
kb_status kb_sample(const kb_batch *batch, const kb_sample_params *sp,
                    const int32_t *assign, const uint8_t *alive,
                    const float *bound, const float *incumbent,
                    const int32_t *sel, int32_t *ksel, void *ws,
                    size_t ws_bytes, void *stream);

/* The same draw with the paper's own potential (Sec. 3.4):
 *   V_hw(k, S_t) = theta_sat - h[k, target[S_t]],  S_t = sel[g][1],
 * h [N,R] being the hardware signature of every candidate (share of peak
 * throughput of R resources) and target [S] the resource each strategy works on
 * (values in [0,R)).  Same generator, same variates and same tie rule as
 * kb_sample; alive may be NULL. */
kb_status kb_sample_signature(const kb_batch *batch, const kb_sample_params *sp,
                              const int32_t *assign, const uint8_t *alive,
                              int32_t R, const float *h, const int32_t *target,
                              float theta_sat, const int32_t *sel, int32_t *ksel,
                              void *ws, size_t ws_bytes, void *stream);

/* Representative and radius of every cluster (Sec. 3.3 "Representative
 * profiling"; Alg. 1 "Update centroids k_c"; covering term of Theorem 1).
 *   rep[j]    = GLOBAL index of the member of cluster j nearest cent[j] (squared
 *               L2 distance in fp64 from direct differences, exactly as the
 *               definition; lowest index on ties); -1 for an empty cluster
 *   radius[j] = largest distance from cent[j] to a member, rounded to fp32
 *               (0 for an empty cluster); diam(C_j) <= 2 radius[j]
 * X [N,D], cent [Ksum,D] (16-byte aligned), assign [N] with values in [0,K_g). */
kb_status kb_cluster_geometry(const kb_batch *batch, const float *X,
                              const float *cent, const int32_t *assign,
                              int32_t *rep, float *radius, void *ws,
                              size_t ws_bytes, void *stream);

/* diam(C_i), the largest distance between two members of cluster i (the quantity
 * in the approximation term L * max_i diam(C_i) of Theorem 1): every pair of
 * members, squared L2 distance from direct differences in fp32 (relative error
 * of a distance below (D + 2) 2^-24), square root of the largest.  diam [Ksum]
 * out; 0 for clusters with fewer than two members.  Work grows with the sum of
 * the squared cluster sizes. */
kb_status kb_cluster_diameter(const kb_batch *batch, const float *X,
                              const int32_t *assign, float *diam, void *ws,
                              size_t ws_bytes, void *stream);

/* Farthest-point initial centroids, an option beside "the first K rows" for the
 * cent_init of kb_cluster: cent[koff[g]] = the first row of search g, and every
 * further centroid is the row farthest from those chosen so far,
 *   argmax_k min_i ||x_k - c_i||^2      (fp64 from direct differences, exactly as
 * the definition; lowest k on ties).  The cover's largest radius is within a
 * factor two of the smallest possible one (the covering radius of Theorem 1's
 * approximation term).  cent [Ksum,D] out (exact copies of the chosen rows),
 * pick [Ksum] out: their global candidate indices (may be NULL).  K_g dependent
 * passes over the rows of each search: searches of up to 4096 rows are read once
 * and kept on chip by one workgroup each; a batch with longer searches (Nmax >
 * 4096) enqueues Kmax further launches that advance all of those by one centroid
 * each. */
kb_status kb_seed_farthest(const kb_batch *batch, const float *X, float *cent,
                           int32_t *pick, void *ws, size_t ws_bytes,
                           void *stream);

/* Randomised initial centroids in the manner of k-means++, the seeding of the
 * scikit-learn default the paper runs (Sec. 3.6): the first centroid of a search
 * is a uniformly drawn row, every further one is drawn with probability
 * proportional to its squared distance to the nearest centroid chosen so far.
 * Reproducible like kb_sample: the j-th centroid of a search is
 *   argmax_k ( ln D_k^2 - ln(-ln u_k) ),   D_k^2 = min_i ||x_k - c_i||^2  (fp64),
 * with u_k the variate of candidate k (global index) in draw number draw0 + j
 * under `seed` (ln D^2 replaced by 0 for j = 0), lowest k on exact ties; rows at
 * distance 0 are never drawn while another row exists.  Outputs as
 * kb_seed_farthest.  A batch that seeds again should move draw0 on by at least
 * Kmax. */
kb_status kb_seed_dsquared(const kb_batch *batch, const float *X, uint64_t seed,
                           uint64_t draw0, float *cent, int32_t *pick, void *ws,
                           size_t ws_bytes, void *stream);

/* The binary mask of Eq. 5 in the paper's own form,
 *   M[i,s] = [ h[rep[i], target[s]] < theta_sat ]        (0 for rep[i] < 0),
 * and nvalid[g] = the number of valid cluster arms of search g (K |S_valid| in
 * Theorem 1).  h [N,R], target [S] in [0,R), rep [Ksum] as returned by
 * kb_cluster_geometry, M [Ksum,S] out, nvalid [G] out.  Needs no workspace. */
kb_status kb_strategy_mask(const kb_batch *batch, int32_t R, const float *h,
                           const int32_t *target, const int32_t *rep,
                           float theta_sat, uint8_t *M, int32_t *nvalid,
                           void *stream);

/* kb_ucb_select with the cluster-arm mask of Eq. 6: arm (i,s) takes part in the
 * argmax iff cluster i has an alive member and M[i,s] != 0 (M == NULL: no
 * mask); a masked arm gets ucb = -inf.  Here alive may be NULL (every candidate
 * alive) and bound may be NULL (k* = the lowest-index alive member of I). */
kb_status kb_ucb_select_masked(const kb_batch *batch, const kb_params *params,
                               const int32_t *assign, const uint8_t *alive,
                               const float *bound, const uint8_t *M,
                               const int32_t *visits, const float *rsum,
                               const int64_t *t, int32_t *Ncs, float *mu,
                               float *ucb, int32_t *sel, void *ws,
                               size_t ws_bytes, void *stream);

/* The statistics update that ends an iteration of Alg. 1, for all searches at
 * once and in place.  With (I, S*) = sel[g][0..1], k = ksel[g], r = reward[g]:
 *   t[g] += 1                                              always
 *   if ok[g] != 0 and an arm and a candidate were chosen:
 *     Ncs[I,S*] += 1;  mu[I,S*] += (r - mu[I,S*]) / (Ncs[I,S*] + prior_n)
 *     visits[k,S*] += 1;  rsum[k,S*] += r      (the per-candidate history the
 *                       cluster statistics are rebuilt from after re-clustering)
 * reward [G] in [0,1], ok [G] (1 = the generated kernel was verified).  Entries
 * of sel / ksel outside their search are ignored. */
kb_status kb_update_stats(const kb_batch *batch, const kb_params *params,
                          const int32_t *sel, const int32_t *ksel,
                          const float *reward, const uint8_t *ok,
                          int32_t *visits, float *rsum, int32_t *Ncs, float *mu,
                          int64_t *t, void *stream);

/* Several iterations of Alg. 1 in one call, enqueued on the stream without any
 * host round trip: what is left of an iteration once generation, verification
 * and timing of the new kernel are taken out - their results, the reward r and
 * the verified flag of every round, are supplied up front.  Round r = 0 ..
 * rounds-1, iteration number it = t0 + r:
 *   if tau_recluster > 0 and it % tau_recluster == 0   ("if t mod tau = 0")
 *       kb_cluster (params->iters steps, params->scorer) on every search with
 *       N_g >= 2 K_g ("and |P| >= 2K"; the others keep their clustering), from
 *       the first K_g rows or - warm_start != 0 - from the current centroids;
 *       kb_cluster_geometry -> rep, radius; kb_strategy_mask -> M, nvalid
 *   kb_ucb_select_masked (alive as given, bound = NULL) -> Ncs, mu, ucb, sel_log[r]
 *       (the cluster-arm statistics are those an aggregation of visits / rsum over the
 *       alive members of every cluster gives, so they follow a re-clustering: they
 *       are aggregated in the first round and after every re-clustering, kept as
 *       integer tables in the workspace and advanced by the update step in between,
 *       which gives the same bits as aggregating again)
 *   kb_sample_signature, draw number sample.draw + r       -> ksel_log[r]
 *   kb_update_stats with reward[r], ok[r]                  -> visits, rsum, Ncs, mu, t
 * The frontier is fixed during the call (new kernels are appended by the caller
 * between calls).  assign, cent, counts, objective, rep, radius, M and nvalid are
 * in-out: they must hold a valid state on entry wherever the first round does not
 * rebuild them (no re-clustering in round 0, or searches with N_g < 2 K_g).
 * Validation and errors as in the calls it is made of; rounds >= 1, t0 >= 0. */
typedef struct {
    int32_t rounds;         /* T, number of iterations to run */
    int32_t tau_recluster;  /* re-cluster every this many iterations (the paper: 10); <= 0: never */
    int64_t t0;             /* iteration number of the first round (host copy) */
    int32_t warm_start;     /* 0: Lloyd from the first K_g rows; else from the current centroids */
    int32_t R;              /* resources in the hardware signature h */
    float theta_sat;        /* saturation threshold of Eq. 5 (the paper: 0.75 of peak) */
    kb_sample_params sample; /* seed, draw number of the first round, temperature */
} kb_iterate_params;

typedef struct {
    const float *X;         /* [N, D] */
    const float *h;         /* [N, R] hardware signature of every candidate */
    const int32_t *target;  /* [S] resource each strategy works on, in [0, R) */
    const uint8_t *alive;   /* [N] or NULL (every candidate alive) */
    const float *reward;    /* [rounds, G] reward of round r in search g, in [0, 1] */
    const uint8_t *ok;      /* [rounds, G] 1 = the kernel generated in round r verified */
    int32_t *visits;        /* [N, S] in-out */
    float *rsum;            /* [N, S] in-out */
    int64_t *t;             /* [G]    in-out */
    int32_t *assign;        /* [N]    in-out */
    float *cent;            /* [Ksum, D] in-out */
    int32_t *counts;        /* [Ksum] in-out */
    float *objective;       /* [G]    in-out */
    int32_t *rep;           /* [Ksum] in-out */
    float *radius;          /* [Ksum] in-out */
    uint8_t *M;             /* [Ksum, S] in-out */
    int32_t *nvalid;        /* [G]    in-out */
    int32_t *Ncs;           /* [Ksum, S] out: tables after the last round's update */
    float *mu;              /* [Ksum, S] out */
    float *ucb;             /* [Ksum, S] out: scores of the last round */
    int32_t *sel_log;       /* [rounds, G, 3] out: (I_t, S_t, lowest-index alive member of I_t) */
    int32_t *ksel_log;      /* [rounds, G] out: the sampled k_t */
} kb_iterate_io;

kb_status kb_iterate(const kb_batch *batch, const kb_params *params,
                     const kb_iterate_params *ip, const kb_iterate_io *io,
                     void *ws, size_t ws_bytes, void *stream);

/* Static, never NULL. */
const char *kb_status_str(kb_status status);

/* Library version, "major.minor". Static. */
const char *kb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KB_H_ */
