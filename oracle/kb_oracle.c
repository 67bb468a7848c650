/*
 * CPU oracle for the arm-scoring pass of a KernelBand search round.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code with the GPU path and the
 * product never calls it; only tests, the smoke check and the benchmark's CPU
 * baseline leg may load it.
 *
 * What it computes, with the passage of the paper each part follows:
 *
 *   kbo_prune        hardware-aware gain bound made concrete as a roofline
 *                    lower-bound runtime per candidate, and the binary mask of
 *                    arms that can still beat the incumbent
 *                    (Assumption 1 / Eq. 2; mask Eq. 5 with strict '<').
 *   kbo_assign,      one K-Means (Lloyd) step on the behavioural features phi(k)
 *   kbo_update,      under the L2 norm of Assumption 2 / Eq. 3: nearest centroid,
 *   kbo_cluster_step then centroid = mean of members (Sec. 3.3 "Periodic
 *                    re-clustering"; Alg. 1 "KMeans" and "Update centroids").
 *   kbo_cluster      a fixed number of such steps from the first K rows.
 *   kbo_ucb_select   per-cluster visit counts N_{i,s} and mean rewards mu_{i,s},
 *                    the masked UCB index mu + c sqrt(ln t / N) and its argmax
 *                    over valid cluster arms (Eq. 6), then the member of the
 *                    chosen cluster with the most headroom (Sec. 3.4, zero-
 *                    temperature limit of the softmax over V_hw).
 *   kbo_round        the three in sequence.
 *   kbo_cluster_geometry  the representative (centroid kernel) of each cluster
 *                    and the cluster radius (Sec. 3.3; Theorem 1's covering term).
 *   kbo_cluster_diameter  the largest distance between two members of a cluster
 *                    (diam(C_i) of Theorem 1).
 *   kbo_seed_farthest     farthest-point initial centroids (greedy cover; the
 *                    covering radius of Theorem 1's approximation term).
 *   kbo_seed_dsquared     randomised initial centroids drawn with probability
 *                    proportional to the squared distance to the chosen ones
 *                    (k-means++ seeding, the scikit-learn default of Sec. 3.6).
 *   kbo_strategy_mask     the mask of Eq. 5 in the paper's own form, from the
 *                    hardware signature of the representatives.
 *   kbo_update_stats the statistics update that ends an iteration of Alg. 1.
 *   kbo_sample       the draw of k_t inside the chosen cluster with probability
 *                    proportional to exp(headroom) (Sec. 3.4; Alg. 1 "Sample
 *                    k_t"), made reproducible by a counter-based generator and
 *                    the Gumbel-max identity.
 *
 * Arithmetic: fp64 everywhere, straight loops in index order, no blocking, no
 * reordering - except the roofline bound, which is computed in fp32 on purpose:
 * the incumbent is one of the candidates' own bounds, so the equality case of
 * the strict compare must round the same way on every implementation (IEEE
 * single-precision division, round to nearest even).
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math).
 * The only parallelism is an OpenMP loop over independent searches.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KBO_NEAR_TIE_REL 1e-6
#define KBO_TINY 1e-30

/* ------------------------------------------------------------------ prune */

/* bound[k] = max(flops[k]/peak_flops, bytes[k]/peak_bw) in seconds (fp32);
 * alive[k] = bound[k] < incumbent[g(k)].  A pruned candidate therefore has
 * bound >= incumbent: even at the hardware limit it cannot beat the best
 * runtime already found.  bound may be NULL. */
void kbo_prune(int32_t G, const int32_t *seg_off, const float *flops,
               const float *bytes, float peak_flops, float peak_bw,
               const float *incumbent, float *bound, uint8_t *alive)
{
    for (int32_t g = 0; g < G; ++g) {
        const float inc = incumbent[g];
        for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
            volatile float t_compute = flops[k] / peak_flops;
            volatile float t_memory = bytes[k] / peak_bw;
            float b = t_compute > t_memory ? t_compute : t_memory;
            if (bound) bound[k] = b;
            alive[k] = (uint8_t)(b < inc);
        }
    }
}

/* ---------------------------------------------------------------- cluster */

static double sqdist(const float *x, const float *c, int32_t D)
{
    double acc = 0.0;
    for (int32_t d = 0; d < D; ++d) {
        double diff = (double)x[d] - (double)c[d];
        acc += diff * diff;
    }
    return acc;
}

/* Nearest centroid of every candidate under squared L2 distance in fp64.
 * assign[k]  = lowest cluster index (local to the search) attaining the min;
 * mind2[k]   = that minimal squared distance;
 * flag[k]    = 1 if the runner-up is within 1e-6 (relative) of the winner, i.e.
 *              d2nd - d1st <= 1e-6 * max(d2nd, 1e-30); a search with one
 *              cluster never flags.  flag and mind2 may be NULL. */
void kbo_assign(int32_t G, int32_t D, const int32_t *seg_off,
                const int32_t *koff, const float *X, const float *cent,
                int32_t *assign, double *mind2, uint8_t *flag)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t K = koff[g + 1] - koff[g];
        const float *cg = cent + (size_t)koff[g] * D;
        for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
            const float *x = X + (size_t)k * D;
            double best = INFINITY, second = INFINITY;
            int32_t arg = -1;
            for (int32_t j = 0; j < K; ++j) {
                double dj = sqdist(x, cg + (size_t)j * D, D);
                if (dj < best) {
                    second = best;
                    best = dj;
                    arg = j;
                } else if (dj < second) {
                    second = dj;
                }
            }
            assign[k] = arg;
            if (mind2) mind2[k] = best;
            if (flag) {
                uint8_t f = 0;
                if (K > 1) {
                    double scale = second > KBO_TINY ? second : KBO_TINY;
                    f = (uint8_t)((second - best) <= KBO_NEAR_TIE_REL * scale);
                }
                flag[k] = f;
            }
        }
    }
}

/* Centroid update for a given assignment: the mean of each cluster's members,
 * summed in fp64 in candidate order and rounded once to fp32; an empty cluster
 * keeps its previous centroid. */
void kbo_update(int32_t G, int32_t D, const int32_t *seg_off,
                const int32_t *koff, const float *X, const float *cent_in,
                const int32_t *assign, float *cent_out, int32_t *counts)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t K = koff[g + 1] - koff[g];
        if (K <= 0) continue;
        double *sum = (double *)calloc((size_t)K * D, sizeof(double));
        int32_t *cnt = counts + koff[g];
        for (int32_t j = 0; j < K; ++j) cnt[j] = 0;
        for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
            const int32_t j = assign[k];
            const float *x = X + (size_t)k * D;
            for (int32_t d = 0; d < D; ++d) sum[(size_t)j * D + d] += (double)x[d];
            cnt[j] += 1;
        }
        for (int32_t j = 0; j < K; ++j) {
            const size_t row = ((size_t)koff[g] + j) * D;
            for (int32_t d = 0; d < D; ++d) {
                if (cnt[j] > 0)
                    cent_out[row + d] = (float)(sum[(size_t)j * D + d] / (double)cnt[j]);
                else
                    cent_out[row + d] = cent_in[row + d];
            }
        }
        free(sum);
    }
}

/* J_g = sum over the search's candidates of their minimal squared distance. */
void kbo_objective(int32_t G, const int32_t *seg_off, const double *mind2,
                   double *objective)
{
    for (int32_t g = 0; g < G; ++g) {
        double J = 0.0;
        for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) J += mind2[k];
        objective[g] = J;
    }
}

/* One Lloyd step from cent_in: assign, objective, update.  mind2 is scratch of
 * N doubles supplied by the caller; flag may be NULL. */
void kbo_cluster_step(int32_t G, int32_t D, const int32_t *seg_off,
                      const int32_t *koff, const float *X, const float *cent_in,
                      int32_t *assign, float *cent_out, int32_t *counts,
                      double *objective, double *mind2, uint8_t *flag)
{
    kbo_assign(G, D, seg_off, koff, X, cent_in, assign, mind2, flag);
    kbo_objective(G, seg_off, mind2, objective);
    kbo_update(G, D, seg_off, koff, X, cent_in, assign, cent_out, counts);
}

/* iters Lloyd steps.  Initial centroids: cent_init if given, else the first K_g
 * rows of each search.  Outputs are those of the last step (assign, counts and
 * objective refer to the centroids entering it; cent is its updated centroids).
 * iters == 0 only writes cent = initial centroids.  dirty[g] (may be NULL) is
 * set when any candidate of the search was a flagged near-tie in any step. */
void kbo_cluster(int32_t G, int32_t D, const int32_t *seg_off,
                 const int32_t *koff, const float *X, const float *cent_init,
                 int32_t iters, int32_t *assign, float *cent, int32_t *counts,
                 double *objective, uint8_t *dirty)
{
    const int64_t N = seg_off[G];
    const int64_t Ksum = koff[G];
    float *cur = (float *)malloc(sizeof(float) * (size_t)(Ksum > 0 ? Ksum : 1) * D);
    double *mind2 = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    uint8_t *flag = (uint8_t *)malloc((size_t)(N > 0 ? N : 1));
    for (int32_t g = 0; g < G; ++g) {
        const int32_t K = koff[g + 1] - koff[g];
        for (int32_t j = 0; j < K; ++j) {
            const float *src = cent_init
                ? cent_init + ((size_t)koff[g] + j) * D
                : X + ((size_t)seg_off[g] + j) * D;
            memcpy(cur + ((size_t)koff[g] + j) * D, src, sizeof(float) * D);
        }
        if (dirty) dirty[g] = 0;
    }
    for (int32_t it = 0; it < iters; ++it) {
        kbo_cluster_step(G, D, seg_off, koff, X, cur, assign, cent, counts,
                         objective, mind2, flag);
        memcpy(cur, cent, sizeof(float) * (size_t)Ksum * D);
        if (dirty)
            for (int32_t g = 0; g < G; ++g)
                for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k)
                    if (flag[k]) dirty[g] = 1;
    }
    if (iters == 0) memcpy(cent, cur, sizeof(float) * (size_t)Ksum * D);
    free(cur);
    free(mind2);
    free(flag);
}

/* -------------------------------------------------------------------- UCB */

/* Cluster-arm statistics, masked UCB index and arm selection for every search.
 *
 *   Ncs[i,s] = sum of visits[k,s] over alive members k of cluster i
 *   R[i,s]   = sum of rsum[k,s] over the same members
 *   Ntilde   = Ncs + prior_n ; Rtilde = R + prior_n*prior_mu ; mu = Rtilde/Ntilde
 *   a cluster is valid iff it has an alive member; with a strategy mask M
 *   ([Ksum,S], may be NULL: the paper's own form of Eq. 5) arm (i,s) is valid
 *   iff cluster i is and M[i,s] != 0
 *   ucb = mu + c*sqrt(ln t_g / Ntilde)  (valid, Ntilde > 0)
 *       = +inf                          (valid, Ntilde == 0: untried arm first)
 *       = -inf                          (not valid: masked)
 *   (I, S*) = lowest flat index i*S+s attaining the max over valid arms
 *   k*      = alive member of cluster I with the smallest bound, lowest k on ties
 *             (alive == NULL: every candidate alive; bound == NULL: lowest k)
 *   sel[g]  = (I, S*, k*) with k* a global candidate index, or (-1,-1,-1).
 *
 * near[g] (may be NULL) = 1 if the best score is finite and the largest score
 * that is not equal to it is finite and within 1e-6*max(|best|,1e-30) of it.
 * mu is written as NaN where Ntilde == 0.
 */
void kbo_ucb_select(int32_t G, int32_t S, const int32_t *seg_off,
                    const int32_t *koff, const int32_t *assign,
                    const uint8_t *alive, const float *bound,
                    const int32_t *visits, const float *rsum, const int64_t *t,
                    double c, double prior_n, double prior_mu, const uint8_t *M,
                    int64_t *Ncs, double *mu, double *ucb, int32_t *sel, uint8_t *near)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t K = koff[g + 1] - koff[g];
        const size_t base = (size_t)koff[g] * S;
        int32_t *nalive = (int32_t *)calloc((size_t)(K > 0 ? K : 1), sizeof(int32_t));
        double *R = (double *)calloc((size_t)(K > 0 ? K : 1) * S, sizeof(double));
        for (size_t a = 0; a < (size_t)K * S; ++a) Ncs[base + a] = 0;
        for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
            if (alive && !alive[k]) continue;
            const int32_t i = assign[k];
            nalive[i] += 1;
            for (int32_t s = 0; s < S; ++s) {
                Ncs[base + (size_t)i * S + s] += (int64_t)visits[(size_t)k * S + s];
                R[(size_t)i * S + s] += (double)rsum[(size_t)k * S + s];
            }
        }
        const double lnt = log((double)t[g]);
        double best = -INFINITY;
        int32_t best_flat = -1;
        for (int32_t i = 0; i < K; ++i) {
            for (int32_t s = 0; s < S; ++s) {
                const size_t a = (size_t)i * S + s;
                const double nt = (double)Ncs[base + a] + prior_n;
                const double rt = R[a] + prior_n * prior_mu;
                double m = nt > 0.0 ? rt / nt : NAN;
                double u;
                const int valid = nalive[i] > 0 && (!M || M[base + a]);
                if (!valid) u = -INFINITY;
                else if (nt > 0.0) u = m + c * sqrt(lnt / nt);
                else u = INFINITY;
                mu[base + a] = m;
                ucb[base + a] = u;
                if (valid && (best_flat < 0 || u > best)) {
                    best = u;
                    best_flat = (int32_t)a;
                }
            }
        }
        int32_t I = -1, Sstar = -1, kstar = -1;
        if (best_flat >= 0) {
            I = best_flat / S;
            Sstar = best_flat % S;
            float bmin = 0.0f;
            for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
                if ((alive && !alive[k]) || assign[k] != I) continue;
                if (kstar < 0 || (bound && bound[k] < bmin)) {
                    bmin = bound ? bound[k] : 0.0f;
                    kstar = k;
                }
            }
        }
        sel[3 * (size_t)g + 0] = I;
        sel[3 * (size_t)g + 1] = Sstar;
        sel[3 * (size_t)g + 2] = kstar;
        if (near) {
            uint8_t f = 0;
            if (best_flat >= 0 && isfinite(best)) {
                double runner = -INFINITY;
                for (int32_t i = 0; i < K; ++i) {
                    if (nalive[i] == 0) continue;
                    for (int32_t s = 0; s < S; ++s) {
                        if (M && !M[base + (size_t)i * S + s]) continue;
                        double u = ucb[base + (size_t)i * S + s];
                        if (u != best && u > runner) runner = u;
                    }
                }
                if (isfinite(runner)) {
                    double scale = fabs(best) > KBO_TINY ? fabs(best) : KBO_TINY;
                    f = (uint8_t)((best - runner) <= KBO_NEAR_TIE_REL * scale);
                }
            }
            near[g] = f;
        }
        free(nalive);
        free(R);
    }
}

/* --------------------------------------------------------------- sampling */

/* Philox4x32 with 10 rounds: the counter-based generator of Salmon, Moraes,
 * Dror and Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11), written
 * from its published definition: each round multiplies counter words 0 and 2 by
 * the two round constants, mixes the high halves with the other two words and
 * the key, and the key is advanced by the Weyl constants between rounds. */
void kbo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform variate of candidate k (global index) in draw number `draw` under
 * `seed`: counter = (k, 0, draw low, draw high), key = (seed low, seed high);
 * the first two output words give 52 random bits m and u = (m + 1/2) 2^-52,
 * which lies strictly inside (0, 1) and is exact in fp64. */
double kbo_uniform(uint64_t seed, uint64_t draw, int32_t k)
{
    const uint32_t ctr[4] = {(uint32_t)k, 0u, (uint32_t)draw, (uint32_t)(draw >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    kbo_philox4x32_10(ctr, key, out);
    const uint64_t m = ((uint64_t)out[0] << 20) | (uint64_t)(out[1] >> 12);
    return ((double)m + 0.5) * (1.0 / 4503599627370496.0);
}

/* Sampling of k_t inside the chosen cluster (Sec. 3.4, Alg. 1 "Sample k_t"):
 * P(k) proportional to exp(V(k)/tau) over the alive members of cluster I_t,
 * where V is the remaining headroom of candidate k.  With the roofline reading
 * of the bound the headroom is the fraction of the incumbent's runtime the
 * candidate could still gain, V(k) = 1 - bound[k]/incumbent[g]  (in (0, 1] for
 * an alive candidate; incumbent = +inf gives V = 1 for all, a uniform draw).
 *
 * The draw is made reproducible by the Gumbel-max identity: with independent
 * standard Gumbel variates g_k = -ln(-ln u_k), argmax_k (V(k)/tau + g_k) is
 * distributed exactly as the softmax above.  Lowest index on exact ties.
 *
 *   sel[g]  = (I, S*, .) from the selection step; I < 0 gives ksel[g] = -1
 *   ksel[g] = the sampled candidate, a global index
 *   near[g] = 1 if the runner-up key is within 1e-6*max(|best|,1e-30) of the
 *             best (the logarithms differ between libraries in the last bits)
 * alive may be NULL (every candidate alive). */
void kbo_sample(int32_t G, const int32_t *seg_off, const int32_t *assign,
                const uint8_t *alive, const float *bound, const float *incumbent,
                const int32_t *sel, uint64_t seed, uint64_t draw, double tau,
                int32_t *ksel, uint8_t *near)
{
#pragma omp parallel for schedule(dynamic, 16) if (G > 64)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t I = sel[3 * (size_t)g];
        double best = -INFINITY, runner = -INFINITY;
        int32_t arg = -1;
        if (I >= 0) {
            const double inc = (double)incumbent[g];
            for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
                if ((alive && !alive[k]) || assign[k] != I) continue;
                const double V = 1.0 - (double)bound[k] / inc;
                const double u = kbo_uniform(seed, draw, k);
                const double gumbel = -log(-log(u));
                const double key = V / tau + gumbel;
                if (arg < 0 || key > best) {
                    runner = best;
                    best = key;
                    arg = k;
                } else if (key > runner) {
                    runner = key;
                }
            }
        }
        ksel[g] = arg;
        if (near) {
            uint8_t f = 0;
            if (arg >= 0 && runner > -INFINITY) {
                double scale = fabs(best) > KBO_TINY ? fabs(best) : KBO_TINY;
                f = (uint8_t)((best - runner) <= KBO_NEAR_TIE_REL * scale);
            }
            near[g] = f;
        }
    }
}

/* ------------------------------------------------- cluster representatives */

/* The centroid kernel k_c^(i) of every cluster - the member whose feature vector
 * is nearest the centroid (Sec. 3.3 "Representative profiling"; Alg. 1 "Update
 * centroids k_c") - and the cluster's radius, the largest distance from the
 * centroid to a member.  The radius is the covering radius epsilon of the
 * approximation term of Theorem 1 (Appendix "Bounding Approximation Regret"),
 * and diam(C_i) <= 2 radius_i.
 *
 *   rep[j]    = global index of the member of cluster j with the smallest squared
 *               distance to cent[j] (fp64, direct differences), lowest index on
 *               ties; -1 for a cluster without members
 *   radius[j] = sqrt(largest such squared distance); 0 for an empty cluster
 *   dist2[k]  = squared distance of candidate k to its own centroid (may be NULL)
 */
void kbo_cluster_geometry(int32_t G, int32_t D, const int32_t *seg_off,
                          const int32_t *koff, const float *X, const float *cent,
                          const int32_t *assign, int32_t *rep, double *radius,
                          double *dist2)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t K = koff[g + 1] - koff[g];
        if (K <= 0) continue;
        double *dmin = (double *)malloc(sizeof(double) * (size_t)K);
        double *dmax = (double *)malloc(sizeof(double) * (size_t)K);
        int32_t *r = rep + koff[g];
        for (int32_t j = 0; j < K; ++j) {
            r[j] = -1;
            dmin[j] = 0.0;
            dmax[j] = 0.0;
        }
        for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
            const int32_t j = assign[k];
            const double d = sqdist(X + (size_t)k * D, cent + ((size_t)koff[g] + j) * D, D);
            if (dist2) dist2[k] = d;
            if (r[j] < 0 || d < dmin[j]) {
                dmin[j] = d;
                r[j] = k;
            }
            if (d > dmax[j]) dmax[j] = d;
        }
        for (int32_t j = 0; j < K; ++j) radius[koff[g] + j] = sqrt(dmax[j]);
        free(dmin);
        free(dmax);
    }
}

/* ----------------------------------------------------------- cluster diameters */

/* diam(C_i) = the largest distance between two members of cluster i, the
 * quantity in the approximation term L * max_i diam(C_i) of Theorem 1.  Plain
 * definition: every pair of members, squared L2 distance in fp64 from direct
 * differences, square root of the largest.  0 for clusters with fewer than two
 * members. */
void kbo_cluster_diameter(int32_t G, int32_t D, const int32_t *seg_off,
                          const int32_t *koff, const float *X, const int32_t *assign,
                          double *diam)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t K = koff[g + 1] - koff[g];
        for (int32_t j = 0; j < K; ++j) diam[koff[g] + j] = 0.0;
        for (int32_t a = seg_off[g]; a < seg_off[g + 1]; ++a) {
            const int32_t j = assign[a];
            double far = 0.0;
            for (int32_t b = a + 1; b < seg_off[g + 1]; ++b) {
                if (assign[b] != j) continue;
                const double d = sqdist(X + (size_t)a * D, X + (size_t)b * D, D);
                if (d > far) far = d;
            }
            far = sqrt(far);
            if (far > diam[koff[g] + j]) diam[koff[g] + j] = far;
        }
    }
}

/* ------------------------------------------------------ farthest-point seeding */

/* Initial centroids that spread over the frontier (an option beside "the first
 * K rows"): the first centroid is the search's first row, and every further one
 * is the candidate farthest from the centroids chosen so far,
 *     c_{j+1} = x_k  with  k = argmax_k min_{i <= j} ||x_k - c_i||^2 ,
 * lowest k on ties (squared L2 distances in fp64, direct differences).  This is
 * the greedy cover whose largest cluster radius is within a factor two of the
 * smallest possible one - the covering radius epsilon that the approximation
 * term of Theorem 1 (Appendix "Bounding Approximation Regret") is linear in.
 *
 *   cent[koff[g] + j, :] = the j-th chosen row of search g (an exact copy)
 *   pick[koff[g] + j]    = its global candidate index (may be NULL)
 * When all remaining candidates coincide with chosen centroids the farthest
 * distance is 0 and the lowest-index candidate is taken again. */
void kbo_seed_farthest(int32_t G, int32_t D, const int32_t *seg_off,
                       const int32_t *koff, const float *X, float *cent, int32_t *pick)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t n0 = seg_off[g], n = seg_off[g + 1] - seg_off[g];
        const int32_t K = koff[g + 1] - koff[g];
        if (n <= 0 || K <= 0) continue;
        double *mind = (double *)malloc(sizeof(double) * (size_t)n);
        for (int32_t k = 0; k < n; ++k) mind[k] = INFINITY;
        int32_t chosen = 0;                 /* local index of the newest centroid */
        for (int32_t j = 0; j < K; ++j) {
            float *c = cent + ((size_t)koff[g] + j) * D;
            memcpy(c, X + ((size_t)n0 + chosen) * D, sizeof(float) * D);
            if (pick) pick[koff[g] + j] = n0 + chosen;
            double far = -1.0;
            int32_t arg = 0;
            for (int32_t k = 0; k < n; ++k) {
                const double d = sqdist(X + ((size_t)n0 + k) * D, c, D);
                if (d < mind[k]) mind[k] = d;
                if (mind[k] > far) {
                    far = mind[k];
                    arg = k;
                }
            }
            chosen = arg;
        }
        free(mind);
    }
}

/* ------------------------------------------------- D^2-weighted seeding (++) */

double kbo_uniform(uint64_t seed, uint64_t draw, int32_t k);

/* Randomised initial centroids in the manner of k-means++ (the seeding behind
 * the scikit-learn default the paper runs, Sec. 3.6): the first centroid is a
 * uniformly drawn row of the search, every further one is drawn with
 * probability proportional to its squared distance to the nearest centroid
 * chosen so far,  P(k) = D_k^2 / sum D^2,  D_k^2 = min_i ||x_k - c_i||^2 (fp64,
 * direct differences).  Every draw is made reproducible the same way as the
 * draw of k_t: with independent Gumbel variates, argmax_k (ln D_k^2 - ln(-ln u_k))
 * is distributed exactly as P, and u_k is the variate of candidate k (global
 * index) in draw number draw0 + j under `seed`, j the position of the centroid
 * in its search.  A row at distance 0 has weight 0 (key -inf) and is never
 * drawn while a row at positive distance exists; lowest index on exact ties.
 *
 *   cent[koff[g] + j, :] = the j-th drawn row (an exact copy), pick = its index
 *   near[g] = 1 if, in any of the K_g draws, the runner-up key was within
 *             1e-6*max(|best|,1e-30) of the best (logarithms differ between
 *             libraries in the last bits; the later draws then depend on it) */
void kbo_seed_dsquared(int32_t G, int32_t D, const int32_t *seg_off, const int32_t *koff,
                       const float *X, uint64_t seed, uint64_t draw0, float *cent,
                       int32_t *pick, uint8_t *near)
{
#pragma omp parallel for schedule(dynamic, 1) if (G > 1)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t n0 = seg_off[g], n = seg_off[g + 1] - seg_off[g];
        const int32_t K = koff[g + 1] - koff[g];
        if (near) near[g] = 0;
        if (n <= 0 || K <= 0) continue;
        double *mind = (double *)malloc(sizeof(double) * (size_t)n);
        for (int32_t k = 0; k < n; ++k) mind[k] = INFINITY;
        for (int32_t j = 0; j < K; ++j) {
            /* draw with weights mind (all equal, i.e. uniform, for the first) */
            double best = -INFINITY, runner = -INFINITY;
            int32_t arg = -1;
            for (int32_t k = 0; k < n; ++k) {
                const double u = kbo_uniform(seed, draw0 + (uint64_t)j, n0 + k);
                const double gumbel = -log(-log(u));
                const double key = (j == 0 ? 0.0 : log(mind[k])) + gumbel;
                if (arg < 0 || key > best) {
                    runner = best;
                    best = key;
                    arg = k;
                } else if (key > runner) {
                    runner = key;
                }
            }
            if (near && runner > -INFINITY) {
                const double scale = fabs(best) > KBO_TINY ? fabs(best) : KBO_TINY;
                if ((best - runner) <= KBO_NEAR_TIE_REL * scale) near[g] = 1;
            }
            float *c = cent + ((size_t)koff[g] + j) * D;
            memcpy(c, X + ((size_t)n0 + arg) * D, sizeof(float) * D);
            if (pick) pick[koff[g] + j] = n0 + arg;
            for (int32_t k = 0; k < n; ++k) {
                const double d = sqdist(X + ((size_t)n0 + k) * D, c, D);
                if (d < mind[k]) mind[k] = d;
            }
        }
        free(mind);
    }
}

/* ------------------------------------------------- paper-form strategy mask */

/* The binary mask of Eq. 5 in the paper's own form: strategy s is valid for
 * cluster i iff the resource it targets is not saturated on the cluster's
 * representative,  M[i,s] = [ h(k_c^(i))[Target(s)] < theta_sat ].
 *
 *   h[N,R]      hardware signature of every candidate (throughput as a share of
 *               peak for R resources; the paper uses DRAM, L2 and SM)
 *   target[S]   the resource each strategy targets, in [0, R)
 *   rep[Ksum]   representative of each cluster (-1: empty cluster, nothing valid)
 *   M[Ksum,S]   out, 0/1
 *   nvalid[G]   out: number of valid cluster arms of the search, K |S_valid| in
 *               the estimation term of Theorem 1
 * The comparison is made on the fp32 values as they are (strict '<'). */
void kbo_strategy_mask(int32_t G, int32_t S, int32_t R, const int32_t *koff,
                       const float *h, const int32_t *target, const int32_t *rep,
                       float theta_sat, uint8_t *M, int32_t *nvalid)
{
    for (int32_t g = 0; g < G; ++g) {
        int32_t n = 0;
        for (int32_t i = koff[g]; i < koff[g + 1]; ++i) {
            for (int32_t s = 0; s < S; ++s) {
                uint8_t m = 0;
                if (rep[i] >= 0) m = (uint8_t)(h[(size_t)rep[i] * R + target[s]] < theta_sat);
                M[(size_t)i * S + s] = m;
                n += m;
            }
        }
        nvalid[g] = n;
    }
}

/* Draw of k_t with the paper's own potential (Sec. 3.4):
 * V_hw(k, S_t) = theta_sat - h(k)[Target(S_t)], P(k) proportional to
 * exp(V_hw/tau) over the members of cluster I_t (alive may be NULL), by the same
 * Gumbel-max construction and the same variates as kbo_sample. */
void kbo_sample_signature(int32_t G, int32_t R, const int32_t *seg_off,
                          const int32_t *assign, const uint8_t *alive, const float *h,
                          const int32_t *target, float theta_sat, const int32_t *sel,
                          uint64_t seed, uint64_t draw, double tau, int32_t *ksel,
                          uint8_t *near)
{
#pragma omp parallel for schedule(dynamic, 16) if (G > 64)
    for (int32_t g = 0; g < G; ++g) {
        const int32_t I = sel[3 * (size_t)g];
        double best = -INFINITY, runner = -INFINITY;
        int32_t arg = -1;
        if (I >= 0) {
            const int32_t col = target[sel[3 * (size_t)g + 1]];
            for (int32_t k = seg_off[g]; k < seg_off[g + 1]; ++k) {
                if ((alive && !alive[k]) || assign[k] != I) continue;
                const double V = (double)theta_sat - (double)h[(size_t)k * R + col];
                const double u = kbo_uniform(seed, draw, k);
                const double gumbel = -log(-log(u));
                const double key = V / tau + gumbel;
                if (arg < 0 || key > best) {
                    runner = best;
                    best = key;
                    arg = k;
                } else if (key > runner) {
                    runner = key;
                }
            }
        }
        ksel[g] = arg;
        if (near) {
            uint8_t f = 0;
            if (arg >= 0 && runner > -INFINITY) {
                double scale = fabs(best) > KBO_TINY ? fabs(best) : KBO_TINY;
                f = (uint8_t)((best - runner) <= KBO_NEAR_TIE_REL * scale);
            }
            near[g] = f;
        }
    }
}

/* ------------------------------------------------------- statistics update */

/* The update at the end of an iteration of Alg. 1 for every search at once.
 * For search g with the chosen arm (I, S*) = sel[g][0..1], the expanded
 * candidate k = ksel[g] and the observed reward r = reward[g] in [0,1]:
 *   t[g] <- t[g] + 1                                    (always)
 * and, only if the new kernel was verified (ok[g] != 0) and an arm was chosen:
 *   N_{I,S*}  <- N_{I,S*} + 1
 *   mu_{I,S*} <- mu_{I,S*} + (r - mu_{I,S*}) / (N_{I,S*} + prior_n)
 *   visits[k,S*] += 1 ; rsum[k,S*] += r                 (the per-candidate history
 *                    from which the cluster statistics are rebuilt after a
 *                    re-clustering)
 * mu is read as fp32, updated in fp64 and rounded once; rsum likewise. */
void kbo_update_stats(int32_t G, int32_t S, const int32_t *koff, const int32_t *sel,
                      const int32_t *ksel, const float *reward, const uint8_t *ok,
                      double prior_n, int32_t *visits, float *rsum, int32_t *Ncs,
                      float *mu, int64_t *t)
{
    for (int32_t g = 0; g < G; ++g) {
        t[g] += 1;
        const int32_t I = sel[3 * (size_t)g], s = sel[3 * (size_t)g + 1];
        const int32_t k = ksel[g];
        if (!ok[g] || I < 0 || s < 0 || k < 0) continue;
        const size_t arm = ((size_t)koff[g] + I) * S + s;
        Ncs[arm] += 1;
        const double n = (double)Ncs[arm] + prior_n;
        const double m = (double)mu[arm];
        mu[arm] = (float)(m + ((double)reward[g] - m) / n);
        visits[(size_t)k * S + s] += 1;
        rsum[(size_t)k * S + s] = (float)((double)rsum[(size_t)k * S + s] + (double)reward[g]);
    }
}

/* ------------------------------------------------------------------ round */

/* One scoring round: prune every candidate, cluster ALL candidates (pruned ones
 * included - the frontier is clustered first and masked afterwards, Alg. 1),
 * then statistics, UCB and selection over the alive members. */
void kbo_round(int32_t G, int32_t D, int32_t S, const int32_t *seg_off,
               const int32_t *koff, const float *X, const float *flops,
               const float *bytes, const float *incumbent,
               const int32_t *visits, const float *rsum, const int64_t *t,
               float peak_flops, float peak_bw, double c, double prior_n,
               double prior_mu, int32_t iters, float *bound, uint8_t *alive,
               int32_t *assign, float *cent, int32_t *counts, double *objective,
               int64_t *Ncs, double *mu, double *ucb, int32_t *sel,
               uint8_t *dirty, uint8_t *near)
{
    kbo_prune(G, seg_off, flops, bytes, peak_flops, peak_bw, incumbent, bound, alive);
    kbo_cluster(G, D, seg_off, koff, X, NULL, iters, assign, cent, counts,
                objective, dirty);
    kbo_ucb_select(G, S, seg_off, koff, assign, alive, bound, visits, rsum, t, c,
                   prior_n, prior_mu, NULL, Ncs, mu, ucb, sel, near);
}

int32_t kbo_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
