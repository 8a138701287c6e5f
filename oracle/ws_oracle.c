/*
 * ws_oracle.c -- plain CPU oracle for the Topological Synapse hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test suite, the
 * smoke check and the benchmark's cpu_baseline leg may build, link or call it.
 * It shares no code, header, table or helper with the HIP library and is kept
 * deliberately slow and literal: float64 everywhere, one head at a time,
 * distances by direct coordinate differences, no blocking, no fusion, no
 * re-association beyond the loop order written here.  OpenMP is applied only to
 * outer loops whose iterations are independent; every reduction that decides a
 * result (sums, max, argmax) runs serially in index order.
 *
 * What the paper fixes (Warp-Cortex, Sec. 3.3 "The Topological Synapse" and the
 * first paragraph of Sec. 2):
 *   - the cached keys of the context are a point cloud in latent space;
 *   - landmarks are chosen by a hybrid score that balances geometric coverage
 *     (Hausdorff-style distance of the cloud to the chosen set) against an
 *     inverse kernel density;
 *   - k << L landmarks (about 2 % of L) go into a shared buffer, the synapse;
 *   - side agents attend over those k rows with the usual 1/sqrt(d_k) scale.
 * The paper gives no formula for the score, no kernel, no bandwidth and no
 * normalisation.  The readings below are therefore fixed HERE, in writing:
 *
 *   R1  density: Gaussian kernel density over the keys of one head,
 *         rho_i = (1/L) * sum_{j=0}^{L-1} exp(-||k_i - k_j||^2 / (2 sigma^2)),
 *       self term j = i included, no (2 pi sigma^2)^(-d/2) constant
 *       (so 1/L <= rho_i <= 1).  sigma > 0 is an argument, one per head.
 *   R2  inverse density, scaled to (0,1]:  u_i = rho_min / rho_i.
 *   R3  hybrid score: convex mix  score_i = alpha * c_i + (1-alpha) * u_i,
 *       alpha = 1 -> coverage only, alpha = 0 -> density only.
 *   R4  coverage term: c_i = D_i / D_max with D_i the Euclidean (not squared)
 *       distance from k_i to the nearest landmark chosen so far and D_max the
 *       CURRENT maximum of D over the not-yet-chosen points, recomputed every
 *       step; if D_max == 0 then c_i = 0 for every i.
 *   R5  selection is greedy, one landmark per step, k steps; a chosen point is
 *       never chosen again; ties go to the lowest index.
 *   R6  first landmark: with no landmark chosen the coverage term is the same
 *       (1) for every point, so for alpha < 1 the first pick is argmax u
 *       (the lowest-density point) and for alpha == 1 it is index 0.
 *   R7  selection is per KV head; only keys form the cloud; values are only
 *       gathered; the synapse holds rows in pick order.
 *   R8  attention: z_t = (q . K_S[t]) * scale, softmax over the k landmarks,
 *       no mask, O = sum_t p_t V_S[t]; query head q reads KV head q / (Hq/Hkv).
 *
 * Steps next to the hot path (built after it), each with its own reading:
 *
 *   R9  attention mass (Sec. 3.3, "Attention Score Summation"): the printed
 *       formula sums a softmax over the heads of one layer but names no token
 *       axis.  Reading: per query head q of the layer, softmax over the L cached
 *       tokens of z_{q,i} = scale * (Q_q . K_{kv(q),i}), kv(q) = q / (Hq/Hkv);
 *       A_i = sum over the layer's query heads of that softmax.  sum_i A_i = Hq.
 *   R10 the same passage calls A the INVERSE density estimator: the array handed
 *       to the selection in place of rho is 1 / max(A_i, 1e-30), so that
 *       u_i = A_i / A_max.
 *   R11 validation gate (Sec. 3.5 and its equation): cosine similarity of each
 *       side thought's hidden state with the main agent's; a thought passes when
 *       score >= theta (the text rejects score < theta); a zero vector scores 0.
 *   R12 referential injection (Sec. 3.6): the appended key rows are rotated by
 *       RoPE at a caller-given virtual position p before they join the cache,
 *       values join unchanged.  Convention (the paper's model family): pairs
 *       (c, c + d/2), angle p * base^(-2c/d), c < d/2:
 *         y_c = x_c cos - x_{c+d/2} sin,   y_{c+d/2} = x_{c+d/2} cos + x_c sin.
 *   R13 refresh while the main agent decodes (Sec. 4, the listing's main-stream
 *       loop): the density of the grown context is R1 on the grown cloud; an
 *       incremental update must reproduce it, so its oracle is wso_density.
 *
 * Pins (see tests/test_oracle_pins.py): two-point and three-point closed forms
 * of the density, scipy logsumexp/cdist, per-step exhaustive re-evaluation of
 * the score from its definition on tiny clouds, Gonzalez farthest-point
 * traversal and the 2-approximation bound at alpha = 1, stable argsort of rho
 * at alpha = 0, hand-worked tie and hybrid examples, k = L dense softmax
 * attention, and a library scaled-dot-product attention in f64.  The chain as
 * a whole has no published vector to compare with: beyond those pins, parity
 * of the whole chain is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define WSO_INF (1.0 / 0.0)

/* squared Euclidean distance by direct differences (R1, R4) */
static double sqdist(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) {
        double t = a[c] - b[c];
        s += t * t;
    }
    return s;
}

/* R1.  K is [L,d] row-major.  rho is [L]. */
void wso_density(const double *K, int L, int d, double sigma, double *rho)
{
    const double inv = 1.0 / (2.0 * sigma * sigma);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < L; ++i) {
        double s = 0.0;
        for (int j = 0; j < L; ++j)
            s += exp(-sqdist(K + (size_t)i * d, K + (size_t)j * d, d) * inv);
        rho[i] = s / (double)L;
    }
}

/* R1 for a handful of rows only: rho_rows[r] = rho_{rows[r]}.  Same arithmetic
 * as wso_density; lets a test check single rows of a cloud that is too large
 * to sweep completely. */
void wso_density_rows(const double *K, int L, int d, double sigma,
                      const int32_t *rows, int nrows, double *rho_rows)
{
    const double inv = 1.0 / (2.0 * sigma * sigma);
#pragma omp parallel for schedule(static)
    for (int r = 0; r < nrows; ++r) {
        const double *ki = K + (size_t)rows[r] * d;
        double s = 0.0;
        for (int j = 0; j < L; ++j)
            s += exp(-sqdist(ki, K + (size_t)j * d, d) * inv);
        rho_rows[r] = s / (double)L;
    }
}

/* R2 */
void wso_inverse_density(const double *rho, int L, double *u)
{
    double rmin = rho[0];
    for (int i = 1; i < L; ++i)
        if (rho[i] < rmin) rmin = rho[i];
    for (int i = 0; i < L; ++i) u[i] = rmin / rho[i];
}

/* One greedy step (R3-R6) on the state (D, chosen, u) with `nsel` landmarks
 * already chosen.  Writes the best and second-best score among the points not
 * yet chosen and returns the argmax (lowest index on ties).  If `probe` >= 0
 * the score of that point is written to *probe_score. */
static int greedy_step(const double *D, const unsigned char *chosen, const double *u,
                       int L, int nsel, double alpha,
                       double *top1, double *top2, int probe, double *probe_score)
{
    double dmax = 0.0;
    if (nsel > 0)
        for (int i = 0; i < L; ++i)
            if (!chosen[i] && D[i] > dmax) dmax = D[i];

    int best = -1;
    double b1 = -WSO_INF, b2 = -WSO_INF;
    if (nsel == 0 && alpha == 1.0) {
        /* R6: every score equals alpha; lowest index wins.  No runner-up gap. */
        best = 0;
        b1 = alpha;
        b2 = -WSO_INF;
        if (probe >= 0) *probe_score = alpha;
    } else {
        for (int i = 0; i < L; ++i) {
            if (chosen[i]) continue;
            double c;
            if (nsel == 0) c = 1.0;
            else if (dmax == 0.0) c = 0.0;
            else c = D[i] / dmax;
            double s = alpha * c + (1.0 - alpha) * u[i];
            if (i == probe) *probe_score = s;
            if (s > b1) { b2 = b1; b1 = s; best = i; }
            else if (s > b2) b2 = s;
        }
    }
    *top1 = b1;
    *top2 = b2;
    return best;
}

static void absorb_landmark(const double *K, int L, int d, int s, double *D,
                            unsigned char *chosen)
{
    chosen[s] = 1;
    const double *ks = K + (size_t)s * d;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < L; ++i) {
        double dist = sqrt(sqdist(K + (size_t)i * d, ks, d));
        if (dist < D[i]) D[i] = dist;
    }
}

static double rel_gap(double top1, double top2)
{
    if (top2 == -WSO_INF) return WSO_INF;
    if (top1 == 0.0) return (top1 == top2) ? 0.0 : WSO_INF;
    return (top1 - top2) / fabs(top1);
}

/* R3-R6.  idx[k] landmark indices in pick order; score[k] winning score per
 * step; gap[k] relative distance (top1 - top2)/|top1| between the two best
 * scores of the step (+inf when there is no runner-up).  score and gap may be
 * NULL.  Returns 0, or -1 on bad sizes / allocation failure. */
int wso_select(const double *K, const double *rho, int L, int d, int k, double alpha,
               int32_t *idx, double *score, double *gap)
{
    if (L < 1 || k < 1 || k > L || d < 1) return -1;
    double *u = (double *)malloc(sizeof(double) * (size_t)L);
    double *D = (double *)malloc(sizeof(double) * (size_t)L);
    unsigned char *chosen = (unsigned char *)calloc((size_t)L, 1);
    if (!u || !D || !chosen) { free(u); free(D); free(chosen); return -1; }
    wso_inverse_density(rho, L, u);
    for (int i = 0; i < L; ++i) D[i] = WSO_INF;

    for (int t = 0; t < k; ++t) {
        double t1, t2;
        int s = greedy_step(D, chosen, u, L, t, alpha, &t1, &t2, -1, NULL);
        idx[t] = s;
        if (score) score[t] = t1;
        if (gap) gap[t] = rel_gap(t1, t2);
        absorb_landmark(K, L, d, s, D, chosen);
    }
    free(u); free(D); free(chosen);
    return 0;
}

/* Verify mode.  Replays the greedy rule along the CANDIDATE's own prefix: at
 * step t the state holds cand[0..t), the oracle's own pick under that state is
 * written to oracle_pick[t], and deficit[t] = (top1 - score(cand[t]))/|top1|
 * (0 when cand[t] is the strict argmax with the lowest-index tie-break).
 * Returns the number of steps where cand[t] != oracle_pick[t]; -1 on bad sizes;
 * -2 if the candidate repeats an index or holds one out of range. */
int wso_select_verify(const double *K, const double *rho, int L, int d, int k, double alpha,
                      const int32_t *cand, int32_t *oracle_pick, double *deficit)
{
    if (L < 1 || k < 1 || k > L || d < 1) return -1;
    double *u = (double *)malloc(sizeof(double) * (size_t)L);
    double *D = (double *)malloc(sizeof(double) * (size_t)L);
    unsigned char *chosen = (unsigned char *)calloc((size_t)L, 1);
    if (!u || !D || !chosen) { free(u); free(D); free(chosen); return -1; }
    wso_inverse_density(rho, L, u);
    for (int i = 0; i < L; ++i) D[i] = WSO_INF;

    int forks = 0;
    for (int t = 0; t < k; ++t) {
        int c = cand[t];
        if (c < 0 || c >= L || chosen[c]) { forks = -2; break; }
        double t1, t2, sc = 0.0;
        int s = greedy_step(D, chosen, u, L, t, alpha, &t1, &t2, c, &sc);
        oracle_pick[t] = s;
        if (s == c) {
            deficit[t] = 0.0;
        } else {
            ++forks;
            deficit[t] = (t1 == 0.0) ? ((sc == t1) ? 0.0 : WSO_INF) : (t1 - sc) / fabs(t1);
        }
        absorb_landmark(K, L, d, c, D, chosen);
    }
    free(u); free(D); free(chosen);
    return forks;
}

/* R7: bit copy of the chosen rows.  `row_bytes` = d * element size. */
void wso_gather(const void *K, const void *V, int row_bytes, const int32_t *idx, int k,
                void *Ks, void *Vs)
{
    for (int t = 0; t < k; ++t) {
        memcpy((char *)Ks + (size_t)t * row_bytes, (const char *)K + (size_t)idx[t] * row_bytes, row_bytes);
        memcpy((char *)Vs + (size_t)t * row_bytes, (const char *)V + (size_t)idx[t] * row_bytes, row_bytes);
    }
}

/* R8.  Q [N,Hq,d], Ks,Vs [Hkv,k,d], O [N,Hq,d], all row-major f64. */
int wso_attend(const double *Q, const double *Ks, const double *Vs,
               int N, int Hq, int Hkv, int k, int d, double scale, double *O)
{
    if (N < 1 || Hq < 1 || Hkv < 1 || k < 1 || d < 1 || Hq % Hkv != 0) return -1;
    const int g = Hq / Hkv;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int nq = 0; nq < N * Hq; ++nq) {
        const int q = nq % Hq;
        const int h = q / g;
        const double *qv = Q + (size_t)nq * d;
        const double *Kh = Ks + (size_t)h * k * d;
        const double *Vh = Vs + (size_t)h * k * d;
        double *z = (double *)malloc(sizeof(double) * (size_t)k);
        if (!z) { fail = 1; continue; }
        double zmax = -WSO_INF;
        for (int t = 0; t < k; ++t) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += qv[c] * Kh[(size_t)t * d + c];
            z[t] = s * scale;
            if (z[t] > zmax) zmax = z[t];
        }
        double den = 0.0;
        for (int t = 0; t < k; ++t) { z[t] = exp(z[t] - zmax); den += z[t]; }
        double *o = O + (size_t)nq * d;
        for (int c = 0; c < d; ++c) {
            double s = 0.0;
            for (int t = 0; t < k; ++t) s += (z[t] / den) * Vh[(size_t)t * d + c];
            o[c] = s;
        }
        free(z);
    }
    return fail ? -1 : 0;
}

/* R9.  K [Hkv,L,d], Q [Hq,d] of ONE layer -> A [L].  Serial over heads so the sum order is fixed. */
int wso_attention_mass(const double *K, const double *Q, int Hkv, int Hq, int L, int d, double scale, double *A)
{
    if (Hkv < 1 || Hq < 1 || L < 1 || d < 1 || Hq % Hkv != 0) return -1;
    const int g = Hq / Hkv;
    double *z = (double *)malloc(sizeof(double) * (size_t)L);
    if (!z) return -1;
    for (int i = 0; i < L; ++i) A[i] = 0.0;
    for (int q = 0; q < Hq; ++q) {
        const double *Kh = K + (size_t)(q / g) * L * d;
        const double *qv = Q + (size_t)q * d;
        double zmax = -WSO_INF;
        for (int i = 0; i < L; ++i) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += qv[c] * Kh[(size_t)i * d + c];
            z[i] = s * scale;
            if (z[i] > zmax) zmax = z[i];
        }
        double den = 0.0;
        for (int i = 0; i < L; ++i) { z[i] = exp(z[i] - zmax); den += z[i]; }
        for (int i = 0; i < L; ++i) A[i] += z[i] / den;
    }
    free(z);
    return 0;
}

/* R10.  The array that replaces rho in the selection. */
void wso_mass_to_density(const double *A, int L, double *rho)
{
    for (int i = 0; i < L; ++i) rho[i] = 1.0 / (A[i] > 1e-30 ? A[i] : 1e-30);
}

/* R11.  hmain [dm], T [N,dm] -> score [N], accept [N] (1 = passes). */
void wso_gate(const double *hmain, const double *T, int N, int dm, double theta, double *score, int32_t *accept)
{
    double nh = 0.0;
    for (int c = 0; c < dm; ++c) nh += hmain[c] * hmain[c];
    nh = sqrt(nh);
    for (int n = 0; n < N; ++n) {
        const double *t = T + (size_t)n * dm;
        double dot = 0.0, nt = 0.0;
        for (int c = 0; c < dm; ++c) { dot += hmain[c] * t[c]; nt += t[c] * t[c]; }
        nt = sqrt(nt);
        score[n] = (nh > 0.0 && nt > 0.0) ? dot / (nh * nt) : 0.0;
        accept[n] = score[n] >= theta ? 1 : 0;
    }
}

/* R12.  X [m,d] rows, pos [m] virtual positions -> Y [m,d] rotated rows. */
int wso_rope(const double *X, const int32_t *pos, int m, int d, double base, double *Y)
{
    if (m < 0 || d < 2 || (d & 1) || !(base > 0.0)) return -1;
    const int half = d / 2;
    for (int r = 0; r < m; ++r)
        for (int c = 0; c < half; ++c) {
            const double ang = (double)pos[r] * pow(base, -2.0 * (double)c / (double)d);
            const double cs = cos(ang), sn = sin(ang);
            const double x0 = X[(size_t)r * d + c], x1 = X[(size_t)r * d + c + half];
            Y[(size_t)r * d + c] = x0 * cs - x1 * sn;
            Y[(size_t)r * d + c + half] = x1 * cs + x0 * sn;
        }
    return 0;
}

int wso_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
