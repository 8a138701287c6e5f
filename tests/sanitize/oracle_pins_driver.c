/* Runs the oracle's closed-form pins inside one executable built with
 * -fsanitize=address,undefined, so that an out-of-bounds access, a leak, a signed overflow or a
 * misaligned access in oracle/ws_oracle.c ends the run with a report.  Values: the two-point and
 * three-point densities (Sec. 3.3 density ingredient, closed forms), the exact-tie and hybrid hand
 * examples of the greedy choice, and the k = 1 / Q = 0 special cases of the attention. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void wso_density(const double *, int, int, double, double *);
void wso_density_rows(const double *, int, int, double, const int32_t *, int, double *);
void wso_inverse_density(const double *, int, double *);
int wso_select(const double *, const double *, int, int, int, double, int32_t *, double *, double *);
int wso_select_verify(const double *, const double *, int, int, int, double, const int32_t *, int32_t *, double *);
void wso_gather(const void *, const void *, int, const int32_t *, int, void *, void *);
int wso_attend(const double *, const double *, const double *, int, int, int, int, int, double, double *);
int wso_attention_mass(const double *, const double *, int, int, int, int, double, double *);
void wso_mass_to_density(const double *, int, double *);
void wso_gate(const double *, const double *, int, int, double, double *, int32_t *);
int wso_rope(const double *, const int32_t *, int, int, double, double *);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)
static int close_to(double a, double b, double rel) { return fabs(a - b) <= rel * fabs(b) + 1e-300; }

int main(void)
{
    /* two points at distance 5, sigma^2 = 12.5: rho = (1 + e^-1) / 2 */
    {
        double K[4] = {0, 0, 3, 4}, rho[2];
        wso_density(K, 2, 2, sqrt(12.5), rho);
        CHECK(close_to(rho[0], 0.6839397205857212, 1e-15) && rho[0] == rho[1]);
    }
    /* 0, 1, 3 on a line, sigma^2 = 1/2 */
    {
        double K[3] = {0, 1, 3}, rho[3], u[3], rr[2];
        int32_t rows[2] = {2, 0};
        wso_density(K, 3, 1, sqrt(0.5), rho);
        CHECK(close_to(rho[0], (1 + exp(-1.0) + exp(-9.0)) / 3, 1e-14));
        CHECK(close_to(rho[1], (1 + exp(-1.0) + exp(-4.0)) / 3, 1e-14));
        CHECK(close_to(rho[2], (1 + exp(-9.0) + exp(-4.0)) / 3, 1e-14));
        wso_density_rows(K, 3, 1, sqrt(0.5), rows, 2, rr);
        CHECK(rr[0] == rho[2] && rr[1] == rho[0]);
        wso_inverse_density(rho, 3, u);
        CHECK(u[2] == 1.0 && close_to(u[0], 0.744471, 1e-5) && close_to(u[1], 0.734701, 1e-5));
        int32_t idx[3], pick[3];
        double sc[3], gap[3], def[3];
        CHECK(wso_select(K, rho, 3, 1, 3, 0.5, idx, sc, gap) == 0);
        CHECK(idx[0] == 2 && idx[1] == 0 && idx[2] == 1 && close_to(sc[1], 0.8722357186487468, 1e-12));
        CHECK(wso_select_verify(K, rho, 3, 1, 3, 0.5, idx, pick, def) == 0);
        int32_t other[3] = {2, 1, 0};
        CHECK(wso_select_verify(K, rho, 3, 1, 3, 0.5, other, pick, def) == 1 && pick[1] == 0);
        CHECK(close_to(def[1], (0.8722357186487468 - 0.700684) / 0.8722357186487468, 1e-5));
        int32_t rep[3] = {2, 2, 0};
        CHECK(wso_select_verify(K, rho, 3, 1, 3, 0.5, rep, pick, def) == -2);
        CHECK(wso_select(K, rho, 3, 1, 4, 0.5, idx, sc, gap) == -1);
    }
    /* farthest-point traversal with an exact tie: 0,3,7,10,5 -> 0,3,4,1,2 */
    {
        double K[5] = {0, 3, 7, 10, 5}, rho[5] = {1, 1, 1, 1, 1}, gap[5];
        int32_t idx[5];
        CHECK(wso_select(K, rho, 5, 1, 5, 1.0, idx, NULL, gap) == 0);
        CHECK(idx[0] == 0 && idx[1] == 3 && idx[2] == 4 && idx[3] == 1 && idx[4] == 2 && gap[3] == 0.0);
    }
    /* gather and attention special cases on a cloud large enough for the parallel loops */
    {
        const int L = 97, d = 6, k = 13, N = 5, Hq = 4, Hkv = 2;
        double *K = malloc(sizeof(double) * L * d), *V = malloc(sizeof(double) * L * d);
        double *rho = malloc(sizeof(double) * L);
        srand(3);
        for (int i = 0; i < L * d; ++i) { K[i] = rand() / (double)RAND_MAX - 0.5; V[i] = rand() / (double)RAND_MAX; }
        wso_density(K, L, d, 0.7, rho);
        for (int i = 0; i < L; ++i) CHECK(rho[i] >= 1.0 / L && rho[i] <= 1.0);
        int32_t idx[13];
        CHECK(wso_select(K, rho, L, d, k, 0.5, idx, NULL, NULL) == 0);
        double *Ks = malloc(sizeof(double) * Hkv * k * d), *Vs = malloc(sizeof(double) * Hkv * k * d);
        for (int h = 0; h < Hkv; ++h)
            wso_gather(K, V, d * (int)sizeof(double), idx, k, Ks + h * k * d, Vs + h * k * d);
        CHECK(memcmp(Ks + 3 * d, K + (size_t)idx[3] * d, sizeof(double) * d) == 0);
        double *Q = calloc((size_t)N * Hq * d, sizeof(double)), *O = malloc(sizeof(double) * N * Hq * d);
        CHECK(wso_attend(Q, Ks, Vs, N, Hq, Hkv, k, d, 1.0 / sqrt(d), O) == 0);      /* Q = 0: mean of the rows */
        double mean0 = 0;
        for (int t = 0; t < k; ++t) mean0 += Vs[t * d] / k;
        CHECK(close_to(O[0], mean0, 1e-13));
        for (int i = 0; i < N * Hq * d; ++i) Q[i] = rand() / (double)RAND_MAX - 0.5;
        CHECK(wso_attend(Q, Ks, Vs, N, Hq, Hkv, 1, d, 1.0, O) == 0);                /* k = 1: the row itself */
        CHECK(O[0] == Vs[0] && O[(N * Hq - 1) * d + d - 1] == Vs[d + d - 1]);   /* last query head reads KV head 1 of a [Hkv,1,d] buffer */
        CHECK(wso_attend(Q, Ks, Vs, N, 3, Hkv, k, d, 1.0, O) == -1);
        double *A = malloc(sizeof(double) * L), sum = 0;
        double *K2 = malloc(sizeof(double) * Hkv * L * d);
        for (int i = 0; i < Hkv * L * d; ++i) K2[i] = rand() / (double)RAND_MAX - 0.5;
        CHECK(wso_attention_mass(K2, Q, Hkv, Hq, L, d, 0.4, A) == 0);
        for (int i = 0; i < L; ++i) sum += A[i];
        CHECK(close_to(sum, Hq, 1e-12));
        wso_mass_to_density(A, L, rho);
        CHECK(close_to(rho[5] * A[5], 1.0, 1e-15));
        double score[5];
        int32_t acc[5];
        wso_gate(K, K, 5, d, 0.5, score, acc);                                       /* row 0 against itself */
        CHECK(close_to(score[0], 1.0, 1e-15) && acc[0] == 1);
        int32_t pos[4] = {0, 7, 100000, 2000000000};
        double Y[4 * 6];
        CHECK(wso_rope(K, pos, 4, d, 1e6, Y) == 0);
        CHECK(memcmp(Y, K, sizeof(double) * d) == 0);                                /* position 0: no rotation */
        free(K); free(V); free(rho); free(Ks); free(Vs); free(Q); free(O); free(A); free(K2);
    }
    printf(failures ? "%d check(s) failed\n" : "all checks passed\n", failures);
    return failures ? 1 : 0;
}
