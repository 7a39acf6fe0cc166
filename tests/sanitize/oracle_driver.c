/* Runs the CPU oracle (both precisions) on small shapes under AddressSanitizer and
 * UndefinedBehaviorSanitizer: ragged regions, one token per region, k = S^2, forced routing, every
 * optional output.  Exit status 0 means no report.  Test infrastructure. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_bra_forward_f32(int, int, int, int, int, int, int, double, const float *, const float *, const float *,
                           const float *, const int32_t *, float *, int32_t *, float *, float *, float *, float *,
                           int64_t *, int);
int oracle_bra_forward_f64(int, int, int, int, int, int, int, double, const double *, const double *, const double *,
                           const double *, const int32_t *, double *, int32_t *, double *, double *, double *, double *,
                           int64_t *, int);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state % 20001) / 10000.0 - 1.0;
}

#define RUN(REAL, FN)                                                                                          \
    static int run_##FN(int B, int H, int W, int C, int heads, int S, int k, int forced, int threads)          \
    {                                                                                                          \
        const int R = S * S, n = (H / S) * (W / S);                                                            \
        const size_t tok = (size_t)B * H * W * C;                                                              \
        REAL *X = malloc(sizeof(REAL) * tok), *Wqkv = malloc(sizeof(REAL) * 3 * C * C);                        \
        REAL *Wo = malloc(sizeof(REAL) * C * C), *Wl = malloc(sizeof(REAL) * C * 25);                          \
        REAL *Y = malloc(sizeof(REAL) * tok), *Ar = malloc(sizeof(REAL) * (size_t)B * R * R);                  \
        REAL *P = malloc(sizeof(REAL) * (size_t)B * heads * R * n * k * n);                                    \
        REAL *Oa = malloc(sizeof(REAL) * tok), *Lc = malloc(sizeof(REAL) * tok);                               \
        int32_t *Ir = malloc(sizeof(int32_t) * (size_t)B * R * k), *Iin = malloc(sizeof(int32_t) * (size_t)B * R * k); \
        int64_t macs[3];                                                                                       \
        for (size_t e = 0; e < tok; ++e) X[e] = (REAL)rnd();                                                   \
        for (int e = 0; e < 3 * C * C; ++e) Wqkv[e] = (REAL)(rnd() / 4);                                       \
        for (int e = 0; e < C * C; ++e) Wo[e] = (REAL)(rnd() / 4);                                             \
        for (int e = 0; e < C * 25; ++e) Wl[e] = (REAL)(rnd() / 5);                                            \
        for (int e = 0; e < B * R * k; ++e) Iin[e] = (e * 7 + e / k) % R;                                      \
        const int rc = FN(B, H, W, C, heads, S, k, 0.25, X, Wqkv, Wo, Wl, forced ? Iin : NULL, Y, Ir, Ar, P, Oa, Lc, \
                          macs, threads);                                                                      \
        double sum = 0;                                                                                        \
        for (size_t e = 0; e < tok; ++e) sum += (double)Y[e];                                                  \
        printf("%s B%d %dx%dx%d h%d S%d k%d forced%d rc=%d sum=%.6g\n", #FN, B, H, W, C, heads, S, k, forced, rc, sum); \
        free(X); free(Wqkv); free(Wo); free(Wl); free(Y); free(Ar); free(P); free(Oa); free(Lc); free(Ir); free(Iin); \
        return rc;                                                                                             \
    }
RUN(float, oracle_bra_forward_f32)
RUN(double, oracle_bra_forward_f64)

int main(void)
{
    int bad = 0;
    bad |= run_oracle_bra_forward_f32(2, 6, 9, 8, 2, 3, 2, 0, 1);
    bad |= run_oracle_bra_forward_f64(1, 7, 7, 6, 3, 7, 49, 0, 1);
    bad |= run_oracle_bra_forward_f64(3, 8, 4, 4, 1, 2, 3, 1, 2);
    bad |= run_oracle_bra_forward_f32(1, 5, 5, 2, 1, 1, 1, 0, 1);
    bad |= run_oracle_bra_forward_f32(1, 8, 8, 4, 2, 4, 16, 1, 2);
    /* invalid shapes are refused before anything is touched */
    if (oracle_bra_forward_f32(1, 7, 7, 4, 2, 3, 1, 1.0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL,
                               NULL, 1) != -1)
        bad = 1;
    return bad ? 1 : 0;
}
