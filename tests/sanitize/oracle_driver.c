/* Calls every entry point of oracle/attn_oracle.c on small seeded inputs; built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py.  Prints one checksum. */
#include <stdio.h>
#include <stdlib.h>

void oracle_attn_fwd(int, int, int, int, double, int, int, int, const unsigned char *, const double *,
                     const double *, const double *, double *, double *);
void oracle_attn_bwd(int, int, int, int, double, int, int, int, const unsigned char *, const double *,
                     const double *, const double *, const double *, const double *, const double *,
                     double *, double *, double *);
void oracle_attn_bwd_head(int, int, double, int, int, int, const unsigned char *, const double *,
                          const double *, const double *, const double *, const double *, const double *,
                          double *, double *, double *, double *, double *, double *);
void oracle_attn_bwd_sampled(int, int, double, int, int, int, const unsigned char *, const double *,
                             const double *, const double *, const double *, const double *,
                             const double *, int, const int *, double *, int, const int *, double *,
                             double *);
void oracle_wgrad(int, int, const double *, const double *, const double *, const double *,
                  const double *, const double *, double *, double *, double *, double *);
void oracle_small_cache_wgrad(int, int, int, const double *, const double *, const double *,
                              const double *, const double *, const double *, double *, long long *);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state % 2000001ULL) / 1000000.0 - 1.0;
}
static double *vec(size_t n)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = 0.7 * rnd();
    return p;
}

int main(void)
{
    double sum = 0.0;
    const int shapes[4][4] = {{1, 1, 1, 1}, {2, 3, 7, 5}, {1, 2, 13, 4}, {1, 1, 0, 3}};
    for (int s = 0; s < 4; ++s)
        for (int causal = 0; causal < 2; ++causal)
            for (int masked = 0; masked < 2; ++masked) {
                const int b = shapes[s][0], h = shapes[s][1], n = shapes[s][2], d = shapes[s][3];
                const int block = 3, nblk = (n + block - 1) / block;
                unsigned char *keep = (unsigned char *)malloc((size_t)nblk * nblk + 1);
                for (int i = 0; i < nblk * nblk; ++i) keep[i] = (i % (nblk + 1) == 0) || (i % 3 == 1);
                const unsigned char *kp = masked ? keep : NULL;
                const size_t t = (size_t)b * h * n * d, r = (size_t)b * h * n;
                double *Q = vec(t), *K = vec(t), *V = vec(t), *dO = vec(t), *O = vec(t), *L = vec(r);
                double *dQ = vec(t), *dK = vec(t), *dV = vec(t);
                oracle_attn_fwd(b, h, n, d, 0.4, causal, masked ? block : 1, masked ? nblk : 1, kp, Q, K, V, O, L);
                oracle_attn_bwd(b, h, n, d, 0.4, causal, masked ? block : 1, masked ? nblk : 1, kp, Q, K, V, O, dO,
                                L, dQ, dK, dV);
                for (size_t i = 0; i < t; ++i) sum += dQ[i] + dK[i] + dV[i];
                if (n > 0) {
                    double *f = vec((size_t)n * n), *q = vec((size_t)n * n), *p = vec((size_t)n * n);
                    oracle_attn_bwd_head(n, d, 0.4, causal, masked ? block : 1, masked ? nblk : 1, kp, Q, K, V, O,
                                         dO, L, dQ, dK, dV, f, q, p);
                    int rows[2] = {0, n - 1};
                    double *sq = vec(2 * (size_t)d), *sk = vec(2 * (size_t)d), *sv = vec(2 * (size_t)d);
                    oracle_attn_bwd_sampled(n, d, 0.4, causal, masked ? block : 1, masked ? nblk : 1, kp, Q + 0, K, V,
                                            O, dO, L, 2, rows, sq, 2, rows, sk, sv);
                    sum += f[0] + q[0] + p[0] + sq[0] + sk[d] + sv[2 * d - 1];
                    free(f); free(q); free(p); free(sq); free(sk); free(sv);
                }
                free(Q); free(K); free(V); free(dO); free(O); free(L); free(dQ); free(dK); free(dV); free(keep);
            }
    {
        const int n = 9, d = 4;
        double *A1 = vec(n * d), *A2 = vec(n * d), *A3 = vec(n * d), *dO = vec(n * d), *X = vec(d * d), *Y = vec(d * d);
        double *g = vec(d * d), *f = vec(n * n), *q = vec(n * n), *p = vec(n * n);
        long long io[2];
        oracle_wgrad(n, d, A1, A2, A3, dO, X, Y, g, f, q, p);
        oracle_wgrad(n, d, A1, A2, A3, dO, X, Y, g, NULL, NULL, NULL);
        for (int B = 1; B <= 10; B += 3) {
            oracle_small_cache_wgrad(n, d, B, A1, A2, A3, dO, X, Y, g, io);
            sum += g[0] + (double)io[0];
        }
        free(A1); free(A2); free(A3); free(dO); free(X); free(Y); free(g); free(f); free(q); free(p);
    }
    printf("checksum %.6f\n", sum);
    return 0;
}
