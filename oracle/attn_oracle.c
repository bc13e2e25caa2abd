/*
 * attn_oracle.c -- float64 CPU oracle for exact softmax attention, forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the GPU
 * library must compute.  It shares no code, header, table or helper with the HIP path
 * and must never be called from it: only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark use it.
 *
 * Source of each formula: "On Fine-Grained I/O Complexity of Attention Backward Passes"
 * (arXiv 2410.09397).  The paper works with S = A_1 X (queries), A_2 (keys), h = A_3 Y
 * (values); here they are called Q, K, V.  The paper has no 1/sqrt(d) factor, no mask
 * and stores l = A 1_n rather than its logarithm; the readings taken are:
 *   - scores are scale * Q K^T; with scale = 1 and no mask everything below is the
 *     paper's definition verbatim in meaning,
 *   - a masked (i,j) pair is simply absent from every sum over j (its f, q-weight and p
 *     entries are 0),
 *   - LSE_i = log l_i, evaluated as m_i + log sum_j exp(s_ij - m_i),
 *   - the matrix form "f = diag(l) A" in the definition of f is read as diag(l)^{-1} A,
 *     as the row form two lines above it and the forward definition (D^{-1}) require,
 *   - a query row with no visible key has O = 0, LSE = -inf and contributes nothing to
 *     any gradient,
 *   - dV is not derived in the paper (Y is held fixed there); it follows from O = f h.
 *
 * Parity pins (tests/test_oracle_*.py): central finite differences of the forward loss,
 * the paper's own gradient g = A_1^T p A_2 evaluated by oracle_wgrad below (and the same by
 * the four-phase small-cache scheme, oracle_small_cache_wgrad),
 * closed forms (n = 1, Q = 0, causal first row), the zero row-sum of p, key-shift and
 * key-permutation invariances, and an independent library evaluation (softmax +
 * autograd in float64).  No function here is "parity unpinned".
 *
 * Layout: every [batch, heads, n, d] tensor is contiguous, d fastest; LSE is
 * [batch, heads, n].  keep is NULL or an nblk x nblk byte matrix, row = query block,
 * column = key block, nonzero = block kept; block is the block edge in rows.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* Visibility of key j to query i: the causal rule and the block mask both apply. */
static int allowed(int i, int j, int causal, int block, int nblk, const unsigned char *keep)
{
    if (causal && j > i)
        return 0;
    if (keep && !keep[(size_t)(i / block) * nblk + (j / block)])
        return 0;
    return 1;
}

static double dot(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int k = 0; k < d; ++k)
        s += a[k] * b[k];
    return s;
}

/*
 * Forward for one query row i of one head (forward definition, Sec. 3.1; A, l, f, O of
 * App. B.4 with the max-subtraction reading above).  s is scratch of n doubles.
 */
static void fwd_row(int i, int n, int d, double scale, int causal, int block, int nblk,
                    const unsigned char *keep, const double *Q, const double *K,
                    const double *V, double *O_i, double *LSE_i, double *s)
{
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        if (!allowed(i, j, causal, block, nblk, keep))
            continue;
        s[j] = scale * dot(Q + (size_t)i * d, K + (size_t)j * d, d);
        if (s[j] > m)
            m = s[j];
    }
    for (int k = 0; k < d; ++k)
        O_i[k] = 0.0;
    if (m == -INFINITY) { /* no visible key */
        *LSE_i = -INFINITY;
        return;
    }
    double l = 0.0;
    for (int j = 0; j < n; ++j)
        if (allowed(i, j, causal, block, nblk, keep))
            l += exp(s[j] - m);
    double lse = m + log(l);
    for (int j = 0; j < n; ++j) {
        if (!allowed(i, j, causal, block, nblk, keep))
            continue;
        double f = exp(s[j] - lse); /* f_ij = A_ij / l_i */
        for (int k = 0; k < d; ++k)
            O_i[k] += f * V[(size_t)j * d + k]; /* O = f h */
    }
    *LSE_i = lse;
}

/* O [b,h,n,d] and LSE [b,h,n] from Q, K, V.  Rows are independent. */
void oracle_attn_fwd(int batch, int heads, int n, int d, double scale, int causal,
                     int block, int nblk, const unsigned char *keep, const double *Q,
                     const double *K, const double *V, double *O, double *LSE)
{
    long total = (long)batch * heads * n;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
#pragma omp for schedule(dynamic, 16)
        for (long r = 0; r < total; ++r) {
            long bh = r / n;
            int i = (int)(r % n);
            size_t off = (size_t)bh * n * d;
            fwd_row(i, n, d, scale, causal, block, nblk, keep, Q + off, K + off, V + off,
                    O + off + (size_t)i * d, LSE + (size_t)bh * n + i, s);
        }
        free(s);
    }
}

/*
 * Backward for one head, from the GIVEN O and LSE (the backward pass assumes l and O
 * were kept by the forward; large-cache algorithm, App. D).  Steps, per query row i:
 *   f_ij  = exp(scale q_i.k_j - LSE_i)               (definition of f)
 *   v_i   = sum_k dO_ik O_ik                         (second matrix form of p)
 *   q_ij  = dO_i . V_j                               (definition of q)
 *   p_ij  = f_ij (q_ij - v_i)                        (definition of p)
 *   dV_j += f_ij dO_i        (from O = f h)
 *   dK_j += scale p_ij Q_i   (same contraction as T = A_1^T p)
 *   dQ_i += scale p_ij K_j   (the p A_2 factor of g = A_1^T p A_2)
 * f_out, q_out, p_out are NULL or n x n matrices receiving f, q, p (0 where masked).
 */
void oracle_attn_bwd_head(int n, int d, double scale, int causal, int block, int nblk,
                          const unsigned char *keep, const double *Q, const double *K,
                          const double *V, const double *O, const double *dO,
                          const double *LSE, double *dQ, double *dK, double *dV,
                          double *f_out, double *q_out, double *p_out)
{
    size_t nd = (size_t)n * d;
    memset(dQ, 0, sizeof(double) * nd);
    memset(dK, 0, sizeof(double) * nd);
    memset(dV, 0, sizeof(double) * nd);
    if (f_out) memset(f_out, 0, sizeof(double) * (size_t)n * n);
    if (q_out) memset(q_out, 0, sizeof(double) * (size_t)n * n);
    if (p_out) memset(p_out, 0, sizeof(double) * (size_t)n * n);
    for (int i = 0; i < n; ++i) {
        const double *Qi = Q + (size_t)i * d, *dOi = dO + (size_t)i * d;
        if (LSE[i] == -INFINITY)
            continue;
        double v = dot(dOi, O + (size_t)i * d, d);
        for (int j = 0; j < n; ++j) {
            if (!allowed(i, j, causal, block, nblk, keep))
                continue;
            const double *Kj = K + (size_t)j * d, *Vj = V + (size_t)j * d;
            double f = exp(scale * dot(Qi, Kj, d) - LSE[i]);
            double q = dot(dOi, Vj, d);
            double p = f * (q - v);
            for (int k = 0; k < d; ++k) {
                dV[(size_t)j * d + k] += f * dOi[k];
                dK[(size_t)j * d + k] += scale * p * Qi[k];
                dQ[(size_t)i * d + k] += scale * p * Kj[k];
            }
            if (f_out) f_out[(size_t)i * n + j] = f;
            if (q_out) q_out[(size_t)i * n + j] = q;
            if (p_out) p_out[(size_t)i * n + j] = p;
        }
    }
}

/* dQ, dK, dV [b,h,n,d] for every (batch, head); heads are independent. */
void oracle_attn_bwd(int batch, int heads, int n, int d, double scale, int causal,
                     int block, int nblk, const unsigned char *keep, const double *Q,
                     const double *K, const double *V, const double *O, const double *dO,
                     const double *LSE, double *dQ, double *dK, double *dV)
{
    long nbh = (long)batch * heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < nbh; ++bh) {
        size_t off = (size_t)bh * n * d;
        oracle_attn_bwd_head(n, d, scale, causal, block, nblk, keep, Q + off, K + off,
                             V + off, O + off, dO + off, LSE + (size_t)bh * n, dQ + off,
                             dK + off, dV + off, NULL, NULL, NULL);
    }
}

/*
 * Sampled backward for one head, for full-size problems where the whole head is too
 * slow: dQ for the listed query rows and dK, dV for the listed key rows, each the same
 * sums as oracle_attn_bwd_head restricted to that row.  dQ_rows is [nq, d], dK_rows and
 * dV_rows are [nk, d].
 */
void oracle_attn_bwd_sampled(int n, int d, double scale, int causal, int block, int nblk,
                             const unsigned char *keep, const double *Q, const double *K,
                             const double *V, const double *O, const double *dO,
                             const double *LSE, int nq, const int *q_rows, double *dQ_rows,
                             int nk, const int *k_rows, double *dK_rows, double *dV_rows)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int a = 0; a < nq; ++a) {
        int i = q_rows[a];
        const double *Qi = Q + (size_t)i * d, *dOi = dO + (size_t)i * d;
        double *out = dQ_rows + (size_t)a * d;
        for (int k = 0; k < d; ++k)
            out[k] = 0.0;
        if (LSE[i] == -INFINITY)
            continue;
        double v = dot(dOi, O + (size_t)i * d, d);
        for (int j = 0; j < n; ++j) {
            if (!allowed(i, j, causal, block, nblk, keep))
                continue;
            const double *Kj = K + (size_t)j * d;
            double f = exp(scale * dot(Qi, Kj, d) - LSE[i]);
            double p = f * (dot(dOi, V + (size_t)j * d, d) - v);
            for (int k = 0; k < d; ++k)
                out[k] += scale * p * Kj[k];
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int a = 0; a < nk; ++a) {
        int j = k_rows[a];
        const double *Kj = K + (size_t)j * d, *Vj = V + (size_t)j * d;
        double *oK = dK_rows + (size_t)a * d, *oV = dV_rows + (size_t)a * d;
        for (int k = 0; k < d; ++k)
            oK[k] = oV[k] = 0.0;
        for (int i = 0; i < n; ++i) {
            if (!allowed(i, j, causal, block, nblk, keep) || LSE[i] == -INFINITY)
                continue;
            const double *Qi = Q + (size_t)i * d, *dOi = dO + (size_t)i * d;
            double v = dot(dOi, O + (size_t)i * d, d);
            double f = exp(scale * dot(Qi, Kj, d) - LSE[i]);
            double p = f * (dot(dOi, Vj, d) - v);
            for (int k = 0; k < d; ++k) {
                oV[k] += f * dOi[k];
                oK[k] += scale * p * Qi[k];
            }
        }
    }
}

/* C[m x n] = A[m x k] B[k x n], or with A^T / B^T when ta / tb is set (row-major). */
static void matmul(int m, int n, int k, const double *A, int ta, const double *B, int tb,
                   double *C)
{
    for (int i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int t = 0; t < k; ++t) {
                double a = ta ? A[(size_t)t * m + i] : A[(size_t)i * k + t];
                double b = tb ? B[(size_t)j * k + t] : B[(size_t)t * n + j];
                s += a * b;
            }
            C[(size_t)i * n + j] = s;
        }
}

/*
 * The paper's own target (Def. 3.2): g = dL/dX = A_1^T p A_2, a d x d matrix, with
 * S = A_1 X, h = A_3 Y and, per query row i (App. B.4, definitions of A, l, f, q, p):
 *   f_ij = exp(<S_i, A_2j>) / sum_j' exp(<S_i, A_2j'>),  q_ij = <dO_i, h_j>,
 *   v_i = sum_j f_ij q_ij,  p_ij = f_ij (q_ij - v_i).
 * Evaluated row by row as g = sum_i A_1i^T (sum_j p_ij A_2j).  No scale, no mask and no
 * max-subtraction, as in the paper (inputs must keep exp in range).  f_out, q_out, p_out are
 * NULL or n x n.
 */
void oracle_wgrad(int n, int d, const double *A1, const double *A2, const double *A3,
                  const double *dO, const double *X, const double *Y, double *g,
                  double *f_out, double *q_out, double *p_out)
{
    size_t nd = (size_t)n * d;
    double *S = (double *)malloc(sizeof(double) * nd);
    double *h = (double *)malloc(sizeof(double) * nd);
    double *f = (double *)malloc(sizeof(double) * (size_t)n);
    double *q = (double *)malloc(sizeof(double) * (size_t)n);
    double *u = (double *)malloc(sizeof(double) * (size_t)d);
    matmul(n, d, d, A1, 0, X, 0, S);
    matmul(n, d, d, A3, 0, Y, 0, h);
    for (int a = 0; a < d * d; ++a)
        g[a] = 0.0;
    for (int i = 0; i < n; ++i) {
        double l = 0.0, v = 0.0;
        for (int j = 0; j < n; ++j) {
            f[j] = exp(dot(S + (size_t)i * d, A2 + (size_t)j * d, d));
            l += f[j];
        }
        for (int j = 0; j < n; ++j) {
            f[j] /= l;
            q[j] = dot(dO + (size_t)i * d, h + (size_t)j * d, d);
            v += f[j] * q[j];
        }
        for (int k = 0; k < d; ++k)
            u[k] = 0.0;
        for (int j = 0; j < n; ++j) {
            double p = f[j] * (q[j] - v);
            for (int k = 0; k < d; ++k)
                u[k] += p * A2[(size_t)j * d + k];
            if (f_out) f_out[(size_t)i * n + j] = f[j];
            if (q_out) q_out[(size_t)i * n + j] = q[j];
            if (p_out) p_out[(size_t)i * n + j] = p;
        }
        for (int a = 0; a < d; ++a)
            for (int k = 0; k < d; ++k)
                g[(size_t)a * d + k] += A1[(size_t)i * d + a] * u[k];
    }
    free(S); free(h); free(f); free(q); free(u);
}

/*
 * The same g by the small-cache scheme of App. C: four phases over B x B blocks, every n x n
 * intermediate (A, f, q, p) and the d x n matrix T passing through memory, so that no more than
 * a few B x B blocks are ever needed at once (the paper takes B = floor(sqrt(M / 4))).  Written
 * as blocked loops of our own; what is kept from the paper is the phase structure:
 *   phase 1: S = A_1 X;  A = exp(S A_2^T) with the row sums l gathered on the way;  f = A / l
 *   phase 2: h = A_3 Y;  q = dO h^T
 *   phase 3: v = rowsum(f o q);  p = f o q - diag(v) f
 *   phase 4: T = A_1^T p;  g = T A_2
 * Every product is a block product with a k-loop whose accumulator block stays in cache.
 * io[0] / io[1] receive the number of elements read from / written to memory (blocks at the
 * ragged edge count with their real size; the row vectors l and v count once per row block
 * and sweep).  Pinned by equality with oracle_wgrad for block edges that do and do not
 * divide n and d, and by the closed-form count of its own schedule.
 */
typedef struct { long long rd, wr; } io_count;

static int bmin(int a, int b) { return a < b ? a : b; }

/* C[m x n] = A B (or with transposes) in B x B blocks with the k-loop innermost; counts the
 * block transfers: per output block, 2 operand blocks per k-step in, one block out. */
static void blocked_matmul(int m, int n, int k, int B, const double *A, int ta, const double *Bm,
                           int tb, double *C, io_count *io)
{
    for (int i0 = 0; i0 < m; i0 += B)
        for (int j0 = 0; j0 < n; j0 += B) {
            int mi = bmin(B, m - i0), nj = bmin(B, n - j0);
            for (int i = 0; i < mi; ++i)
                for (int j = 0; j < nj; ++j)
                    C[(size_t)(i0 + i) * n + j0 + j] = 0.0;
            for (int k0 = 0; k0 < k; k0 += B) {
                int kk = bmin(B, k - k0);
                io->rd += (long long)mi * kk + (long long)kk * nj;
                for (int i = 0; i < mi; ++i)
                    for (int j = 0; j < nj; ++j) {
                        double acc = 0.0;
                        for (int t = 0; t < kk; ++t) {
                            double a = ta ? A[(size_t)(k0 + t) * m + i0 + i] : A[(size_t)(i0 + i) * k + k0 + t];
                            double b = tb ? Bm[(size_t)(j0 + j) * k + k0 + t] : Bm[(size_t)(k0 + t) * n + j0 + j];
                            acc += a * b;
                        }
                        C[(size_t)(i0 + i) * n + j0 + j] += acc;
                    }
            }
            io->wr += (long long)mi * nj;
        }
}

void oracle_small_cache_wgrad(int n, int d, int B, const double *A1, const double *A2,
                              const double *A3, const double *dO, const double *X, const double *Y,
                              double *g, long long *io_out)
{
    size_t nn = (size_t)n * n, nd = (size_t)n * d;
    io_count io = {0, 0};
    double *S = (double *)malloc(sizeof(double) * nd);
    double *h = (double *)malloc(sizeof(double) * nd);
    double *f = (double *)malloc(sizeof(double) * nn);
    double *q = (double *)malloc(sizeof(double) * nn);
    double *p = (double *)malloc(sizeof(double) * nn);
    double *T = (double *)malloc(sizeof(double) * nd);
    double *l = (double *)malloc(sizeof(double) * (size_t)n);
    double *v = (double *)malloc(sizeof(double) * (size_t)n);
    /* phase 1 */
    blocked_matmul(n, d, d, B, A1, 0, X, 0, S, &io);
    blocked_matmul(n, n, d, B, S, 0, A2, 1, f, &io);     /* f holds S A_2^T, block by block */
    for (int i0 = 0; i0 < n; i0 += B) {                  /* exp and row sums: one more pass over the blocks */
        int mi = bmin(B, n - i0);
        for (int i = 0; i < mi; ++i)
            l[i0 + i] = 0.0;
        for (int j0 = 0; j0 < n; j0 += B) {
            int nj = bmin(B, n - j0);
            io.rd += (long long)mi * nj;
            for (int i = 0; i < mi; ++i)
                for (int j = 0; j < nj; ++j) {
                    double a = exp(f[(size_t)(i0 + i) * n + j0 + j]);
                    f[(size_t)(i0 + i) * n + j0 + j] = a;
                    l[i0 + i] += a;
                }
            io.wr += (long long)mi * nj;
        }
        io.wr += mi;                                     /* l of this row block */
    }
    for (int i0 = 0; i0 < n; i0 += B) {                  /* f = A / l */
        int mi = bmin(B, n - i0);
        io.rd += mi;
        for (int j0 = 0; j0 < n; j0 += B) {
            int nj = bmin(B, n - j0);
            io.rd += (long long)mi * nj;
            for (int i = 0; i < mi; ++i)
                for (int j = 0; j < nj; ++j)
                    f[(size_t)(i0 + i) * n + j0 + j] /= l[i0 + i];
            io.wr += (long long)mi * nj;
        }
    }
    /* phase 2 */
    blocked_matmul(n, d, d, B, A3, 0, Y, 0, h, &io);
    blocked_matmul(n, n, d, B, dO, 0, h, 1, q, &io);
    /* phase 3: two sweeps over each row block */
    for (int i0 = 0; i0 < n; i0 += B) {
        int mi = bmin(B, n - i0);
        for (int i = 0; i < mi; ++i)
            v[i0 + i] = 0.0;
        for (int j0 = 0; j0 < n; j0 += B) {
            int nj = bmin(B, n - j0);
            io.rd += 2LL * mi * nj;
            for (int i = 0; i < mi; ++i)
                for (int j = 0; j < nj; ++j)
                    v[i0 + i] += f[(size_t)(i0 + i) * n + j0 + j] * q[(size_t)(i0 + i) * n + j0 + j];
        }
        for (int j0 = 0; j0 < n; j0 += B) {
            int nj = bmin(B, n - j0);
            io.rd += 2LL * mi * nj;
            for (int i = 0; i < mi; ++i)
                for (int j = 0; j < nj; ++j) {
                    size_t a = (size_t)(i0 + i) * n + j0 + j;
                    p[a] = f[a] * q[a] - v[i0 + i] * f[a];
                }
            io.wr += (long long)mi * nj;
        }
    }
    /* phase 4 */
    blocked_matmul(d, n, n, B, A1, 1, p, 0, T, &io);
    blocked_matmul(d, d, n, B, T, 0, A2, 0, g, &io);
    io_out[0] = io.rd;
    io_out[1] = io.wr;
    free(S); free(h); free(f); free(q); free(p); free(T); free(l); free(v);
}
