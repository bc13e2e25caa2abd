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
 * the paper's own gradient g = A_1^T p A_2 evaluated by oracle_alg1_wgrad below,
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
 * The paper's own target, in the order of its no-cache algorithm (App. C.1):
 *   A = exp(A_1 X A_2^T); l = A 1; f = diag(l)^{-1} A; h = A_3 Y; q = dO h^T;
 *   p = f o q - diag((f o q) 1) f;  g = A_1^T p A_2   (definition of the backward gradient).
 * No scale, no mask, no max-subtraction (inputs must keep exp in range).  g is d x d;
 * f_out, q_out, p_out are NULL or n x n.
 */
void oracle_alg1_wgrad(int n, int d, const double *A1, const double *A2, const double *A3,
                       const double *dO, const double *X, const double *Y, double *g,
                       double *f_out, double *q_out, double *p_out)
{
    size_t nn = (size_t)n * n, nd = (size_t)n * d;
    double *S = (double *)malloc(sizeof(double) * nd);
    double *A = (double *)malloc(sizeof(double) * nn);
    double *l = (double *)malloc(sizeof(double) * (size_t)n);
    double *h = (double *)malloc(sizeof(double) * nd);
    double *q = (double *)malloc(sizeof(double) * nn);
    double *p = (double *)malloc(sizeof(double) * nn);
    double *T = (double *)malloc(sizeof(double) * nd);
    matmul(n, d, d, A1, 0, X, 0, S);  /* S = A_1 X */
    matmul(n, n, d, S, 0, A2, 1, A);  /* A = S A_2^T */
    for (size_t t = 0; t < nn; ++t)
        A[t] = exp(A[t]);
    for (int i = 0; i < n; ++i) {
        l[i] = 0.0;
        for (int j = 0; j < n; ++j)
            l[i] += A[(size_t)i * n + j];
    }
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            A[(size_t)i * n + j] /= l[i]; /* A now holds f */
    matmul(n, d, d, A3, 0, Y, 0, h);  /* h = A_3 Y */
    matmul(n, n, d, dO, 0, h, 1, q);  /* q = dO h^T */
    for (int i = 0; i < n; ++i) {
        double v = 0.0;
        for (int j = 0; j < n; ++j)
            v += A[(size_t)i * n + j] * q[(size_t)i * n + j];
        for (int j = 0; j < n; ++j)
            p[(size_t)i * n + j] = A[(size_t)i * n + j] * q[(size_t)i * n + j] - v * A[(size_t)i * n + j];
    }
    matmul(d, n, n, A1, 1, p, 0, T);  /* T = A_1^T p  (d x n) */
    matmul(d, d, n, T, 0, A2, 0, g);  /* g = T A_2 */
    if (f_out) memcpy(f_out, A, sizeof(double) * nn);
    if (q_out) memcpy(q_out, q, sizeof(double) * nn);
    if (p_out) memcpy(p_out, p, sizeof(double) * nn);
    free(S); free(A); free(l); free(h); free(q); free(p); free(T);
}
