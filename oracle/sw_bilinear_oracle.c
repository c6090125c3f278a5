/*
 * sw_bilinear_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * The generalisation of Section 6.6: a recursive algorithm built from a way to multiply 2 x 2 block matrices
 * with q block products.  It forms q linear combinations of the quadrants of A and of B, multiplies them
 * pairwise (recursively), and forms the quadrants of C as linear combinations of the q products.  Two
 * schemes are tabulated here, both with coefficients in {-1, 0, +1}:
 *   scheme 0  Strassen's original algorithm (q = 7, 18 additions; the count Section 3.3.2 uses),
 *   scheme 1  the classical algorithm written recursively (q = 8, 4 additions; Section 6.6.1).
 * Every combination is summed left to right over the quadrants 11, 12, 21, 22 (or over the products 0..q-1),
 * a leading -1 being a negation.  Leaf: the classical product, k ascending, multiply then add.
 * Shares no code with the HIP path.  Compile with -ffp-contract=off.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int q; int U[8][4]; int V[8][4]; int W[4][8]; } scheme_t;

static const scheme_t SCHEMES[2] = {
    /* Strassen 1969: M1=(A11+A22)(B11+B22) M2=(A21+A22)B11 M3=A11(B12-B22) M4=A22(B21-B11) M5=(A11+A12)B22
       M6=(A21-A11)(B11+B12) M7=(A12-A22)(B21+B22); C11=M1+M4-M5+M7 C12=M3+M5 C21=M2+M4 C22=M1-M2+M3+M6 */
    {7,
     {{1, 0, 0, 1}, {0, 0, 1, 1}, {1, 0, 0, 0}, {0, 0, 0, 1}, {1, 1, 0, 0}, {-1, 0, 1, 0}, {0, 1, 0, -1}, {0, 0, 0, 0}},
     {{1, 0, 0, 1}, {1, 0, 0, 0}, {0, 1, 0, -1}, {-1, 0, 1, 0}, {0, 0, 0, 1}, {1, 1, 0, 0}, {0, 0, 1, 1}, {0, 0, 0, 0}},
     {{1, 0, 0, 1, -1, 0, 1, 0}, {0, 0, 1, 0, 1, 0, 0, 0}, {0, 1, 0, 1, 0, 0, 0, 0}, {1, -1, 1, 0, 0, 1, 0, 0}}},
    /* classical: C11=A11B11+A12B21 C12=A11B12+A12B22 C21=A21B11+A22B21 C22=A21B12+A22B22 */
    {8,
     {{1, 0, 0, 0}, {0, 1, 0, 0}, {1, 0, 0, 0}, {0, 1, 0, 0}, {0, 0, 1, 0}, {0, 0, 0, 1}, {0, 0, 1, 0}, {0, 0, 0, 1}},
     {{1, 0, 0, 0}, {0, 0, 1, 0}, {0, 1, 0, 0}, {0, 0, 0, 1}, {1, 0, 0, 0}, {0, 0, 1, 0}, {0, 1, 0, 0}, {0, 0, 0, 1}},
     {{1, 1, 0, 0, 0, 0, 0, 0}, {0, 0, 1, 1, 0, 0, 0, 0}, {0, 0, 0, 0, 1, 1, 0, 0}, {0, 0, 0, 0, 0, 0, 1, 1}}},
};

typedef struct { int64_t leaf_mul, leaf_add, block_add, leaf_calls; } bil_counters;
static bil_counters g_cnt;
void sw_bilinear_reset_counters(void) { memset(&g_cnt, 0, sizeof g_cnt); }
void sw_bilinear_get_counters(bil_counters *out) { *out = g_cnt; }

__attribute__((target_clones("avx2", "default")))
static void classical(const double *A, int64_t lda, const double *B, int64_t ldb, double *C, int64_t ldc, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        double *c = C + i * ldc;
        const double a0 = A[i * lda];
        for (int64_t j = 0; j < n; ++j) c[j] = a0 * B[j];
        for (int64_t k = 1; k < n; ++k) {
            const double a = A[i * lda + k];
            const double *b = B + k * ldb;
            for (int64_t j = 0; j < n; ++j) c[j] = c[j] + a * b[j];
        }
    }
    g_cnt.leaf_mul += n * n * n;
    g_cnt.leaf_add += n * n * n - n * n;
    g_cnt.leaf_calls += 1;
}

/* Z = sum_k coef[k] * X[k], left to right over the nonzero coefficients; counts (terms - 1) block additions */
static void combine(double *Z, int64_t ldz, const double *const *X, const int64_t *ldx, const int *coef, int nterms, int64_t h)
{
    int first = 1;
    for (int k = 0; k < nterms; ++k) {
        if (coef[k] == 0) continue;
        for (int64_t i = 0; i < h; ++i)
            for (int64_t j = 0; j < h; ++j) {
                const double x = X[k][i * ldx[k] + j];
                if (first) Z[i * ldz + j] = coef[k] > 0 ? x : -x;
                else Z[i * ldz + j] = coef[k] > 0 ? Z[i * ldz + j] + x : Z[i * ldz + j] - x;
            }
        if (!first) g_cnt.block_add += h * h;
        first = 0;
    }
}

static int rec(const scheme_t *s, const double *A, int64_t lda, const double *B, int64_t ldb, double *C, int64_t ldc,
               int64_t n, int levels)
{
    if (levels == 0) { classical(A, lda, B, ldb, C, ldc, n); return 0; }
    const int64_t h = n / 2;
    const size_t hh = (size_t)h * (size_t)h;
    double *buf = (double *)malloc((size_t)(2 + s->q) * hh * sizeof(double));
    if (!buf) return -1;
    double *T = buf, *S = buf + hh, *Q = S + hh;
    const double *Aq[4] = {A, A + h, A + h * lda, A + h * lda + h};
    const double *Bq[4] = {B, B + h, B + h * ldb, B + h * ldb + h};
    const int64_t la[4] = {lda, lda, lda, lda}, lb[4] = {ldb, ldb, ldb, ldb};
    int rc = 0;
    for (int i = 0; i < s->q && rc == 0; ++i) {
        combine(T, h, Aq, la, s->U[i], 4, h);
        combine(S, h, Bq, lb, s->V[i], 4, h);
        rc = rec(s, T, h, S, h, Q + (size_t)i * hh, h, h, levels - 1);
    }
    if (rc == 0) {
        const double *Qp[8];
        int64_t lq[8];
        for (int i = 0; i < s->q; ++i) { Qp[i] = Q + (size_t)i * hh; lq[i] = h; }
        double *Cq[4] = {C, C + h, C + h * ldc, C + h * ldc + h};
        for (int c = 0; c < 4; ++c) combine(Cq[c], ldc, Qp, lq, s->W[c], s->q, h);
    }
    free(buf);
    return rc;
}

/* C = A*B, n x n row-major dense, n a multiple of 2^levels.  scheme 0 = Strassen, 1 = recursive classical.
 * Returns 0, -1 out of memory, -2 bad argument. */
int sw_bilinear_gemm(int64_t n, const double *A, const double *B, double *C, int levels, int scheme)
{
    if (n < 0 || levels < 0 || levels > 30 || scheme < 0 || scheme > 1 || (n > 0 && (!A || !B || !C))) return -2;
    if (n == 0) return 0;
    if (n % ((int64_t)1 << levels)) return -2;
    return rec(&SCHEMES[scheme], A, n, B, n, C, n, n, levels);
}

/* the tables themselves, for tests: out[0..q*4) = U, then V, then W as 4 x q; returns q */
int sw_bilinear_tables(int scheme, int *out)
{
    if (scheme < 0 || scheme > 1) return -1;
    const scheme_t *s = &SCHEMES[scheme];
    int k = 0;
    for (int i = 0; i < s->q; ++i) for (int j = 0; j < 4; ++j) out[k++] = s->U[i][j];
    for (int i = 0; i < s->q; ++i) for (int j = 0; j < 4; ++j) out[k++] = s->V[i][j];
    for (int c = 0; c < 4; ++c) for (int i = 0; i < s->q; ++i) out[k++] = s->W[c][i];
    return s->q;
}
