/*
 * sw_bilinear_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * The generalisation of Section 6.6: a recursive algorithm built from a way to multiply n0 x n0 block matrices
 * with q block products (Section 6.6.2: q < n0^3 for a fast algorithm, exponent w0 = log_n0 q).  It forms q
 * linear combinations of the n0^2 blocks of A and of B, multiplies them pairwise (recursively), and forms the
 * blocks of C as linear combinations of the q products.  Four schemes are tabulated here, all with coefficients
 * in {-1, 0, +1}:
 *   scheme 0  Strassen's original algorithm (n0 = 2, q = 7, 18 additions; the count Section 3.3.2 uses),
 *   scheme 1  the classical algorithm written recursively on 2 x 2 blocks (q = 8, 4 additions; Section 6.6.1),
 *   scheme 2  Laderman's algorithm for 3 x 3 blocks (n0 = 3, q = 23; a scheme of the kind Section 6.6.2 names),
 *   scheme 3  the classical algorithm written recursively on 3 x 3 blocks (q = 27, 18 additions).
 * Blocks are numbered row-major (11, 12, .., n0 n0).  Every combination is summed left to right over the
 * blocks (or over the products 0..q-1), a leading -1 being a negation.  The scheme may change from level to
 * level (a 2 x 2 step above a 3 x 3 step, ...).  Leaf: the classical product, k ascending, multiply then add.
 * Shares no code with the HIP path.  Compile with -ffp-contract=off.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MAXQ 27
#define MAXB 9
#define NSCHEMES 4

typedef struct { int n0; int q; int U[MAXQ][MAXB]; int V[MAXQ][MAXB]; int W[MAXB][MAXQ]; } scheme_t;

static scheme_t SCHEMES[NSCHEMES];
static int g_built = 0;

/* terms of one combination: entries are +-(10 r + c) for block (r, c), 1-based; 0 ends the list */
static void fill_row(int *row, int n0, const int *terms)
{
    for (; *terms; ++terms) {
        const int t = *terms > 0 ? *terms : -*terms;
        row[(t / 10 - 1) * n0 + (t % 10 - 1)] = *terms > 0 ? 1 : -1;
    }
}

/* products contributing to one block of C: +-(index + 1); 0 ends the list */
static void fill_out(int *row, const int *prods)
{
    for (; *prods; ++prods) row[(*prods > 0 ? *prods : -*prods) - 1] = *prods > 0 ? 1 : -1;
}

static void build_schemes(void)
{
    if (g_built) return;
    memset(SCHEMES, 0, sizeof SCHEMES);

    /* Strassen 1969: M1=(A11+A22)(B11+B22) M2=(A21+A22)B11 M3=A11(B12-B22) M4=A22(B21-B11) M5=(A11+A12)B22
       M6=(A21-A11)(B11+B12) M7=(A12-A22)(B21+B22); C11=M1+M4-M5+M7 C12=M3+M5 C21=M2+M4 C22=M1-M2+M3+M6 */
    {
        scheme_t *s = &SCHEMES[0];
        s->n0 = 2; s->q = 7;
        static const int a[7][5] = {{11, 22}, {21, 22}, {11}, {22}, {11, 12}, {-11, 21}, {12, -22}};
        static const int b[7][5] = {{11, 22}, {11}, {12, -22}, {-11, 21}, {22}, {11, 12}, {21, 22}};
        static const int c[4][8] = {{1, 4, -5, 7}, {3, 5}, {2, 4}, {1, -2, 3, 6}};
        for (int i = 0; i < 7; ++i) { fill_row(s->U[i], 2, a[i]); fill_row(s->V[i], 2, b[i]); }
        for (int k = 0; k < 4; ++k) fill_out(s->W[k], c[k]);
    }
    /* classical on n0 x n0 blocks: product (i, j, k) = A_ik * B_kj, numbered with k fastest, C_ij = sum_k */
    for (int id = 1; id <= 3; id += 2) {
        scheme_t *s = &SCHEMES[id];
        const int n0 = id == 1 ? 2 : 3;
        s->n0 = n0; s->q = n0 * n0 * n0;
        int p = 0;
        for (int i = 0; i < n0; ++i)
            for (int j = 0; j < n0; ++j)
                for (int k = 0; k < n0; ++k, ++p) {
                    s->U[p][i * n0 + k] = 1;
                    s->V[p][k * n0 + j] = 1;
                    s->W[i * n0 + j][p] = 1;
                }
    }
    /* Laderman 1976, 23 products for 3 x 3 (a_ij, b_ij the blocks):
       m1 =(a11+a12+a13-a21-a22-a32-a33) b22            m2 =(a11-a21)(-b12+b22)
       m3 = a22 (-b11+b12+b21-b22-b23-b31+b33)          m4 =(-a11+a21+a22)(b11-b12+b22)
       m5 =(a21+a22)(-b11+b12)                          m6 = a11 b11
       m7 =(-a11+a31+a32)(b11-b13+b23)                  m8 =(-a11+a31)(b13-b23)
       m9 =(a31+a32)(-b11+b13)                          m10=(a11+a12+a13-a22-a23-a31-a32) b23
       m11= a32 (-b11+b13+b21-b22-b23-b31+b32)          m12=(-a13+a32+a33)(b22+b31-b32)
       m13=(a13-a33)(b22-b32)                           m14= a13 b31
       m15=(a32+a33)(-b31+b32)                          m16=(-a13+a22+a23)(b23+b31-b33)
       m17=(a13-a23)(b23-b33)                           m18=(a22+a23)(-b31+b33)
       m19= a12 b21    m20= a23 b32    m21= a21 b13    m22= a31 b12    m23= a33 b33
       c11=m6+m14+m19                 c12=m1+m4+m5+m6+m12+m14+m15      c13=m6+m7+m9+m10+m14+m16+m18
       c21=m2+m3+m4+m6+m14+m16+m17    c22=m2+m4+m5+m6+m20              c23=m14+m16+m17+m18+m21
       c31=m6+m7+m8+m11+m12+m13+m14   c32=m12+m13+m14+m15+m22          c33=m6+m7+m8+m9+m23 */
    {
        scheme_t *s = &SCHEMES[2];
        s->n0 = 3; s->q = 23;
        static const int a[23][8] = {
            {11, 12, 13, -21, -22, -32, -33}, {11, -21}, {22}, {-11, 21, 22}, {21, 22}, {11}, {-11, 31, 32}, {-11, 31},
            {31, 32}, {11, 12, 13, -22, -23, -31, -32}, {32}, {-13, 32, 33}, {13, -33}, {13}, {32, 33}, {-13, 22, 23},
            {13, -23}, {22, 23}, {12}, {23}, {21}, {31}, {33}};
        static const int b[23][8] = {
            {22}, {-12, 22}, {-11, 12, 21, -22, -23, -31, 33}, {11, -12, 22}, {-11, 12}, {11}, {11, -13, 23}, {13, -23},
            {-11, 13}, {23}, {-11, 13, 21, -22, -23, -31, 32}, {22, 31, -32}, {22, -32}, {31}, {-31, 32}, {23, 31, -33},
            {23, -33}, {-31, 33}, {21}, {32}, {13}, {12}, {33}};
        static const int c[9][8] = {
            {6, 14, 19}, {1, 4, 5, 6, 12, 14, 15}, {6, 7, 9, 10, 14, 16, 18},
            {2, 3, 4, 6, 14, 16, 17}, {2, 4, 5, 6, 20}, {14, 16, 17, 18, 21},
            {6, 7, 8, 11, 12, 13, 14}, {12, 13, 14, 15, 22}, {6, 7, 8, 9, 23}};
        for (int i = 0; i < 23; ++i) { fill_row(s->U[i], 3, a[i]); fill_row(s->V[i], 3, b[i]); }
        for (int k = 0; k < 9; ++k) fill_out(s->W[k], c[k]);
    }
    g_built = 1;
}

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

/* one step with the scheme of this level, then the next levels on the q subproblems */
static int rec(const int *scheme, const double *A, int64_t lda, const double *B, int64_t ldb, double *C, int64_t ldc,
               int64_t n, int levels)
{
    if (levels == 0) { classical(A, lda, B, ldb, C, ldc, n); return 0; }
    const scheme_t *s = &SCHEMES[scheme[0]];
    const int n0 = s->n0, nb = n0 * n0;
    const int64_t h = n / n0;
    const size_t hh = (size_t)h * (size_t)h;
    double *buf = (double *)malloc((size_t)(2 + s->q) * hh * sizeof(double));
    if (!buf) return -1;
    double *T = buf, *S = buf + hh, *Q = S + hh;
    const double *Ab[MAXB], *Bb[MAXB];
    double *Cb[MAXB];
    int64_t la[MAXB], lb[MAXB];
    for (int k = 0; k < nb; ++k) {
        Ab[k] = A + (k / n0) * h * lda + (k % n0) * h;
        Bb[k] = B + (k / n0) * h * ldb + (k % n0) * h;
        Cb[k] = C + (k / n0) * h * ldc + (k % n0) * h;
        la[k] = lda;
        lb[k] = ldb;
    }
    int rc = 0;
    for (int i = 0; i < s->q && rc == 0; ++i) {
        combine(T, h, Ab, la, s->U[i], nb, h);
        combine(S, h, Bb, lb, s->V[i], nb, h);
        rc = rec(scheme + 1, T, h, S, h, Q + (size_t)i * hh, h, h, levels - 1);
    }
    if (rc == 0) {
        const double *Qp[MAXQ];
        int64_t lq[MAXQ];
        for (int i = 0; i < s->q; ++i) { Qp[i] = Q + (size_t)i * hh; lq[i] = h; }
        for (int c = 0; c < nb; ++c) combine(Cb[c], ldc, Qp, lq, s->W[c], s->q, h);
    }
    free(buf);
    return rc;
}

/* C = A*B, n x n row-major dense; level i (0 = top) uses scheme schemes[i]; n must be a multiple of the
 * product of the levels' block counts n0.  Returns 0, -1 out of memory, -2 bad argument. */
int sw_bilinear_gemm_levels(int64_t n, const double *A, const double *B, double *C, int levels, const int *schemes)
{
    build_schemes();
    if (n < 0 || levels < 0 || levels > 30 || (levels > 0 && !schemes) || (n > 0 && (!A || !B || !C))) return -2;
    int64_t radix = 1;
    for (int i = 0; i < levels; ++i) {
        if (schemes[i] < 0 || schemes[i] >= NSCHEMES) return -2;
        radix *= SCHEMES[schemes[i]].n0;
        if (radix > ((int64_t)1 << 40)) return -2;
    }
    if (n == 0) return 0;
    if (n % radix) return -2;
    return rec(schemes, A, n, B, n, C, n, n, levels);
}

/* the same scheme at every level */
int sw_bilinear_gemm(int64_t n, const double *A, const double *B, double *C, int levels, int scheme)
{
    int all[31];
    if (levels < 0 || levels > 30) return -2;
    for (int i = 0; i < levels; ++i) all[i] = scheme;
    return sw_bilinear_gemm_levels(n, A, B, C, levels, all);
}

/* the tables themselves, for tests: with b = n0^2, out[0 .. q*b) = U (q rows of b), then V, then W as b rows of q;
 * *n0_out = n0; returns q, or -1 for an unknown scheme.  out must hold 3 * 27 * 9 ints. */
int sw_bilinear_tables(int scheme, int *out, int *n0_out)
{
    build_schemes();
    if (scheme < 0 || scheme >= NSCHEMES) return -1;
    const scheme_t *s = &SCHEMES[scheme];
    const int nb = s->n0 * s->n0;
    int k = 0;
    for (int i = 0; i < s->q; ++i) for (int j = 0; j < nb; ++j) out[k++] = s->U[i][j];
    for (int i = 0; i < s->q; ++i) for (int j = 0; j < nb; ++j) out[k++] = s->V[i][j];
    for (int c = 0; c < nb; ++c) for (int i = 0; i < s->q; ++i) out[k++] = s->W[c][i];
    if (n0_out) *n0_out = s->n0;
    return s->q;
}
