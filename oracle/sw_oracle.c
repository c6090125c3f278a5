/*
 * sw_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded CPU statement of what the Strassen-Winograd
 * hot path computes.  It shares no code with the HIP library and nothing in the
 * product path may call it; only tests, the smoke check and the CPU-baseline
 * leg of the benchmark do.
 *
 * What it follows:
 *   - problem statement C = A*B, A and B n x n (Algorithm 1, Require/Ensure);
 *   - one recursion step = the Strassen-Winograd tables (Appendix A): seven
 *     combinations T_i of A's quadrants, seven S_i of B's, Q_i = T_i*S_i,
 *     U1..U3 and the four quadrants of C from the Q_i;
 *   - below the cutoff the classical algorithm is used (Section 5.4.1, first
 *     modification);
 *   - padding for n not a multiple of 2^levels (Section 3.1, last sentence of
 *     the paragraph that fixes n);
 *   - operation count F(n) = c_s n^w0 - 5 n^2 (Appendix A) -> the counters;
 *   - memory of a BFS step (seven S,T,Q triples, Section 3.3.1) and of a DFS
 *     step (one triple, Section 3.4.1) -> sw_oracle_peak_words.
 *
 * Readings of the paper taken here (all listed again in the design notes):
 *   R1. Appendix A as printed has three garbled tokens (S2 = B12 + B11,
 *       T3 = T2 - A12, T5 = A12 + T3).  With them C12 keeps an A11*B11 term
 *       that nothing cancels.  The standard Winograd form is used instead:
 *       S2 = B12 - B11, T3 = T2 - A11, T5 = A12 - T3.  The as-printed table
 *       is kept behind table=1 so a test can show it is not a product.
 *   R2. Appendix A's letters are used (T from A, S from B, Q0..Q6 0-based);
 *       the body of Section 3 swaps S and T and counts from 1.
 *   R3. Association is as printed: U1 = Q0+Q3, U2 = U1+Q4, U3 = U1+Q2,
 *       C11 = Q0+Q1, C12 = U3+Q5, C21 = U2-Q6, C22 = U2+Q2; the BFS/DFS
 *       choice changes memory and order of independent work, never a value.
 *   R4. Leaf: C_ij = sum_k A_ik*B_kj, k ascending, multiply then add, no FMA
 *       (compile with -ffp-contract=off); cost n0^3 mults + n0^3 - n0^2 adds,
 *       which is what c_s = (2 n0 + 4) / n0^(w0-2) implies.
 *   R5. Rounding: IEEE binary64, round to nearest even, no flush to zero.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int64_t leaf_mul;   /* scalar multiplications in classical leaves        */
    int64_t leaf_add;   /* scalar additions in classical leaves              */
    int64_t sw_add;     /* scalar additions/subtractions in the 15 matrix adds */
    int64_t leaf_calls; /* number of classical leaf products                 */
    int64_t sw_steps;   /* number of Strassen-Winograd steps taken           */
    int64_t mat_adds;   /* number of matrix additions (15 per step)          */
    int64_t mat_mults;  /* number of recursive matrix products (7 per step)  */
} sw_oracle_counters;

static sw_oracle_counters g_cnt;

void sw_oracle_reset_counters(void) { memset(&g_cnt, 0, sizeof g_cnt); }
void sw_oracle_get_counters(sw_oracle_counters *out) { *out = g_cnt; }

/* ---- classical product, the plain definition (Algorithm 1, Ensure) ------- */

/* C = A*B for n x n row-major views.  i-k-j loop order: every C_ij still
 * receives its n terms in ascending k, each a rounded product followed by a
 * rounded sum, so the value equals the textbook i-j-k triple loop.  The
 * avx2 clone only widens the j loop; FMA contraction stays off. */
__attribute__((target_clones("avx2", "default")))
static void classical(const double *A, int64_t lda, const double *B, int64_t ldb,
                      double *C, int64_t ldc, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        double *c = C + i * ldc;
        const double a0 = A[i * lda];
        const double *b0 = B;
        for (int64_t j = 0; j < n; ++j) c[j] = a0 * b0[j];
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

void sw_oracle_naive(int64_t n, const double *A, const double *B, double *C)
{
    if (n <= 0) return;
    classical(A, n, B, n, C, n, n);
}

/* One entry of the product by its definition, ascending k, in long double so
 * that it can referee fp64 results at large n. */
double sw_oracle_entry(int64_t n, const double *A_row_i, const double *B_col_j, int64_t stride_b)
{
    long double s = 0.0L;
    for (int64_t k = 0; k < n; ++k)
        s += (long double)A_row_i[k] * (long double)B_col_j[k * stride_b];
    return (double)s;
}

/* Strips of the product by its definition (Algorithm 1, Ensure), for checking
 * a large result where the whole product is out of reach: every entry gets its
 * n terms in ascending k, each a rounded product followed by a rounded sum,
 * exactly as in `classical` above, so a strip equals the same rows (columns)
 * of sw_oracle_naive bit for bit.
 *
 * Row strip:    C_rows (r x n) = A_rows (r x n) * B (n x n), where A_rows holds
 *               r chosen rows of A one after the other (leading dimension n).
 * Column strip: C_cols (n x c) = A (n x n) * B_cols (n x c), where B_cols holds
 *               c chosen columns of B side by side (leading dimension c).
 * All matrices dense, row-major, host memory, caller-owned. */
__attribute__((target_clones("avx2", "default")))
static void strip(const double *A, int64_t lda, const double *B, int64_t ldb,
                  double *C, int64_t ldc, int64_t rows, int64_t cols, int64_t n)
{
    for (int64_t i = 0; i < rows; ++i) {
        double *c = C + i * ldc;
        const double a0 = A[i * lda];
        for (int64_t j = 0; j < cols; ++j) c[j] = a0 * B[j];
        for (int64_t k = 1; k < n; ++k) {
            const double a = A[i * lda + k];
            const double *b = B + k * ldb;
            for (int64_t j = 0; j < cols; ++j) c[j] = c[j] + a * b[j];
        }
    }
}

void sw_oracle_row_strip(int64_t n, int64_t r, const double *A_rows, const double *B, double *C_rows)
{
    if (n <= 0 || r <= 0) return;
    strip(A_rows, n, B, n, C_rows, n, r, n, n);
}

void sw_oracle_col_strip(int64_t n, int64_t c, const double *A, const double *B_cols, double *C_cols)
{
    if (n <= 0 || c <= 0) return;
    strip(A, n, B_cols, c, C_cols, c, n, c, n);
}

/* ---- matrix add / subtract on row-major views ---------------------------- */

__attribute__((target_clones("avx2", "default")))
static void madd(double *Z, int64_t ldz, const double *X, int64_t ldx,
                 const double *Y, int64_t ldy, int64_t h, int sign)
{
    for (int64_t i = 0; i < h; ++i)
        for (int64_t j = 0; j < h; ++j)
            Z[i * ldz + j] = sign > 0 ? X[i * ldx + j] + Y[i * ldy + j]
                                      : X[i * ldx + j] - Y[i * ldy + j];
    g_cnt.sw_add += h * h;
    g_cnt.mat_adds += 1;
}

/* ---- the recursion ------------------------------------------------------- */

static int sw_rec(const double *A, int64_t lda, const double *B, int64_t ldb,
                  double *C, int64_t ldc, int64_t n, int levels, int table)
{
    if (levels == 0) {
        classical(A, lda, B, ldb, C, ldc, n);
        return 0;
    }
    const int64_t h = n / 2;
    const double *A11 = A, *A12 = A + h, *A21 = A + h * lda, *A22 = A + h * lda + h;
    const double *B11 = B, *B12 = B + h, *B21 = B + h * ldb, *B22 = B + h * ldb + h;
    double *C11 = C, *C12 = C + h, *C21 = C + h * ldc, *C22 = C + h * ldc + h;

    /* T2..T5, S2,S3,S4,S6, Q0..Q6, U1..U3: 18 h x h temporaries */
    const size_t hh = (size_t)h * (size_t)h;
    double *buf = (double *)malloc(18 * hh * sizeof(double));
    if (!buf) return -1;
    double *T2 = buf, *T3 = T2 + hh, *T4 = T3 + hh, *T5 = T4 + hh;
    double *S2 = T5 + hh, *S3 = S2 + hh, *S4 = S3 + hh, *S6 = S4 + hh;
    double *Q[7];
    for (int i = 0; i < 7; ++i) Q[i] = S6 + hh + (size_t)i * hh;
    double *U1 = Q[6] + hh, *U2 = U1 + hh, *U3 = U2 + hh;

    /* Appendix A, first column (T from A) and second column (S from B) */
    madd(T2, h, A21, lda, A22, lda, h, +1);                 /* T2 = A21 + A22 */
    if (table == 0) madd(T3, h, T2, h, A11, lda, h, -1);    /* T3 = T2 - A11  */
    else            madd(T3, h, T2, h, A12, lda, h, -1);    /* as printed     */
    madd(T4, h, A11, lda, A21, lda, h, -1);                 /* T4 = A11 - A21 */
    if (table == 0) madd(T5, h, A12, lda, T3, h, h, -1);    /* T5 = A12 - T3  */
    else            madd(T5, h, A12, lda, T3, h, h, +1);    /* as printed     */
    if (table == 0) madd(S2, h, B12, ldb, B11, ldb, h, -1); /* S2 = B12 - B11 */
    else            madd(S2, h, B12, ldb, B11, ldb, h, +1); /* as printed     */
    madd(S3, h, B22, ldb, S2, h, h, -1);                    /* S3 = B22 - S2  */
    madd(S4, h, B22, ldb, B12, ldb, h, -1);                 /* S4 = B22 - B12 */
    madd(S6, h, S3, h, B21, ldb, h, -1);                    /* S6 = S3 - B21  */

    /* third column: Q_i = T_i * S_i; T0,T1,T6 and S0,S1,S5 are plain quadrants */
    const double *T[7] = {A11, A12, T2, T3, T4, T5, A22};
    const int64_t ldt[7] = {lda, lda, h, h, h, h, lda};
    const double *S[7] = {B11, B21, S2, S3, S4, B22, S6};
    const int64_t lds[7] = {ldb, ldb, h, h, h, ldb, h};
    int rc = 0;
    for (int i = 0; i < 7 && rc == 0; ++i) {
        rc = sw_rec(T[i], ldt[i], S[i], lds[i], Q[i], h, h, levels - 1, table);
        g_cnt.mat_mults += 1;
    }

    /* fourth column */
    if (rc == 0) {
        madd(U1, h, Q[0], h, Q[3], h, h, +1);   /* U1  = Q0 + Q3 */
        madd(U2, h, U1, h, Q[4], h, h, +1);     /* U2  = U1 + Q4 */
        madd(U3, h, U1, h, Q[2], h, h, +1);     /* U3  = U1 + Q2 */
        madd(C11, ldc, Q[0], h, Q[1], h, h, +1);/* C11 = Q0 + Q1 */
        madd(C12, ldc, U3, h, Q[5], h, h, +1);  /* C12 = U3 + Q5 */
        madd(C21, ldc, U2, h, Q[6], h, h, -1);  /* C21 = U2 - Q6 */
        madd(C22, ldc, U2, h, Q[2], h, h, +1);  /* C22 = U2 + Q2 */
        g_cnt.sw_steps += 1;
    }
    free(buf);
    return rc;
}

/* C = A*B with `levels` Strassen-Winograd steps above a classical leaf.
 * A, B, C: n x n, row-major, dense (ld = n), host memory, caller-owned.
 * n not divisible by 2^levels: embed in the next multiple with zeros, run,
 * crop.  table = 0: corrected Appendix A (reading R1); table = 1: as printed.
 * Returns 0, -1 on allocation failure, -2 on bad arguments. */
int sw_oracle_gemm_table(int64_t n, const double *A, const double *B, double *C,
                         int levels, int table)
{
    if (n < 0 || levels < 0 || levels > 30 || (n > 0 && (!A || !B || !C))) return -2;
    if (n == 0) return 0;
    const int64_t q = (int64_t)1 << levels;
    if (q > n) return -2;
    const int64_t np = (n + q - 1) / q * q;
    if (np == n) return sw_rec(A, n, B, n, C, n, n, levels, table);

    const size_t sz = (size_t)np * (size_t)np;
    double *Ap = (double *)calloc(3 * sz, sizeof(double));
    if (!Ap) return -1;
    double *Bp = Ap + sz, *Cp = Bp + sz;
    for (int64_t i = 0; i < n; ++i) {
        memcpy(Ap + i * np, A + i * n, (size_t)n * sizeof(double));
        memcpy(Bp + i * np, B + i * n, (size_t)n * sizeof(double));
    }
    int rc = sw_rec(Ap, np, Bp, np, Cp, np, np, levels, table);
    if (rc == 0)
        for (int64_t i = 0; i < n; ++i)
            memcpy(C + i * n, Cp + i * np, (size_t)n * sizeof(double));
    free(Ap);
    return rc;
}

int sw_oracle_gemm(int64_t n, const double *A, const double *B, double *C, int levels)
{
    return sw_oracle_gemm_table(n, A, B, C, levels, 0);
}

/* ---- dynamic peeling (Section 3.1 names it beside padding) ---------------- */

/* The same recursion for any n >= 2^levels without padding: whenever the size
 * at some level is odd, the last row and column are peeled off, the step is
 * taken on the leading even block, and the peeled parts are finished by their
 * definitions:
 *   C11 += a12 * b21            (column of A times row of B, one term more)
 *   c12  = [A11 a12] * [b12; b22]   (last column of C, rows above the last)
 *   [c21 c22] = [a21 a22] * B       (last row of C)
 * each sum in ascending k, multiply then add.  The children of the even block
 * have half its size and may be odd again ("dynamic": decided level by level). */
static int sw_rec_peel(const double *A, int64_t lda, const double *B, int64_t ldb,
                       double *C, int64_t ldc, int64_t n, int levels)
{
    if (levels == 0) {
        classical(A, lda, B, ldb, C, ldc, n);
        return 0;
    }
    if (n % 2 == 1) {
        const int64_t m = n - 1;
        int rc = sw_rec_peel(A, lda, B, ldb, C, ldc, m, levels);   /* C11 = A11 * B11 */
        if (rc != 0) return rc;
        for (int64_t i = 0; i < m; ++i) {
            const double a = A[i * lda + m];
            for (int64_t j = 0; j < m; ++j) C[i * ldc + j] = C[i * ldc + j] + a * B[m * ldb + j];
            double s = A[i * lda] * B[m];                           /* column m of B */
            for (int64_t k = 1; k < n; ++k) s = s + A[i * lda + k] * B[k * ldb + m];
            C[i * ldc + m] = s;
        }
        for (int64_t j = 0; j < n; ++j) {
            double s = A[m * lda] * B[j];
            for (int64_t k = 1; k < n; ++k) s = s + A[m * lda + k] * B[k * ldb + j];
            C[m * ldc + j] = s;
        }
        return 0;
    }
    const int64_t h = n / 2;
    const double *A11 = A, *A12 = A + h, *A21 = A + h * lda, *A22 = A + h * lda + h;
    const double *B11 = B, *B12 = B + h, *B21 = B + h * ldb, *B22 = B + h * ldb + h;
    double *C11 = C, *C12 = C + h, *C21 = C + h * ldc, *C22 = C + h * ldc + h;
    const size_t hh = (size_t)h * (size_t)h;
    double *buf = (double *)malloc(18 * hh * sizeof(double));
    if (!buf) return -1;
    double *T2 = buf, *T3 = T2 + hh, *T4 = T3 + hh, *T5 = T4 + hh;
    double *S2 = T5 + hh, *S3 = S2 + hh, *S4 = S3 + hh, *S6 = S4 + hh;
    double *Q[7];
    for (int i = 0; i < 7; ++i) Q[i] = S6 + hh + (size_t)i * hh;
    double *U1 = Q[6] + hh, *U2 = U1 + hh, *U3 = U2 + hh;
    /* Appendix A with the corrected tokens, as in sw_rec */
    madd(T2, h, A21, lda, A22, lda, h, +1);
    madd(T3, h, T2, h, A11, lda, h, -1);
    madd(T4, h, A11, lda, A21, lda, h, -1);
    madd(T5, h, A12, lda, T3, h, h, -1);
    madd(S2, h, B12, ldb, B11, ldb, h, -1);
    madd(S3, h, B22, ldb, S2, h, h, -1);
    madd(S4, h, B22, ldb, B12, ldb, h, -1);
    madd(S6, h, S3, h, B21, ldb, h, -1);
    const double *T[7] = {A11, A12, T2, T3, T4, T5, A22};
    const int64_t ldt[7] = {lda, lda, h, h, h, h, lda};
    const double *S[7] = {B11, B21, S2, S3, S4, B22, S6};
    const int64_t lds[7] = {ldb, ldb, h, h, h, ldb, h};
    int rc = 0;
    for (int i = 0; i < 7 && rc == 0; ++i) rc = sw_rec_peel(T[i], ldt[i], S[i], lds[i], Q[i], h, h, levels - 1);
    if (rc == 0) {
        madd(U1, h, Q[0], h, Q[3], h, h, +1);
        madd(U2, h, U1, h, Q[4], h, h, +1);
        madd(U3, h, U1, h, Q[2], h, h, +1);
        madd(C11, ldc, Q[0], h, Q[1], h, h, +1);
        madd(C12, ldc, U3, h, Q[5], h, h, +1);
        madd(C21, ldc, U2, h, Q[6], h, h, -1);
        madd(C22, ldc, U2, h, Q[2], h, h, +1);
    }
    free(buf);
    return rc;
}

/* C = A*B with `levels` Strassen-Winograd steps and peeling at every level whose
 * size is odd; n >= 2^levels.  Returns 0, -1 on allocation failure, -2 on bad arguments. */
int sw_oracle_gemm_peel(int64_t n, const double *A, const double *B, double *C, int levels)
{
    if (n < 0 || levels < 0 || levels > 30 || (n > 0 && (!A || !B || !C))) return -2;
    if (n == 0) return 0;
    if (((int64_t)1 << levels) > n) return -2;
    return sw_rec_peel(A, n, B, n, C, n, n, levels);
}

/* ---- memory of a traversal (Sections 3.3.1 and 3.4.1) --------------------- */

/* Peak number of words of S/T/Q storage, beyond A, B and C, that a traversal
 * with the given step order holds at once, obtained by walking the tree:
 *   BFS step on a node of size n: the seven (S,T,Q) triples of size n/2 are
 *     all allocated, and the seven subproblems are in flight together, so
 *     their own needs add up;
 *   DFS step: one triple at a time, subproblems in sequence, so only the
 *     largest child's need is added.
 * schedule: `levels` characters 'B' or 'D', top level first.
 * Returns the word count, or -1 on a bad argument. */
static int64_t peak_rec(int64_t n, const char *s)
{
    if (*s == '\0') return 0;
    const int64_t h = n / 2;
    const int64_t child = peak_rec(h, s + 1);
    if (*s == 'B') return 7 * 3 * h * h + 7 * child;
    return 3 * h * h + child;
}

int64_t sw_oracle_peak_words(int64_t n, int levels, const char *schedule)
{
    if (n <= 0 || levels < 0 || !schedule || (int)strlen(schedule) != levels) return -1;
    for (int i = 0; i < levels; ++i)
        if (schedule[i] != 'B' && schedule[i] != 'D') return -1;
    if (n % ((int64_t)1 << levels)) return -1;
    return peak_rec(n, schedule);
}
