// Other recursive algorithms on the same machinery (Section 6.6): any way to multiply n0 x n0 block matrices with
// q block products -- q combinations of A's blocks, q of B's, the blocks of C as combinations of the q products
// (Section 6.6.2; exponent w0 = log_n0 q) -- run through the same BFS steps (all q subproblems of every parent in
// flight, 3q buffers of 1/n0 the size per parent), DFS steps (one subproblem after the other, 3 buffers per
// parent) and batched leaf products as the Strassen-Winograd path.  Tabulated: Strassen's original algorithm
// (2 x 2 blocks, 7 products, 18 additions), the classical algorithm written recursively on 2 x 2 blocks (8
// products; Section 6.6.1) and on 3 x 3 blocks (27 products), and Laderman's algorithm for 3 x 3 blocks (23
// products).  The scheme may differ from level to level, so the radices 2 and 3 mix (94080 = 2^7 * 3 * 5 * 7^2).
// Every combination is summed left to right, so BFS and DFS steps give the same bits.
//
// The kernels here are generic over the coefficient table and move more data than the specialised
// Strassen-Winograd kernels; they are the comparison algorithms, not the headline path.
#include <string.h>

#include <string>

#include "sw_internal.h"

namespace sw {
namespace {

constexpr int NT = 256;
constexpr int MAXQ = 27;    // products per step
constexpr int MAXB = 9;     // blocks per operand (n0 * n0)

struct Scheme {
    int n0, q;
    int8_t u[MAXQ][MAXB];   // product i takes sum_k u[i][k] * A_k, blocks k numbered row-major (11, 12, ..)
    int8_t v[MAXQ][MAXB];   // ... times sum_k v[i][k] * B_k
    int8_t w[MAXB][MAXQ];   // C_c = sum_i w[c][i] * M_i
};

// A scheme is written down as its formulas: one string per product, "a-combination * b-combination", blocks
// as two digits (row, column) with a sign, and one string per block of C listing signed product numbers.
struct Formulas { int n0, q; const char* products[MAXQ]; const char* outputs[MAXB]; };

// Strassen's algorithm
const Formulas kStrassenText = {2, 7,
    {"+11+22 * +11+22", "+21+22 * +11", "+11 * +12-22", "+22 * +21-11", "+11+12 * +22", "+21-11 * +11+12", "+12-22 * +21+22"},
    {"+1+4-5+7", "+3+5", "+2+4", "+1-2+3+6"}};

// Laderman's algorithm for 3 x 3 blocks with 23 products
const Formulas kLadermanText = {3, 23,
    {"+11+12+13-21-22-32-33 * +22",            // m1
     "+11-21 * -12+22",                        // m2
     "+22 * -11+12+21-22-23-31+33",            // m3
     "-11+21+22 * +11-12+22",                  // m4
     "+21+22 * -11+12",                        // m5
     "+11 * +11",                              // m6
     "-11+31+32 * +11-13+23",                  // m7
     "-11+31 * +13-23",                        // m8
     "+31+32 * -11+13",                        // m9
     "+11+12+13-22-23-31-32 * +23",            // m10
     "+32 * -11+13+21-22-23-31+32",            // m11
     "-13+32+33 * +22+31-32",                  // m12
     "+13-33 * +22-32",                        // m13
     "+13 * +31",                              // m14
     "+32+33 * -31+32",                        // m15
     "-13+22+23 * +23+31-33",                  // m16
     "+13-23 * +23-33",                        // m17
     "+22+23 * -31+33",                        // m18
     "+12 * +21", "+23 * +32", "+21 * +13", "+31 * +12", "+33 * +33"},   // m19 .. m23
    {"+6+14+19", "+1+4+5+6+12+14+15", "+6+7+9+10+14+16+18",
     "+2+3+4+6+14+16+17", "+2+4+5+6+20", "+14+16+17+18+21",
     "+6+7+8+11+12+13+14", "+12+13+14+15+22", "+6+7+8+9+23"}};

// coefficient of a combination string: every "+rc" / "-rc" sets block (r, c); the order of the terms in the
// string does not matter (sums are always formed in block order, see `term` below)
void parse_blocks(const char* s, const char* end, int n0, int8_t* row)
{
    for (; s + 2 < end; ++s)
        if (*s == '+' || *s == '-') {
            row[(s[1] - '1') * n0 + (s[2] - '1')] = (int8_t)(*s == '+' ? 1 : -1);
            s += 2;
        }
}

Scheme from_formulas(const Formulas& f)
{
    Scheme sc;
    memset(&sc, 0, sizeof sc);
    sc.n0 = f.n0;
    sc.q = f.q;
    for (int i = 0; i < f.q; ++i) {
        const char* p = f.products[i];
        const char* star = strchr(p, '*');
        parse_blocks(p, star, f.n0, sc.u[i]);
        parse_blocks(star + 1, p + strlen(p), f.n0, sc.v[i]);
    }
    for (int c = 0; c < f.n0 * f.n0; ++c) {
        const char* p = f.outputs[c];
        while (*p) {
            const int sign = *p == '+' ? 1 : -1;
            int k = 0;
            for (++p; *p >= '0' && *p <= '9'; ++p) k = 10 * k + (*p - '0');
            sc.w[c][k - 1] = (int8_t)sign;
        }
    }
    return sc;
}

// The classical algorithm on n0 x n0 blocks: C_ij = sum_k A_ik B_kj, product number (i n0 + j) n0 + k.
Scheme classical_scheme(int n0)
{
    Scheme sc;
    memset(&sc, 0, sizeof sc);
    sc.n0 = n0;
    sc.q = n0 * n0 * n0;
    for (int i = 0; i < n0; ++i)
        for (int j = 0; j < n0; ++j)
            for (int k = 0; k < n0; ++k) {
                const int p = (i * n0 + j) * n0 + k;
                sc.u[p][i * n0 + k] = 1;
                sc.v[p][k * n0 + j] = 1;
                sc.w[i * n0 + j][p] = 1;
            }
    return sc;
}

const Scheme* scheme_of(int id)
{
    static const Scheme strassen = from_formulas(kStrassenText), laderman = from_formulas(kLadermanText),
                        classical2 = classical_scheme(2), classical3 = classical_scheme(3);
    if (id == SW_SCHEME_STRASSEN) return &strassen;
    if (id == SW_SCHEME_CLASSICAL) return &classical2;
    if (id == SW_SCHEME_LADERMAN) return &laderman;
    if (id == SW_SCHEME_CLASSICAL3) return &classical3;
    return nullptr;
}

// ---- kernels ---------------------------------------------------------------------------------------------------

template <int VEC> struct Pack;
template <> struct Pack<1> {
    double x;
    __device__ static Pack ld(const double* p) { return Pack{*p}; }
    __device__ void st(double* p) const { *p = x; }
    __device__ Pack neg() const { return Pack{-x}; }
    __device__ Pack add(Pack o) const { return Pack{x + o.x}; }
    __device__ Pack sub(Pack o) const { return Pack{x - o.x}; }
};
template <> struct Pack<2> {
    double x, y;
    __device__ static Pack ld(const double* p) { const double2 v = *reinterpret_cast<const double2*>(p); return Pack{v.x, v.y}; }
    __device__ void st(double* p) const { *reinterpret_cast<double2*>(p) = make_double2(x, y); }
    __device__ Pack neg() const { return Pack{-x, -y}; }
    __device__ Pack add(Pack o) const { return Pack{x + o.x, y + o.y}; }
    __device__ Pack sub(Pack o) const { return Pack{x - o.x, y - o.y}; }
};

// acc (started) <- acc + c * x, left to right; a leading -1 is a negation
template <class P>
__device__ inline void term(P& acc, bool& started, int c, P x)
{
    if (c == 0) return;
    if (!started) acc = c > 0 ? x : x.neg();
    else acc = c > 0 ? acc.add(x) : acc.sub(x);
    started = true;
}

struct Rows { int n, n0; int8_t c[MAXQ][MAXB]; };     // n combinations of the n0 * n0 blocks
struct Cols { int q, n0; int8_t c[MAXB][MAXQ]; };     // the blocks as combinations of q products

// Block b of a launch covers NT * VEC consecutive elements (row-major over an h x h matrix) of matrix b / bpm.
#define BIL_DECODE()                                                        \
    const int64_t p = b / bpm;                                              \
    const int64_t t = (b - p * bpm) * NT + threadIdx.x;                     \
    const int64_t hv = h / VEC;                                             \
    if (t >= h * hv) continue;                                              \
    const int64_t r = t / hv, cc = (t - r * hv) * VEC

// children[rows.n * p + i] = sum_k rows.c[i][k] * block k of parent p   (h x h each; block k = (k / n0, k % n0))
// (the block count per side N0 is a template parameter so that every loop over blocks unrolls)
template <int VEC, int N0>
__global__ __launch_bounds__(NT) void bil_pre_kernel(const double* parent, int64_t pld, int64_t pstride, int64_t h,
                                                     double* child, int64_t cld, int64_t cstride, Rows rows, int64_t bpm,
                                                     int64_t nblocks)
{
    using P = Pack<VEC>;
    constexpr int NB = N0 * N0;
    for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        BIL_DECODE();
        const double* src = parent + p * pstride + r * pld + cc;
        P x[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            bool used = false;
            for (int i = 0; i < rows.n; ++i) used = used || rows.c[i][k] != 0;
            if (used) x[k] = P::ld(src + (k / N0) * h * pld + (k % N0) * h);
        }
        for (int i = 0; i < rows.n; ++i) {
            P acc{};
            bool started = false;
#pragma unroll
            for (int k = 0; k < NB; ++k) term(acc, started, rows.c[i][k], x[k]);
            acc.st(child + (p * rows.n + i) * cstride + r * cld + cc);
        }
    }
}

// block c of parent p = sum_i cols.c[c][i] * prod[cols.q * p + i]
template <int VEC, int N0>
__global__ __launch_bounds__(NT) void bil_post_kernel(const double* prod, int64_t qld, int64_t qstride, int64_t h,
                                                      double* parent, int64_t pld, int64_t pstride, Cols cols, int64_t bpm,
                                                      int64_t nblocks)
{
    using P = Pack<VEC>;
    constexpr int NB = N0 * N0, QMAX = N0 * N0 * N0;      // no scheme has more products than the classical one
    for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        BIL_DECODE();
        P x[QMAX];
#pragma unroll
        for (int i = 0; i < QMAX; ++i)
            if (i < cols.q) x[i] = P::ld(prod + (p * cols.q + i) * qstride + r * qld + cc);
        double* dst = parent + p * pstride + r * pld + cc;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            P acc{};
            bool started = false;
#pragma unroll
            for (int i = 0; i < QMAX; ++i)
                if (i < cols.q) term(acc, started, cols.c[c][i], x[i]);
            acc.st(dst + (c / N0) * h * pld + (c % N0) * h);
        }
    }
}

// One product of a DFS step folded into C: for every block c with w[c] != 0,
// C_c = w[c] * Q when it is the block's first product, else C_c = C_c + w[c] * Q.
struct Fold { int n0; int8_t w[MAXB]; int8_t first[MAXB]; };

template <int VEC, int N0>
__global__ __launch_bounds__(NT) void bil_fold_kernel(const double* prod, int64_t qld, int64_t qstride, int64_t h,
                                                      double* parent, int64_t pld, int64_t pstride, Fold f, int64_t bpm,
                                                      int64_t nblocks)
{
    using P = Pack<VEC>;
    constexpr int NB = N0 * N0;
    for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        BIL_DECODE();
        const P x = P::ld(prod + p * qstride + r * qld + cc);
        double* dst = parent + p * pstride + r * pld + cc;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            if (f.w[c] == 0) continue;
            double* d = dst + (c / N0) * h * pld + (c % N0) * h;
            P acc{};
            bool started = false;
            if (!f.first[c]) { acc = P::ld(d); started = true; }
            term(acc, started, f.w[c], x);
            acc.st(d);
        }
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool vec2(const Mat& m) { return aligned16(m.p) && m.ld % 2 == 0 && m.stride % 2 == 0; }

struct Grid { int64_t bpm, nblocks; unsigned blocks; };
inline Grid grid_for(int64_t live, int64_t h, int vec)
{
    Grid g;
    g.bpm = (h * (h / vec) + NT - 1) / NT;
    g.nblocks = g.bpm * live;
    g.blocks = (unsigned)(g.nblocks < (1 << 20) ? g.nblocks : (1 << 20));
    return g;
}

hipError_t launch_pre(Mat parent, int64_t live, int64_t h, Mat child, const Rows& rows, hipStream_t s)
{
    if (live == 0 || h == 0) return hipSuccess;
    const bool v2 = h % 2 == 0 && vec2(parent) && vec2(child);
    const Grid g = grid_for(live, h, v2 ? 2 : 1);
    if (v2 && rows.n0 == 2)      hipLaunchKernelGGL((bil_pre_kernel<2, 2>), dim3(g.blocks), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, h,
                               child.p, child.ld, child.stride, rows, g.bpm, g.nblocks);
    else if (v2)                hipLaunchKernelGGL((bil_pre_kernel<2, 3>), dim3(g.blocks), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, h,
                               child.p, child.ld, child.stride, rows, g.bpm, g.nblocks);
    else if (rows.n0 == 2)     hipLaunchKernelGGL((bil_pre_kernel<1, 2>), dim3(g.blocks), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, h,
                               child.p, child.ld, child.stride, rows, g.bpm, g.nblocks);
    else                        hipLaunchKernelGGL((bil_pre_kernel<1, 3>), dim3(g.blocks), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, h,
                               child.p, child.ld, child.stride, rows, g.bpm, g.nblocks);
    return hipGetLastError();
}

hipError_t launch_post(Mat prod, int64_t live, int64_t h, Mat parent, const Cols& cols, hipStream_t s)
{
    if (live == 0 || h == 0) return hipSuccess;
    const bool v2 = h % 2 == 0 && vec2(parent) && vec2(prod);
    const Grid g = grid_for(live, h, v2 ? 2 : 1);
    if (v2 && cols.n0 == 2)      hipLaunchKernelGGL((bil_post_kernel<2, 2>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, cols, g.bpm, g.nblocks);
    else if (v2)                hipLaunchKernelGGL((bil_post_kernel<2, 3>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, cols, g.bpm, g.nblocks);
    else if (cols.n0 == 2)     hipLaunchKernelGGL((bil_post_kernel<1, 2>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, cols, g.bpm, g.nblocks);
    else                        hipLaunchKernelGGL((bil_post_kernel<1, 3>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, cols, g.bpm, g.nblocks);
    return hipGetLastError();
}

hipError_t launch_fold(Mat prod, int64_t live, int64_t h, Mat parent, const Fold& f, hipStream_t s)
{
    if (live == 0 || h == 0) return hipSuccess;
    const bool v2 = h % 2 == 0 && vec2(parent) && vec2(prod);
    const Grid g = grid_for(live, h, v2 ? 2 : 1);
    if (v2 && f.n0 == 2)      hipLaunchKernelGGL((bil_fold_kernel<2, 2>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, f, g.bpm, g.nblocks);
    else if (v2)                hipLaunchKernelGGL((bil_fold_kernel<2, 3>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, f, g.bpm, g.nblocks);
    else if (f.n0 == 2)     hipLaunchKernelGGL((bil_fold_kernel<1, 2>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, f, g.bpm, g.nblocks);
    else                        hipLaunchKernelGGL((bil_fold_kernel<1, 3>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, f, g.bpm, g.nblocks);
    return hipGetLastError();
}

// ---- workspace and the walk ---------------------------------------------------------------------------------------

// the scheme of every level, top level first
struct Plan {
    const Scheme* at[SW_MAX_LEVELS];
    int levels;
    int64_t radix() const { int64_t r = 1; for (int i = 0; i < levels; ++i) r *= at[i]->n0; return r; }
};

inline int64_t padded_to(int64_t n, int64_t radix) { return (n + radix - 1) / radix * radix; }

// BFS step: T, S, Q for all q children of every parent; DFS step: one T, S, Q per parent.
int64_t need_bytes(const Plan& pl, int level, int64_t n, const char* sched, int64_t live)
{
    if (level == pl.levels) return 0;
    const Scheme* sc = pl.at[level];
    const int64_t h = n / sc->n0;
    const int64_t e = ws_mat_elems(h) * (int64_t)sizeof(double);
    if (sched[level] == 'B') return 3 * sc->q * live * e + need_bytes(pl, level + 1, h, sched, sc->q * live);
    return 3 * live * e + need_bytes(pl, level + 1, h, sched, live);
}

int64_t total_bytes(const Plan& pl, int64_t n, const char* sched)
{
    if (n == 0) return 0;
    const int64_t np = padded_to(n, pl.radix());
    int64_t bytes = need_bytes(pl, 0, np, sched, 1);
    if (np != n) bytes += 3 * ws_mat_elems(np) * (int64_t)sizeof(double);
    return bytes;
}

// a combination that is one block taken as it is needs no copy: returns its index, else -1
int plain_block(const int8_t* c, int nb)
{
    int k = -1;
    for (int j = 0; j < nb; ++j) {
        if (c[j] == 0) continue;
        if (c[j] != 1 || k >= 0) return -1;
        k = j;
    }
    return k;
}

// block (i, j) of a batch of matrices cut into n0 x n0 blocks of h x h; behind a row of every block lies more
// of the same row or the next row, except for the last block, which inherits the question from its parent
inline Mat block_of(const Mat& m, int64_t h, int n0, int k)
{
    const int i = k / n0, j = k % n0;
    return Mat{m.p + i * h * m.ld + j * h, m.ld, m.stride, m.padded || k + 1 < n0 * n0};
}

struct Walk {
    Plan pl;
    char* ws;
    int64_t used = 0;
    const char* sched;
    hipStream_t st;
    Profiler* prof;
    hipError_t err = hipSuccess;

    double* take(int64_t elems)
    {
        double* p = reinterpret_cast<double*>(ws + used);
        used += elems * (int64_t)sizeof(double);
        return p;
    }
    void note(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
    template <class F> void op(int cls, double work, F&& launch)
    {
        if (err != hipSuccess) return;
        ProfMark pm_;
        prof_begin(prof, st, cls, work, &pm_);
        note(launch());
        prof_end(prof, st, &pm_);
    }
    static int nonzero(const int8_t* c, int n) { int k = 0; for (int i = 0; i < n; ++i) k += c[i] != 0; return k; }

    void mul(Mat A, Mat B, Mat C, int64_t n, int level, int64_t live)
    {
        if (err != hipSuccess) return;
        if (level == pl.levels) {
            op(SW_CLASS_LEAF, 2.0 * live * (double)n * n * n, [&] { return launch_leaf_gemm(n, live, A, B, C, st); });
            return;
        }
        const Scheme* sc = pl.at[level];
        const int q = sc->q, n0 = sc->n0, nb = n0 * n0;
        const int64_t h = n / n0, e = ws_mat_elems(h), mark = used;
        const double hb = 8.0 * live * (double)h * h;          // bytes of one block per parent
        if (sched[level] == 'B') {
            Mat T = ws_mat(take(q * live * e), h), S = ws_mat(take(q * live * e), h), Q = ws_mat(take(q * live * e), h);
            Rows ra{q, n0, {}}, rb{q, n0, {}};
            memcpy(ra.c, sc->u, sizeof ra.c);
            memcpy(rb.c, sc->v, sizeof rb.c);
            Cols cw{q, n0, {}};
            memcpy(cw.c, sc->w, sizeof cw.c);
            op(SW_CLASS_PRE_ADD, hb * (nb + q), [&] { return launch_pre(A, live, h, T, ra, st); });
            op(SW_CLASS_PRE_ADD, hb * (nb + q), [&] { return launch_pre(B, live, h, S, rb, st); });
            mul(T, S, Q, h, level + 1, q * live);
            op(SW_CLASS_POST_ADD, hb * (q + nb), [&] { return launch_post(Q, live, h, C, cw, st); });
        } else {
            Mat T = ws_mat(take(live * e), h), S = ws_mat(take(live * e), h), Q = ws_mat(take(live * e), h);
            bool begun[MAXB] = {};
            for (int i = 0; i < q; ++i) {
                Mat ta = T, sb = S;
                const int ka = plain_block(sc->u[i], nb), kb = plain_block(sc->v[i], nb);
                if (ka >= 0) ta = block_of(A, h, n0, ka);
                else {
                    Rows r{1, n0, {}};
                    memcpy(r.c[0], sc->u[i], MAXB);
                    op(SW_CLASS_DFS_ADD, hb * (nonzero(sc->u[i], nb) + 1), [&] { return launch_pre(A, live, h, T, r, st); });
                }
                if (kb >= 0) sb = block_of(B, h, n0, kb);
                else {
                    Rows r{1, n0, {}};
                    memcpy(r.c[0], sc->v[i], MAXB);
                    op(SW_CLASS_DFS_ADD, hb * (nonzero(sc->v[i], nb) + 1), [&] { return launch_pre(B, live, h, S, r, st); });
                }
                Fold f{};
                f.n0 = n0;
                int targets = 0, only = -1;
                for (int c = 0; c < nb; ++c) {
                    f.w[c] = sc->w[c][i];
                    f.first[c] = !begun[c];
                    if (f.w[c]) { ++targets; only = c; }
                }
                if (level + 1 == pl.levels && targets == 1 && f.w[only] == 1) {
                    // a leaf product that goes to one block with coefficient +1: the product kernel writes
                    // or accumulates in place (C_c + M_i is formed in the same order either way)
                    const Mat cq = block_of(C, h, n0, only);
                    const bool acc = begun[only];
                    op(SW_CLASS_LEAF, 2.0 * live * (double)h * h * h, [&] { return launch_gemm(h, h, h, live, ta, sb, cq, acc, st); });
                } else {
                    mul(ta, sb, Q, h, level + 1, live);
                    double moved = 1;
                    for (int c = 0; c < nb; ++c) if (f.w[c]) moved += f.first[c] ? 1 : 2;
                    op(SW_CLASS_DFS_ADD, hb * moved, [&] { return launch_fold(Q, live, h, C, f, st); });
                }
                for (int c = 0; c < nb; ++c) begun[c] = begun[c] || f.w[c] != 0;
            }
        }
        used = mark;
    }
};

int plan_order(const Plan& pl, int64_t n, int64_t budget, char* out)
{
    // most BFS steps, then least memory (which puts the DFS steps first)
    const int levels = pl.levels;
    char cand[SW_MAX_LEVELS + 1];
    int best_b = -1;
    int64_t best_need = 0;
    for (uint32_t mask = 0; mask < (1u << levels); ++mask) {
        int nb = 0;
        for (int i = 0; i < levels; ++i) {
            cand[i] = ((mask >> i) & 1u) ? 'B' : 'D';
            nb += (mask >> i) & 1u;
        }
        cand[levels] = '\0';
        const int64_t need = total_bytes(pl, n, cand);
        if (need > budget) continue;
        if (nb > best_b || (nb == best_b && need < best_need)) {
            best_b = nb;
            best_need = need;
            memcpy(out, cand, (size_t)levels + 1);
        }
    }
    if (best_b < 0) {
        set_error("no step order for n = %lld, levels = %d fits a workspace of %lld bytes", (long long)n, levels, (long long)budget);
        return SW_ENOMEM;
    }
    return SW_OK;
}

// the schemes of a call: SW_OK and the plan, or SW_EINVAL with the error text set
int make_plan(int64_t n, int levels, const int* schemes, Plan* pl)
{
    if (n < 0 || levels < 0 || levels > SW_MAX_LEVELS || n > 200000 || (levels > 0 && !schemes)) {
        set_error("bad shape: n = %lld, levels = %d (0 <= levels <= %d, n <= 200000)", (long long)n, levels, SW_MAX_LEVELS);
        return SW_EINVAL;
    }
    pl->levels = levels;
    for (int i = 0; i < levels; ++i) {
        pl->at[i] = scheme_of(schemes[i]);
        if (!pl->at[i]) { set_error("unknown scheme %d at level %d (the Strassen-Winograd path is sw_gemm)", schemes[i], i); return SW_EINVAL; }
    }
    if (n > 0 && pl->radix() > n) {
        set_error("the levels cut n = %lld into %lld parts", (long long)n, (long long)pl->radix());
        return SW_EINVAL;
    }
    return SW_OK;
}

}  // namespace
}  // namespace sw

using namespace sw;

extern "C" {

int64_t sw_plan_memory_bilinear_levels(int64_t n, int levels, const char* schedule, const int* schemes)
{
    Plan pl;
    int rc = make_plan(n, levels, schemes, &pl);
    if (rc != SW_OK) return rc;
    std::string s = (schedule && *schedule) ? std::string(schedule) : std::string((size_t)levels, 'D');
    if (!schedule_ok(s.c_str(), levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", s.c_str(), levels);
        return SW_EINVAL;
    }
    return total_bytes(pl, n, s.c_str());
}

int64_t sw_plan_memory_bilinear(int64_t n, int levels, const char* schedule, int scheme)
{
    if (scheme == SW_SCHEME_WINOGRAD) return sw_plan_memory(n, levels, schedule);
    if (levels < 0 || levels > SW_MAX_LEVELS) { set_error("bad levels %d", levels); return SW_EINVAL; }
    int all[SW_MAX_LEVELS + 1];
    for (int i = 0; i < levels; ++i) all[i] = scheme;
    return sw_plan_memory_bilinear_levels(n, levels, schedule, all);
}

int sw_gemm_bilinear_levels(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule,
                            const int* schemes)
{
    Plan pl;
    int rc = make_plan(n, levels, schemes, &pl);
    if (rc != SW_OK) return rc;
    if (n == 0) return SW_OK;
    if (!A || !B || !C) { set_error("NULL matrix pointer"); return SW_EINVAL; }
    if (overlaps(C, n * n, A, n * n) || overlaps(C, n * n, B, n * n)) { set_error("C overlaps A or B"); return SW_EINVAL; }
    void* ws = nullptr;
    int64_t ws_bytes = 0;
    hipStream_t st = nullptr;
    library_state(&ws, &ws_bytes, &st);
    char chosen[SW_MAX_LEVELS + 1];
    if (!schedule || !*schedule) {
        rc = plan_order(pl, n, ws ? ws_bytes : 0, chosen);
        if (rc != SW_OK) return rc;
        schedule = chosen;
    } else if (!schedule_ok(schedule, levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", schedule, levels);
        return SW_EINVAL;
    }
    const int64_t need = total_bytes(pl, n, schedule);
    if (need > 0) {
        if (!ws || ws_bytes < need) {
            set_error("workspace of %lld bytes is too small: n = %lld, schedule %s needs %lld", (long long)(ws ? ws_bytes : 0),
                      (long long)n, schedule, (long long)need);
            return SW_ENOMEM;
        }
        if (overlaps((const double*)ws, need / 8, A, n * n) || overlaps((const double*)ws, need / 8, B, n * n) ||
            overlaps((const double*)ws, need / 8, C, n * n)) {
            set_error("workspace overlaps A, B or C");
            return SW_EINVAL;
        }
    }
    const int64_t np = padded_to(n, pl.radix());
    // the leaf batch is the product of q over the BFS steps; the product kernel takes at most 2^31 - 1 workgroups
    {
        double batch = 1;
        for (int i = 0; i < levels; ++i) if (schedule[i] == 'B') batch *= pl.at[i]->q;
        const int64_t m = np / pl.radix();
        const double tiles = (double)((m + 127) / 128) * (double)((m + 127) / 128);
        if (batch * tiles > 2147483647.0) { set_error("schedule %s puts too many leaf products into one launch", schedule); return SW_EINVAL; }
    }
    set_add_block_cap(0);
    Walk wk;
    wk.pl = pl;
    wk.ws = (char*)ws;
    wk.sched = schedule;
    wk.st = st;
    wk.prof = profiler();
    Mat a{const_cast<double*>(A), n, 0}, b{const_cast<double*>(B), n, 0}, c{C, n, 0};
    if (np != n) {
        const int64_t ld = ws_ld(np), e = ws_mat_elems(np);
        a = Mat{wk.take(e), ld, 0, ld > np};
        b = Mat{wk.take(e), ld, 0, ld > np};
        c = Mat{wk.take(e), ld, 0, ld > np};
        wk.op(SW_CLASS_PAD, 8.0 * (2.0 * n * n + 2.0 * np * np), [&] {
            hipError_t e1 = launch_pad_copy(A, n, n, n, a.p, ld, np, np, st);
            hipError_t e2 = launch_pad_copy(B, n, n, n, b.p, ld, np, np, st);
            return e1 != hipSuccess ? e1 : e2;
        });
    }
    wk.mul(a, b, c, np, 0, 1);
    if (np != n) wk.op(SW_CLASS_PAD, 8.0 * 2.0 * n * n, [&] { return launch_pad_copy(c.p, c.ld, np, np, C, n, n, n, st); });
    if (wk.err != hipSuccess) return hip_fail(wk.err, "kernel launch");
    return SW_OK;
}

int sw_gemm_bilinear(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule, int scheme)
{
    if (scheme == SW_SCHEME_WINOGRAD) return sw_gemm(n, A, B, C, levels, schedule);
    if (levels < 0 || levels > SW_MAX_LEVELS) { set_error("bad levels %d", levels); return SW_EINVAL; }
    int all[SW_MAX_LEVELS + 1];
    for (int i = 0; i < levels; ++i) all[i] = scheme;
    return sw_gemm_bilinear_levels(n, A, B, C, levels, schedule, all);
}

double sw_flop_count_bilinear(int64_t n, int levels, int scheme)
{
    if (scheme == SW_SCHEME_WINOGRAD) return sw_flop_count(n, levels);
    const Scheme* sc = scheme_of(scheme);
    if (!sc || n < 0 || levels < 0 || levels > SW_MAX_LEVELS) return -1.0;
    int64_t radix = 1;
    for (int i = 0; i < levels; ++i) radix *= sc->n0;
    if (n > 200000 || (n > 0 && radix > n) || n % radix) return -1.0;
    const int nb = sc->n0 * sc->n0;
    int adds = 0;     // block additions per step: (terms - 1) of every combination
    for (int i = 0; i < sc->q; ++i) adds += Walk::nonzero(sc->u[i], nb) - 1 + Walk::nonzero(sc->v[i], nb) - 1;
    for (int c = 0; c < nb; ++c) adds += Walk::nonzero(sc->w[c], sc->q) - 1;
    const double m = (double)(n / radix);
    double total = 0, live = 1, size = (double)n;
    for (int i = 0; i < levels; ++i) {
        size /= sc->n0;
        total += live * adds * size * size;
        live *= sc->q;
    }
    return total + live * (2.0 * m * m * m - m * m);
}

}  // extern "C"
