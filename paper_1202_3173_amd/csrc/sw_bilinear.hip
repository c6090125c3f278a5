// Other recursive algorithms on the same machinery (Section 6.6): any way to multiply 2 x 2 block matrices with
// q block products -- q combinations of A's quadrants, q of B's, the quadrants of C as combinations of the q
// products -- run through the same BFS steps (all q subproblems of every parent in flight, 3q half-size
// buffers per parent), DFS steps (one subproblem after the other, 3 buffers per parent) and batched leaf
// products as the Strassen-Winograd path.  Two schemes are tabulated: Strassen's original algorithm (7
// products, 18 additions) and the classical algorithm written recursively (8 products, 4 additions;
// Section 6.6.1).  Every combination is summed left to right, so BFS and DFS steps give the same bits.
//
// The kernels here are generic over the coefficient table and move more data than the specialised
// Strassen-Winograd kernels; they are the comparison algorithms, not the headline path.
#include <string.h>

#include <string>

#include "sw_internal.h"

namespace sw {
namespace {

constexpr int NT = 256;
constexpr int MAXQ = 8;

struct Scheme {
    int q;
    int8_t u[MAXQ][4];   // product i takes sum_k u[i][k] * A_k, quadrants k = 11, 12, 21, 22
    int8_t v[MAXQ][4];   // ... times sum_k v[i][k] * B_k
    int8_t w[4][MAXQ];   // C_c = sum_i w[c][i] * M_i
};

// Strassen's algorithm:
//   M1 = (A11 + A22)(B11 + B22)   M2 = (A21 + A22) B11     M3 = A11 (B12 - B22)      M4 = A22 (B21 - B11)
//   M5 = (A11 + A12) B22          M6 = (A21 - A11)(B11 + B12)                        M7 = (A12 - A22)(B21 + B22)
//   C11 = M1 + M4 - M5 + M7       C12 = M3 + M5            C21 = M2 + M4             C22 = M1 - M2 + M3 + M6
const Scheme kStrassen = {
    7,
    {{1, 0, 0, 1}, {0, 0, 1, 1}, {1, 0, 0, 0}, {0, 0, 0, 1}, {1, 1, 0, 0}, {-1, 0, 1, 0}, {0, 1, 0, -1}},
    {{1, 0, 0, 1}, {1, 0, 0, 0}, {0, 1, 0, -1}, {-1, 0, 1, 0}, {0, 0, 0, 1}, {1, 1, 0, 0}, {0, 0, 1, 1}},
    {{1, 0, 0, 1, -1, 0, 1}, {0, 0, 1, 0, 1, 0, 0}, {0, 1, 0, 1, 0, 0, 0}, {1, -1, 1, 0, 0, 1, 0}},
};

// The classical algorithm: C_ij = A_i1 B_1j + A_i2 B_2j, products numbered C11's two, C12's, C21's, C22's.
const Scheme kClassical = {
    8,
    {{1, 0, 0, 0}, {0, 1, 0, 0}, {1, 0, 0, 0}, {0, 1, 0, 0}, {0, 0, 1, 0}, {0, 0, 0, 1}, {0, 0, 1, 0}, {0, 0, 0, 1}},
    {{1, 0, 0, 0}, {0, 0, 1, 0}, {0, 1, 0, 0}, {0, 0, 0, 1}, {1, 0, 0, 0}, {0, 0, 1, 0}, {0, 1, 0, 0}, {0, 0, 0, 1}},
    {{1, 1, 0, 0, 0, 0, 0, 0}, {0, 0, 1, 1, 0, 0, 0, 0}, {0, 0, 0, 0, 1, 1, 0, 0}, {0, 0, 0, 0, 0, 0, 1, 1}},
};

const Scheme* scheme_of(int id)
{
    if (id == SW_SCHEME_STRASSEN) return &kStrassen;
    if (id == SW_SCHEME_CLASSICAL) return &kClassical;
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

struct Rows { int n; int8_t c[MAXQ][4]; };     // n combinations of the four quadrants
struct Cols { int q; int8_t c[4][MAXQ]; };     // the four quadrants as combinations of q products

// Block b of a launch covers NT * VEC consecutive elements (row-major over an h x h matrix) of matrix b / bpm.
#define BIL_DECODE()                                                        \
    const int64_t p = b / bpm;                                              \
    const int64_t t = (b - p * bpm) * NT + threadIdx.x;                     \
    const int64_t hv = h / VEC;                                             \
    if (t >= h * hv) continue;                                              \
    const int64_t r = t / hv, cc = (t - r * hv) * VEC

// children[rows.n * p + i] = sum_k rows.c[i][k] * quadrant k of parent p   (h x h each)
template <int VEC>
__global__ __launch_bounds__(NT) void bil_pre_kernel(const double* parent, int64_t pld, int64_t pstride, int64_t h,
                                                     double* child, int64_t cld, int64_t cstride, Rows rows, int64_t bpm,
                                                     int64_t nblocks)
{
    using P = Pack<VEC>;
    for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        BIL_DECODE();
        const double* src = parent + p * pstride + r * pld + cc;
        P x[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            bool used = false;
            for (int i = 0; i < rows.n; ++i) used = used || rows.c[i][k] != 0;
            if (used) x[k] = P::ld(src + (k >> 1) * h * pld + (k & 1) * h);
        }
        for (int i = 0; i < rows.n; ++i) {
            P acc{};
            bool started = false;
#pragma unroll
            for (int k = 0; k < 4; ++k) term(acc, started, rows.c[i][k], x[k]);
            acc.st(child + (p * rows.n + i) * cstride + r * cld + cc);
        }
    }
}

// quadrant c of parent p = sum_i cols.c[c][i] * prod[cols.q * p + i]
template <int VEC>
__global__ __launch_bounds__(NT) void bil_post_kernel(const double* prod, int64_t qld, int64_t qstride, int64_t h,
                                                      double* parent, int64_t pld, int64_t pstride, Cols cols, int64_t bpm,
                                                      int64_t nblocks)
{
    using P = Pack<VEC>;
    for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        BIL_DECODE();
        P x[MAXQ];
#pragma unroll
        for (int i = 0; i < MAXQ; ++i)
            if (i < cols.q) x[i] = P::ld(prod + (p * cols.q + i) * qstride + r * qld + cc);
        double* dst = parent + p * pstride + r * pld + cc;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            P acc{};
            bool started = false;
#pragma unroll
            for (int i = 0; i < MAXQ; ++i)
                if (i < cols.q) term(acc, started, cols.c[c][i], x[i]);
            acc.st(dst + (c >> 1) * h * pld + (c & 1) * h);
        }
    }
}

// One product of a DFS step folded into C: for every quadrant c with w[c] != 0,
// C_c = w[c] * Q when it is the quadrant's first product, else C_c = C_c + w[c] * Q.
struct Fold { int8_t w[4]; int8_t first[4]; };

template <int VEC>
__global__ __launch_bounds__(NT) void bil_fold_kernel(const double* prod, int64_t qld, int64_t qstride, int64_t h,
                                                      double* parent, int64_t pld, int64_t pstride, Fold f, int64_t bpm,
                                                      int64_t nblocks)
{
    using P = Pack<VEC>;
    for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        BIL_DECODE();
        const P x = P::ld(prod + p * qstride + r * qld + cc);
        double* dst = parent + p * pstride + r * pld + cc;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (f.w[c] == 0) continue;
            double* d = dst + (c >> 1) * h * pld + (c & 1) * h;
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
    if (v2) hipLaunchKernelGGL((bil_pre_kernel<2>), dim3(g.blocks), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, h,
                               child.p, child.ld, child.stride, rows, g.bpm, g.nblocks);
    else    hipLaunchKernelGGL((bil_pre_kernel<1>), dim3(g.blocks), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, h,
                               child.p, child.ld, child.stride, rows, g.bpm, g.nblocks);
    return hipGetLastError();
}

hipError_t launch_post(Mat prod, int64_t live, int64_t h, Mat parent, const Cols& cols, hipStream_t s)
{
    if (live == 0 || h == 0) return hipSuccess;
    const bool v2 = h % 2 == 0 && vec2(parent) && vec2(prod);
    const Grid g = grid_for(live, h, v2 ? 2 : 1);
    if (v2) hipLaunchKernelGGL((bil_post_kernel<2>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, cols, g.bpm, g.nblocks);
    else    hipLaunchKernelGGL((bil_post_kernel<1>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, cols, g.bpm, g.nblocks);
    return hipGetLastError();
}

hipError_t launch_fold(Mat prod, int64_t live, int64_t h, Mat parent, const Fold& f, hipStream_t s)
{
    if (live == 0 || h == 0) return hipSuccess;
    const bool v2 = h % 2 == 0 && vec2(parent) && vec2(prod);
    const Grid g = grid_for(live, h, v2 ? 2 : 1);
    if (v2) hipLaunchKernelGGL((bil_fold_kernel<2>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, f, g.bpm, g.nblocks);
    else    hipLaunchKernelGGL((bil_fold_kernel<1>), dim3(g.blocks), dim3(NT), 0, s, prod.p, prod.ld, prod.stride, h,
                               parent.p, parent.ld, parent.stride, f, g.bpm, g.nblocks);
    return hipGetLastError();
}

// ---- workspace and the walk ---------------------------------------------------------------------------------------

// BFS step: T, S, Q for all q children of every parent; DFS step: one T, S, Q per parent.
int64_t need_bytes(const Scheme* sc, int64_t n, const char* sched, int64_t live)
{
    if (*sched == '\0') return 0;
    const int64_t h = n / 2;
    const int64_t e = ws_mat_elems(h) * (int64_t)sizeof(double);
    if (*sched == 'B') return 3 * sc->q * live * e + need_bytes(sc, h, sched + 1, sc->q * live);
    return 3 * live * e + need_bytes(sc, h, sched + 1, live);
}

int64_t total_bytes(const Scheme* sc, int64_t n, int levels, const char* sched)
{
    if (n == 0) return 0;
    const int64_t np = padded_n(n, levels);
    int64_t bytes = need_bytes(sc, np, sched, 1);
    if (np != n) bytes += 3 * ws_mat_elems(np) * (int64_t)sizeof(double);
    return bytes;
}

// a combination that is one quadrant taken as it is needs no copy: returns its index, else -1
int plain_quadrant(const int8_t c[4])
{
    int k = -1;
    for (int j = 0; j < 4; ++j) {
        if (c[j] == 0) continue;
        if (c[j] != 1 || k >= 0) return -1;
        k = j;
    }
    return k;
}

struct Walk {
    const Scheme* sc;
    char* ws;
    int64_t used = 0;
    const char* sched;
    int levels;
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
        if (level == levels) {
            op(SW_CLASS_LEAF, 2.0 * live * (double)n * n * n, [&] { return launch_leaf_gemm(n, live, A, B, C, st); });
            return;
        }
        const int q = sc->q;
        const int64_t h = n / 2, e = ws_mat_elems(h), mark = used;
        const double hb = 8.0 * live * (double)h * h;          // bytes of one half-size matrix per parent
        if (sched[level] == 'B') {
            Mat T = ws_mat(take(q * live * e), h), S = ws_mat(take(q * live * e), h), Q = ws_mat(take(q * live * e), h);
            Rows ra{q, {}}, rb{q, {}};
            memcpy(ra.c, sc->u, sizeof ra.c);
            memcpy(rb.c, sc->v, sizeof rb.c);
            Cols cw{q, {}};
            memcpy(cw.c, sc->w, sizeof cw.c);
            op(SW_CLASS_PRE_ADD, hb * (4 + q), [&] { return launch_pre(A, live, h, T, ra, st); });
            op(SW_CLASS_PRE_ADD, hb * (4 + q), [&] { return launch_pre(B, live, h, S, rb, st); });
            mul(T, S, Q, h, level + 1, q * live);
            op(SW_CLASS_POST_ADD, hb * (q + 4), [&] { return launch_post(Q, live, h, C, cw, st); });
        } else {
            Mat T = ws_mat(take(live * e), h), S = ws_mat(take(live * e), h), Q = ws_mat(take(live * e), h);
            bool begun[4] = {false, false, false, false};
            for (int i = 0; i < q; ++i) {
                Mat ta = T, sb = S;
                const int ka = plain_quadrant(sc->u[i]), kb = plain_quadrant(sc->v[i]);
                if (ka >= 0) ta = quad(A, h, ka >> 1, ka & 1);
                else {
                    Rows r{1, {}};
                    memcpy(r.c[0], sc->u[i], 4);
                    op(SW_CLASS_DFS_ADD, hb * (nonzero(sc->u[i], 4) + 1), [&] { return launch_pre(A, live, h, T, r, st); });
                }
                if (kb >= 0) sb = quad(B, h, kb >> 1, kb & 1);
                else {
                    Rows r{1, {}};
                    memcpy(r.c[0], sc->v[i], 4);
                    op(SW_CLASS_DFS_ADD, hb * (nonzero(sc->v[i], 4) + 1), [&] { return launch_pre(B, live, h, S, r, st); });
                }
                Fold f{};
                int targets = 0, only = -1;
                for (int c = 0; c < 4; ++c) {
                    f.w[c] = sc->w[c][i];
                    f.first[c] = !begun[c];
                    if (f.w[c]) { ++targets; only = c; }
                }
                if (level + 1 == levels && targets == 1 && f.w[only] == 1) {
                    // a leaf product that goes to one quadrant with coefficient +1: the product kernel writes
                    // or accumulates in place (C_c + M_i is formed in the same order either way)
                    const Mat cq = quad(C, h, only >> 1, only & 1);
                    const bool acc = begun[only];
                    op(SW_CLASS_LEAF, 2.0 * live * (double)h * h * h, [&] { return launch_gemm(h, h, h, live, ta, sb, cq, acc, st); });
                } else {
                    mul(ta, sb, Q, h, level + 1, live);
                    double moved = 1;
                    for (int c = 0; c < 4; ++c) if (f.w[c]) moved += f.first[c] ? 1 : 2;
                    op(SW_CLASS_DFS_ADD, hb * moved, [&] { return launch_fold(Q, live, h, C, f, st); });
                }
                for (int c = 0; c < 4; ++c) begun[c] = begun[c] || f.w[c] != 0;
            }
        }
        used = mark;
    }
};

int plan_order(const Scheme* sc, int64_t n, int levels, int64_t budget, char* out)
{
    // most BFS steps, then least memory (which puts the DFS steps first)
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
        const int64_t need = total_bytes(sc, n, levels, cand);
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

}  // namespace
}  // namespace sw

using namespace sw;

extern "C" {

int64_t sw_plan_memory_bilinear(int64_t n, int levels, const char* schedule, int scheme)
{
    if (scheme == SW_SCHEME_WINOGRAD) return sw_plan_memory(n, levels, schedule);
    const Scheme* sc = scheme_of(scheme);
    if (!sc) { set_error("unknown scheme %d", scheme); return SW_EINVAL; }
    int rc = check_shape(n, levels);
    if (rc != SW_OK) return rc;
    std::string s = (schedule && *schedule) ? std::string(schedule) : std::string((size_t)levels, 'D');
    if (!schedule_ok(s.c_str(), levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", s.c_str(), levels);
        return SW_EINVAL;
    }
    return total_bytes(sc, n, levels, s.c_str());
}

int sw_gemm_bilinear(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule, int scheme)
{
    if (scheme == SW_SCHEME_WINOGRAD) return sw_gemm(n, A, B, C, levels, schedule);
    const Scheme* sc = scheme_of(scheme);
    if (!sc) { set_error("unknown scheme %d", scheme); return SW_EINVAL; }
    int rc = check_shape(n, levels);
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
        rc = plan_order(sc, n, levels, ws ? ws_bytes : 0, chosen);
        if (rc != SW_OK) return rc;
        schedule = chosen;
    } else if (!schedule_ok(schedule, levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", schedule, levels);
        return SW_EINVAL;
    }
    const int64_t need = total_bytes(sc, n, levels, schedule);
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
    // the leaf batch is q^(number of BFS steps); the product kernel takes at most 2^31 - 1 workgroups
    {
        double batch = 1;
        for (int i = 0; i < levels; ++i) if (schedule[i] == 'B') batch *= sc->q;
        const int64_t m = padded_n(n, levels) >> levels;
        const double tiles = (double)((m + 127) / 128) * (double)((m + 127) / 128);
        if (batch * tiles > 2147483647.0) { set_error("schedule %s puts too many leaf products into one launch", schedule); return SW_EINVAL; }
    }
    set_add_block_cap(0);
    Walk wk;
    wk.sc = sc;
    wk.ws = (char*)ws;
    wk.sched = schedule;
    wk.levels = levels;
    wk.st = st;
    wk.prof = profiler();
    Mat a{const_cast<double*>(A), n, 0}, b{const_cast<double*>(B), n, 0}, c{C, n, 0};
    const int64_t np = padded_n(n, levels);
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

double sw_flop_count_bilinear(int64_t n, int levels, int scheme)
{
    if (scheme == SW_SCHEME_WINOGRAD) return sw_flop_count(n, levels);
    const Scheme* sc = scheme_of(scheme);
    if (!sc || check_shape(n, levels) != SW_OK || n % ((int64_t)1 << levels)) return -1.0;
    int adds = 0;     // block additions per step: (terms - 1) of every combination
    for (int i = 0; i < sc->q; ++i) adds += Walk::nonzero(sc->u[i], 4) - 1 + Walk::nonzero(sc->v[i], 4) - 1;
    for (int c = 0; c < 4; ++c) adds += Walk::nonzero(sc->w[c], sc->q) - 1;
    const double m = (double)(n >> levels);
    double total = 0, live = 1, size = (double)n;
    for (int i = 0; i < levels; ++i) {
        size /= 2;
        total += live * adds * size * size;
        live *= sc->q;
    }
    return total + live * (2.0 * m * m * m - m * m);
}

}  // extern "C"
