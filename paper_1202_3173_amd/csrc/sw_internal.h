// Internal declarations shared by the host planner, the executor and the kernel launchers.
// Nothing here is visible through the C ABI (include/sw_gemm.h).
#pragma once

#include <stdint.h>

#include <initializer_list>

#include <hip/hip_runtime.h>

#include "sw_gemm.h"

namespace sw {

// ---- workspace layout rules (used by BOTH the planner and the executor, so they cannot disagree) ---------

// Leading dimension of an h-column matrix the library places in its workspace: a multiple of 16 doubles
// (every row starts on a 128-byte line), and never a multiple of 256 doubles (rows of a power-of-two pitch
// would all fall on the same HBM channels).
inline int64_t ws_ld(int64_t h)
{
    int64_t ld = (h + 15) / 16 * 16;
    if (ld >= 256 && ld % 256 == 0) ld += 16;
    return ld;
}

// Shape of one product: C (m x n) = A (m x k) * B (k x n).  The recursion halves all three at every step.
struct Dims {
    int64_t m, n, k;
    Dims half() const { return Dims{m / 2, n / 2, k / 2}; }
    bool cube() const { return m == n && n == k; }
};

// Elements reserved for one rows x cols workspace matrix (a multiple of 32 doubles = 256 bytes).
inline int64_t ws_mat_elems(int64_t rows, int64_t cols) { return (ws_ld(cols) * rows + 31) / 32 * 32; }
inline int64_t ws_mat_elems(int64_t h) { return ws_mat_elems(h, h); }

// Elements of the dense copies a problem with an odd inner extent sets aside when that index is peeled: the last
// column of A over the even rows and the last row of B over the even columns, each rounded up to 32 doubles.
inline int64_t peel_side_elems(Dims d)
{
    if (!(d.k & 1)) return 0;
    const int64_t em = d.m & ~(int64_t)1, en = d.n & ~(int64_t)1;
    return (em + 31) / 32 * 32 + (en + 31) / 32 * 32;
}

// A run of consecutive BFS steps is executed in fused pairs, deepest pairs first: with an even number of B
// ahead the next two steps share one pass and the operands of the level between them are never stored.
inline bool fuse_two_bfs(const char* sched)
{
    int run = 0;
    while (sched[run] == 'B') ++run;
    return run >= 2 && run % 2 == 0;
}

// ... and only when the level between the two steps has even extents: with peeling at every odd level
// (SW_ODD_PEEL_LEVELS) a child of odd size needs its own peel before the next step, so the pair cannot be one pass.
// (In the other modes every extent is a multiple of 2^levels and this never vetoes.)
inline bool fuse_here(Dims d, const char* sched)
{
    const Dims h = d.half();
    return fuse_two_bfs(sched) && !((h.m | h.n | h.k) & 1);
}

// Bytes of workspace the executor takes for a problem of shape d (every extent a multiple of 2^levels) whose
// remaining step order is `sched`, entered with `live` parents.  With T (m/2 x k/2), S (k/2 x n/2) and
// Q (m/2 x n/2) the operands and the product of one child:  BFS step: T, S, Q for all seven children of
// every parent (Section 3.3.1), or for all 49 grandchildren when two BFS steps are fused; DFS step: two
// temporaries per parent -- one that holds a T and later a Q, one that holds an S -- because products are
// written straight into the parent's C quadrants (the footnote of Section 3.3.1 allows a few temporaries).
//
// rich: bit i set = the DFS step at level `level + i` keeps its four non-trivial T, four S and seven Q (15
// buffers per parent, the storage of a BFS step without the plain copies) while still solving the seven
// subproblems in sequence; its additions are then the one-pass BFS kernels.  0 = the minimum.
// dbl: the buffers of the step whose children are the leaves exist twice (consecutive leaf launches then
// alternate between the two sets, so the additions of one launch overlap the products of another).
inline int64_t ws_need_bytes(Dims d, const char* sched, int64_t live, uint32_t rich = 0, bool dbl = false)
{
    if (*sched == '\0') return 0;
    if ((d.m | d.n | d.k) & 1) {
        // an odd extent is peeled before the step (SW_ODD_PEEL_LEVELS; in the other modes no step sees one): the
        // step runs on the even part, and a peeled inner index sets its column of A and row of B aside
        const Dims e{d.m & ~(int64_t)1, d.n & ~(int64_t)1, d.k & ~(int64_t)1};
        return live * peel_side_elems(d) * (int64_t)sizeof(double) + ws_need_bytes(e, sched, live, rich, dbl);
    }
    const Dims h = d.half();
    const int64_t W = (int64_t)sizeof(double);
    const int64_t eT = ws_mat_elems(h.m, h.k) * W, eS = ws_mat_elems(h.k, h.n) * W, eQ = ws_mat_elems(h.m, h.n) * W;
    if (fuse_here(d, sched)) {
        const Dims q = h.half();
        const int64_t e4 = (ws_mat_elems(q.m, q.k) + ws_mat_elems(q.k, q.n) + ws_mat_elems(q.m, q.n)) * W;
        const int copies = (dbl && sched[2] == '\0') ? 2 : 1;
        return copies * 49 * live * e4 + ws_need_bytes(q, sched + 2, 49 * live, rich >> 2, dbl);
    }
    if (*sched == 'B') {
        const int copies = (dbl && sched[1] == '\0') ? 2 : 1;
        return copies * 7 * live * (eT + eS + eQ) + ws_need_bytes(h, sched + 1, 7 * live, rich >> 1, dbl);
    }
    const int64_t here = (rich & 1u) ? 4 * eT + 4 * eS + 7 * eQ : (eT > eQ ? eT : eQ) + eS;
    return live * here + ws_need_bytes(h, sched + 1, live, rich >> 1, dbl);
}
inline int64_t ws_need_bytes(int64_t n, const char* sched, int64_t live, uint32_t rich = 0, bool dbl = false)
{
    return ws_need_bytes(Dims{n, n, n}, sched, live, rich, dbl);
}

// What to spend a workspace of `budget` bytes on beyond the minimum: first the second set of leaf-side
// buffers (only useful when the leaves are reached more than once, i.e. below some DFS step, and when
// additions and products run on separate streams), then the rich form of DFS steps, deepest first.
inline void choose_options(Dims d, int levels, const char* sched, int64_t budget, bool overlap, uint32_t* rich, bool* dbl)
{
    *rich = 0;
    *dbl = false;
    bool any_dfs = false;
    for (int i = 0; i < levels; ++i) any_dfs = any_dfs || sched[i] == 'D';
    if (overlap && any_dfs && levels > 0 && sched[levels - 1] == 'B' && ws_need_bytes(d, sched, 1, 0, true) <= budget)
        *dbl = true;
    for (int i = levels - 1; i >= 0; --i)
        if (sched[i] == 'D' && ws_need_bytes(d, sched, 1, *rich | (1u << i), *dbl) <= budget) *rich |= 1u << i;
}
inline void choose_options(int64_t n, int levels, const char* sched, int64_t budget, bool overlap, uint32_t* rich, bool* dbl)
{
    choose_options(Dims{n, n, n}, levels, sched, budget, overlap, rich, dbl);
}

inline int64_t padded_n(int64_t n, int levels)
{
    const int64_t q = (int64_t)1 << levels;
    return (n + q - 1) / q * q;
}

// ---- error text ---------------------------------------------------------------------------------------------

void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);

// ---- argument checks and library state shared by the entry points ------------------------------------------------

bool schedule_ok(const char* s, int levels);           // `levels` characters, each B or D
int check_shape(int64_t n, int levels);                // SW_OK or SW_EINVAL with the error text set
bool overlaps(const double* p, int64_t pn, const double* q, int64_t qn);   // element ranges [p, p+pn) and [q, q+qn)
void library_state(void** ws, int64_t* ws_bytes, hipStream_t* stream);     // what sw_set_workspace / sw_set_stream left

// The process-wide settings (sw_set_overlap, sw_set_odd_mode, sw_profile_enable) as one call sees them: an
// entry point reads them once and hands them down; nothing below looks at the globals again.
struct CallOpts {
    int overlap;     // 0: one stream; 1: three streams, leaf-side additions sized to their work; k > 1: capped at k
    int odd_mode;    // SW_ODD_PAD or SW_ODD_PEEL
    bool profile;    // bracket every launch with events
    bool check_only; // stop after the argument checks (the workspace pointer is not looked at, only its size)
};
CallOpts current_opts();

// workspace bytes of the Strassen-Winograd product for this step order (with the padded copies, if any)
int64_t total_need(Dims d, int levels, const char* sched, int odd_mode);
int64_t total_need(Dims d, int levels, const char* sched);                 // odd sizes as sw_set_odd_mode says now
inline int64_t total_need(int64_t n, int levels, const char* sched) { return total_need(Dims{n, n, n}, levels, sched); }
// the planner: the best-scored Limited-Memory shape (DFS steps, then BFS steps) that fits `budget`; writes levels + 1 characters
int plan(Dims d, int levels, int64_t budget, char* out, int odd_mode, bool overlap);
// modelled seconds of one step order with what the executor makes of `budget` bytes; -1.0 if it does not fit
double modelled_order(Dims d, int levels, const char* order, int64_t budget, bool overlap, int odd_mode);
int plan(Dims d, int levels, int64_t budget, char* out);
inline int plan(int64_t n, int levels, int64_t budget, char* out) { return plan(Dims{n, n, n}, levels, budget, out); }
// the depth with the least modelled time among those some step order fits into `budget` bytes (0 < n <= 200000)
int plan_levels(int64_t n, int64_t budget);
// the Strassen-Winograd product itself with explicit leading dimensions, workspace and stream (what sw_gemm_ex calls)
int gemm_impl(int64_t n, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
              int levels, const char* schedule, void* ws, int64_t ws_bytes, hipStream_t stream);
// the same recursion on a rectangular product C (m x n) = A (m x k) * B (k x n); extents that 2^levels does
// not divide are zero-padded into workspace copies
int gemm_rect_impl(Dims d, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                   int levels, const char* schedule, void* ws, int64_t ws_bytes, hipStream_t stream);
// ... with the settings given instead of read from the process-wide ones
int gemm_rect_impl(Dims d, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                   int levels, const char* schedule, void* ws, int64_t ws_bytes, hipStream_t stream, const CallOpts& opts);

// ---- profiling record (sw_profile_enable / sw_profile_read) ---------------------------------------------------

struct Profiler;
struct ProfMark { hipEvent_t e0, e1; int cls; double work; };   // one bracket, owned by the caller between begin and end
Profiler* profiler();                                  // nullptr when profiling is off
void prof_begin(Profiler*, hipStream_t, int cls, double work, ProfMark*);
void prof_end(Profiler*, hipStream_t, const ProfMark*);

// ---- a batch of equally shaped matrices: matrix b starts at p + b * stride, rows ld apart ----------------------

struct Mat {
    double* p;
    int64_t ld;
    int64_t stride;
    bool padded = false;   // one more element behind the end of EVERY row is readable memory of the same buffer
};

// Quadrant (i, j) of a batch of 2h x 2h matrices.  Behind a row of a left or top quadrant lies the right
// quadrant or the next row; only the bottom-right quadrant inherits the question from its parent.
inline Mat quad(const Mat& m, int64_t hr, int64_t hc, int i, int j)
{
    return Mat{m.p + i * hr * m.ld + j * hc, m.ld, m.stride, m.padded || !(i == 1 && j == 1)};
}
inline Mat quad(const Mat& m, int64_t h, int i, int j) { return quad(m, h, h, i, j); }

// A batch of rows x cols matrices in the workspace (pitch ws_ld(cols), slot ws_mat_elems(rows, cols)).
inline Mat ws_mat(double* p, int64_t rows, int64_t cols) { return Mat{p, ws_ld(cols), ws_mat_elems(rows, cols), ws_ld(cols) > cols}; }
inline Mat ws_mat(double* p, int64_t h) { return ws_mat(p, h, h); }

// ---- kernel launchers (each validates nothing: callers pass consistent shapes) --------------------------------

// At most `cap` workgroups per launch of an addition kernel (0: one per logical block).  With a cap the kernels
// become persistent streaming kernels that occupy little of each CU, for running beside the leaf products.
// The cap belongs to the calling host thread: launches of other threads are not affected.
void set_add_block_cap(int cap);

// ---- record-only runs (sw_trace_gemm) ---------------------------------------------------------------------------
//
// While a Tracer is installed on the calling thread nothing is launched and no HIP call is made: every launcher
// below writes down what its kernel WOULD touch, from its own arguments (not from what the executor declared
// to its dependency tracker), and the executor's event records and stream waits are written down in their
// place.  A checker can then rebuild happens-before and look for unordered conflicting accesses.
struct Footprint { const void* p; int64_t rows, cols, ld, count, stride; };   // `count` matrices of rows x cols doubles
struct Tracer {
    enum { KERNEL = 1, RECORD = 2, WAIT = 3, TAKE = 4, POP = 5, JOINED = 6 };
    enum { K_PRE_ADD = 0, K_POST_ADD, K_PRE_ADD2, K_POST_ADD2, K_EW, K_DFS_POST, K_PAD_COPY, K_GEMM };
    int64_t* out = nullptr;      // caller's buffer
    int64_t cap = 0, words = 0;  // its capacity; words produced so far (may exceed cap: then only counted)
    void put(int64_t v) { if (words < cap) out[words] = v; ++words; }
    static int stream_id(hipStream_t s) { return (int)(uintptr_t)s - 1; }     // trace streams are the handles 1, 2, 3
    hipError_t kernel(int kid, hipStream_t s, std::initializer_list<Footprint> reads, std::initializer_list<Footprint> writes)
    {
        put(KERNEL); put(stream_id(s)); put(kid); put((int64_t)reads.size()); put((int64_t)writes.size());
        for (const auto* l : {&reads, &writes})
            for (const Footprint& f : *l) { put((int64_t)(uintptr_t)f.p); put(f.rows); put(f.cols); put(f.ld); put(f.count); put(f.stride); }
        return hipSuccess;
    }
    void record(int stream, int slot) { put(RECORD); put(stream); put(slot); }
    void wait(int stream, int ev_stream, int slot) { put(WAIT); put(stream); put(ev_stream); put(slot); }
    void take(int64_t offset, int64_t bytes) { put(TAKE); put(offset); put(bytes); }
    void pop(int64_t offset) { put(POP); put(offset); }
    void joined(int64_t tracked) { put(JOINED); put(tracked); }
};
Tracer* tracer();                 // the calling thread's tracer, nullptr outside sw_trace_gemm
void set_tracer(Tracer*);
inline Footprint fp(const Mat& m, int64_t rows, int64_t cols, int64_t count = 1) { return Footprint{m.p, rows, cols, m.ld, count, m.stride}; }

// All addition kernels work on batches of hr x hc matrices (rows x columns); the square forms take h for both.
// BFS pre-additions, Appendix A columns 1 (side 0, T from A) and 2 (side 1, S from B).
// copies: write all seven operands (slot 7p + j); otherwise only the four non-trivial ones (slot 4p + 0..3).
hipError_t launch_pre_add(int side, Mat parent, int64_t live, int64_t hr, int64_t hc, Mat child, bool copies, hipStream_t s);
// BFS post-additions, Appendix A column 4.
hipError_t launch_post_add(Mat q, int64_t live, int64_t hr, int64_t hc, Mat parent, hipStream_t s);
// Two consecutive BFS steps in one pass: parent of 4 mr x 4 mc -> 49 grandchildren of mr x mc, and back.
hipError_t launch_pre_add2(int side, Mat parent, int64_t live, int64_t mr, int64_t mc, Mat child, hipStream_t s);
hipError_t launch_post_add2(Mat q, int64_t live, int64_t mr, int64_t mc, Mat parent, hipStream_t s);
// Z = X + sign * Y on hr x hc matrices, `live` of them; Z may be X or Y itself.
hipError_t launch_ew(Mat z, Mat x, Mat y, int sign, int64_t live, int64_t hr, int64_t hc, hipStream_t s);
// Two independent such operations of one shape in one launch (the A-side and B-side pre-addition of a DFS step).
hipError_t launch_ew2(Mat z0, Mat x0, Mat y0, int sign0, Mat z1, Mat x1, Mat y1, int sign1, int64_t live,
                      int64_t hr, int64_t hc, hipStream_t s);
// DFS post-addition block: with X = Q0, C12 = Q3, C21 = Q4, C22 = Q2, C11 = Q5 on entry,
// U1 = X + C12, U2 = U1 + C21, U3 = U1 + C22, then C22 = U2 + C22, C12 = U3 + C11, C21 = U2.
hipError_t launch_dfs_post(Mat x, Mat c11, Mat c12, Mat c21, Mat c22, int64_t live, int64_t hr, int64_t hc, hipStream_t s);
inline hipError_t launch_pre_add(int side, Mat parent, int64_t live, int64_t h, Mat child, bool copies, hipStream_t s)
{
    return launch_pre_add(side, parent, live, h, h, child, copies, s);
}
inline hipError_t launch_post_add(Mat q, int64_t live, int64_t h, Mat parent, hipStream_t s) { return launch_post_add(q, live, h, h, parent, s); }
inline hipError_t launch_pre_add2(int side, Mat parent, int64_t live, int64_t m, Mat child, hipStream_t s)
{
    return launch_pre_add2(side, parent, live, m, m, child, s);
}
inline hipError_t launch_post_add2(Mat q, int64_t live, int64_t m, Mat parent, hipStream_t s) { return launch_post_add2(q, live, m, m, parent, s); }
inline hipError_t launch_ew(Mat z, Mat x, Mat y, int sign, int64_t live, int64_t h, hipStream_t s) { return launch_ew(z, x, y, sign, live, h, h, s); }
inline hipError_t launch_ew2(Mat z0, Mat x0, Mat y0, int sign0, Mat z1, Mat x1, Mat y1, int sign1, int64_t live, int64_t h,
                             hipStream_t s)
{
    return launch_ew2(z0, x0, y0, sign0, z1, x1, y1, sign1, live, h, h, s);
}
inline hipError_t launch_dfs_post(Mat x, Mat c11, Mat c12, Mat c21, Mat c22, int64_t live, int64_t h, hipStream_t s)
{
    return launch_dfs_post(x, c11, c12, c21, c22, live, h, h, s);
}
// Zero-padded copy / crop.
// One-wide products of a peeled level, batched over `live` problems (a column x: element k at x.p + k * x.ld; a row:
// contiguous).  y = A x (A: M x K);  y = x B (B: K x N);  C += u v (u a column of M, v a row of N).
// thin_grid_ok: whether the three fit the launch limits (else the MFMA kernel does the same products).
hipError_t launch_matvec(int64_t M, int64_t K, int64_t live, Mat a, Mat x, Mat y, hipStream_t s);
hipError_t launch_vecmat(int64_t N, int64_t K, int64_t live, Mat x, Mat b, Mat y, hipStream_t s);
hipError_t launch_rank1(int64_t M, int64_t N, int64_t live, Mat u, Mat v, Mat c, hipStream_t s);
inline bool thin_grid_ok(int64_t M, int64_t live) { return live <= 65535 && (M + 3) / 4 <= 65535; }
// dst_b = src_b (rows x cols) for b < live: dense copies of thin strips
hipError_t launch_strip_copy(Mat src, int64_t rows, int64_t cols, Mat dst, int64_t live, hipStream_t s);
hipError_t launch_pad_copy(const double* src, int64_t src_ld, int64_t rows, int64_t cols, double* dst,
                           int64_t dst_ld, int64_t prows, int64_t pcols, hipStream_t s);
// Batched classical product on the fp64 matrix cores: C_b = A_b * B_b, all m x m.
hipError_t launch_leaf_gemm(int64_t m, int64_t batch, Mat a, Mat b, Mat c, hipStream_t s);
// Leading dimensions the kernel can address (its per-lane byte offsets are 32 bit): lda <= 4 227 329 and
// ldb <= 35 791 385 doubles.  launch_gemm returns hipErrorInvalidValue beyond; entry points check first.
bool gemm_pitches_ok(int64_t lda, int64_t ldb);
// The same kernel on general shapes: C_b (M x N) = or += A_b (M x K) * B_b (K x N).
hipError_t launch_gemm(int64_t M, int64_t N, int64_t K, int64_t batch, Mat a, Mat b, Mat c, bool accumulate,
                       hipStream_t s);

// Diagonal scaling (Section 6.1): weighted maxima of |X| over rows / columns, scale vectors, scaled copy.
hipError_t launch_absmax_rows(const double* X, int64_t ld, int64_t n, const double* w, double* out, hipStream_t s);
hipError_t launch_absmax_cols(const double* X, int64_t ld, int64_t n, const double* w, double* out, hipStream_t s);
hipError_t launch_outside_scale(const double* m, int64_t n, double* sc, hipStream_t s);
hipError_t launch_inside_scale(const double* a, const double* b, int64_t n, double* d, double* dinv, hipStream_t s);
hipError_t launch_scale_copy(const double* X, int64_t xld, int64_t n, const double* r, const double* c, double* Y,
                             int64_t yld, hipStream_t s);

}  // namespace sw
