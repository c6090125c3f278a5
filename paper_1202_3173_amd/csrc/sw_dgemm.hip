// The product as a drop-in general matrix multiply: C <- alpha * op(A) * op(B) + beta * C on rectangular
// row-major operands, op(X) = X or its transpose, and the choice of the recursion depth by a cost model.
//
// M, N and K are each cut into 1 .. 4 equal parts (multiples of 2^levels), which gives blocks of
// s.m x s.n x s.k; every block product goes through the Strassen-Winograd recursion on rectangular operands
// into a temporary P and is folded into C by one pass (C_ij <- alpha * P + beta' * C_ij, beta' = beta for the
// first inner slice and 1 afterwards; straight into C when alpha = 1, beta = 0 and K is one slice).  What is
// left over in each dimension (fewer than 4 * 2^levels rows, columns or inner indices) goes through the
// classical MFMA product, the K remainder being accumulated before the fold.  Transposed operands are
// transposed block by block into a workspace buffer, so the recursion and the leaf kernel always see
// row-major blocks.  Block shape and depth are chosen by the cost model below.
#include <math.h>
#include <string.h>

#include <string>

#include "sw_internal.h"

namespace sw {
namespace {

constexpr int TILE = 32;

// dst (cols x rows, pitch dld) = transpose of src (rows x cols, pitch sld)
__global__ __launch_bounds__(TILE * 8) void transpose_kernel(const double* __restrict__ src, int64_t sld, int rows, int cols,
                                                             double* __restrict__ dst, int64_t dld, int tiles_c, int64_t ntiles)
{
    __shared__ double tile[TILE][TILE + 1];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int r0 = (int)(t / tiles_c) * TILE, c0 = (int)(t % tiles_c) * TILE;
        for (int i = threadIdx.y; i < TILE; i += 8) {
            const int r = r0 + i, c = c0 + threadIdx.x;
            if (r < rows && c < cols) tile[i][threadIdx.x] = src[(int64_t)r * sld + c];
        }
        __syncthreads();
        for (int i = threadIdx.y; i < TILE; i += 8) {
            const int c = c0 + i, r = r0 + threadIdx.x;
            if (r < rows && c < cols) dst[(int64_t)c * dld + r] = tile[threadIdx.x][i];
        }
        __syncthreads();
    }
}

// C <- alpha * P + beta * C on rows x cols; beta == 0: C is not read; alpha == 0: P is not read
__global__ __launch_bounds__(256) void axpby_kernel(double* __restrict__ C, int64_t ldc, const double* __restrict__ P, int64_t ldp,
                                                    int rows, int cols, double alpha, double beta)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    for (int r = blockIdx.y; r < rows; r += gridDim.y) {
        double* dst = C + (int64_t)r * ldc + c;
        double v = 0.0;
        if (beta != 0.0) v = beta * *dst;
        if (alpha != 0.0) v = fma(alpha, P[(int64_t)r * ldp + c], v);
        *dst = v;
    }
}

hipError_t launch_transpose(const double* src, int64_t sld, int64_t rows, int64_t cols, double* dst, int64_t dld, hipStream_t s)
{
    if (rows == 0 || cols == 0) return hipSuccess;
    const int tiles_c = (int)((cols + TILE - 1) / TILE);
    const int64_t ntiles = (int64_t)tiles_c * ((rows + TILE - 1) / TILE);
    const unsigned blocks = (unsigned)(ntiles < (1 << 20) ? ntiles : (1 << 20));
    hipLaunchKernelGGL(transpose_kernel, dim3(blocks), dim3(TILE, 8), 0, s, src, sld, (int)rows, (int)cols, dst, dld, tiles_c, ntiles);
    return hipGetLastError();
}

hipError_t launch_axpby(double* C, int64_t ldc, const double* P, int64_t ldp, int64_t rows, int64_t cols, double alpha,
                        double beta, hipStream_t s)
{
    if (rows == 0 || cols == 0) return hipSuccess;
    const dim3 grid((unsigned)((cols + 255) / 256), (unsigned)(rows < 65535 ? rows : 65535));
    hipLaunchKernelGGL(axpby_kernel, grid, dim3(256), 0, s, C, ldc, P, ldp, (int)rows, (int)cols, alpha, beta);
    return hipGetLastError();
}

// ---- cost model for the recursion depth -----------------------------------------------------------------------
// Leaf products: 7^L classical products of the shape 1/2^L of the problem's, launched 7^(BFS steps) at a time,
// at the rate the MFMA kernel reaches for that inner extent (a measured table), times the fill of its
// 128 x 128 tiles, times the fill of the 512 workgroup slots by the tiles of one launch.
// Additions: elements moved per parent and step (see step_elems; for a cube 33, 48.75, 38 or 27 half-size
// matrices) at 5.2 TB/s, plus a few microseconds per launch.  The constants are fitted to measurements on one
// MI355X at n = 2048 .. 94080.
// by inner extent k of the leaf (the length of the K loop decides how much prologue and epilogue weigh)
double table_rate(double k)
{
    // rate on full tiles with all workgroup slots busy, TFLOP/s, by leaf size (measured on square leaves;
    // between the points linear in log2): short inner loops leave prologue and epilogue of every tile exposed
    static const double size[] = {64, 128, 256, 512, 1024, 2048, 4096, 8192};
    static const double rate[] = {12, 27, 47, 61, 72, 74, 75.3, 76.4};
    if (k <= size[0]) return rate[0] * k / size[0];
    for (int i = 1; i < 8; ++i)
        if (k <= size[i]) {
            const double f = (log2(k) - log2(size[i - 1])) / (log2(size[i]) - log2(size[i - 1]));
            return rate[i - 1] + f * (rate[i] - rate[i - 1]);
        }
    return rate[7];
}

double leaf_rate(double m, double n, double k, double batch)
{
    const double em = ceil(m / 128.0), en = ceil(n / 128.0);
    const double fill = (m / (em * 128.0)) * (n / (en * 128.0));             // tiles that hang over the edge
    const double tiles = batch * em * en;
    // 512 workgroup slots (two per CU) are filled in rounds; a last round of at most 256 tiles has every CU
    // to one workgroup, which then runs at 0.89 of the rate of two and finishes in 0.56 of a round
    const double full = floor(tiles / 512.0), rest = tiles - 512.0 * full;
    // (after full rounds the slots free up one by one, so a short rest costs less than a whole lone-workgroup tile)
    const double lone = (full > 0.0 && rest / 512.0 + 0.25 < 0.56) ? rest / 512.0 + 0.25 : 0.56;
    const double rounds = full + (rest == 0.0 ? 0.0 : (rest <= 256.0 ? lone : 1.0));
    return table_rate(k) * 1e12 * fill * (tiles / 512.0) / rounds;
}

// elements moved per parent by the additions of one step on children of shape h (T: h.m x h.k, S: h.k x h.n,
// Q: h.m x h.n): a BFS step reads 4 and writes 7 on each operand side and reads 7, writes 4 for C; two fused
// BFS steps 16 and 49 of the quarter blocks; a DFS step with two temporaries 12, 12 and 14; one that keeps
// its operands 8, 8 and 11
double step_elems(Dims h, double a, double b, double c)
{
    return a * (double)h.m * (double)h.k + b * (double)h.k * (double)h.n + c * (double)h.m * (double)h.n;
}

// dbl: the buffers next to the leaves exist twice and additions run on their own streams (the three-stream
// executor below a DFS step): the additions of the last BFS step (or fused pair) then run beside the leaf
// products of the neighbouring launches, so a launch costs the longer of the two, with the products stretched
// by the share of the machine's power the streaming kernels take (measured: 7 %).
double modelled_seconds(Dims d, int levels, const char* order, uint32_t rich, bool dbl)
{
    constexpr double HBM = 5.2e12, LAUNCH = 6e-6, STRETCH = 1.07;
    const Dims p{padded_n(d.m, levels), padded_n(d.n, levels), padded_n(d.k, levels)};
    double t = 0.0, parents = 1.0, launches = 1.0;   // `launches` subtrees in sequence, `parents` in each
    double beside = 0.0;                             // additions per leaf launch that run beside the products
    Dims h = p;
    for (int i = 0; i < levels;) {
        const Dims cur = h;
        h = h.half();
        if (fuse_here(cur, order + i)) {
            h = h.half();
            const double adds = parents * 8.0 * step_elems(h, 65, 65, 65) / HBM + 3 * LAUNCH;
            if (dbl && i + 2 == levels) beside = adds; else t += launches * adds;
            parents *= 49.0;
            i += 2;
        } else if (order[i] == 'B') {
            const double adds = parents * 8.0 * step_elems(h, 11, 11, 11) / HBM + 3 * LAUNCH;
            if (dbl && i + 1 == levels) beside = adds; else t += launches * adds;
            parents *= 7.0;
            i += 1;
        } else {
            const bool keep = (rich >> i) & 1u;
            t += launches * (parents * 8.0 * (keep ? step_elems(h, 8, 8, 11) : step_elems(h, 12, 12, 14)) / HBM + (keep ? 3 : 9) * LAUNCH);
            launches *= 7.0;
            i += 1;
        }
    }
    // `parents` leaf products of shape h per launch, `launches` launches
    const double leaf = parents * 2.0 * (double)h.m * (double)h.n * (double)h.k / leaf_rate((double)h.m, (double)h.n, (double)h.k, parents) + LAUNCH;
    if (beside > 0.0) {
        const double both = leaf * STRETCH > beside ? leaf * STRETCH : beside;
        t += launches * both + beside;               // the first launch's operands and the last one's fold are exposed
    } else {
        t += launches * leaf;
    }
    if (p.m != d.m || p.n != d.n || p.k != d.k)
        t += 8.0 * ((double)d.m * d.k + (double)d.k * d.n + 2.0 * (double)d.m * d.n + (double)p.m * p.k + (double)p.k * p.n + 2.0 * (double)p.m * p.n) / HBM;
    return t;
}
double modelled_seconds(Dims d, int levels, const char* order, uint32_t rich) { return modelled_seconds(d, levels, order, rich, false); }

// the modelled time of one step order with what the executor would make of `budget` bytes of workspace
// (rich DFS steps, second set of leaf-side buffers); -1.0 when the order does not fit
double modelled_order_impl(Dims d, int levels, const char* order, int64_t budget, bool overlap, int odd_mode)
{
    if (levels == 0) return modelled_seconds(d, 0, order, 0, false);
    const int64_t need = total_need(d, levels, order, odd_mode);
    if (need > budget) return -1.0;
    uint32_t rich = 0;
    bool dbl = false;
    const Dims p{padded_n(d.m, levels), padded_n(d.n, levels), padded_n(d.k, levels)};
    const int64_t fixed = need - ws_need_bytes(p, order, 1);
    choose_options(p, levels, order, budget - fixed, overlap, &rich, &dbl);
    return modelled_seconds(d, levels, order, rich, dbl);
}

double modelled_for_budget(Dims d, int levels, int64_t budget, char* order)
{
    if (levels == 0) { order[0] = '\0'; return modelled_seconds(d, 0, order, 0); }
    const CallOpts o = current_opts();
    if (plan(d, levels, budget, order, o.odd_mode, o.overlap != 0) != SW_OK) return -1.0;   // no step order of this depth fits
    return modelled_order_impl(d, levels, order, budget, o.overlap != 0, o.odd_mode);
}

int best_levels(Dims d, int64_t budget)
{
    const int64_t lo = d.m < d.n ? (d.m < d.k ? d.m : d.k) : (d.n < d.k ? d.n : d.k);
    // below the measured crossover (classical wins at 2048, the recursion by a few percent at 4096) the
    // product is a handful of launch-bound kernels the model does not describe
    if (cbrt((double)d.m * (double)d.n * (double)d.k) < 3072.0) return 0;
    char order[SW_MAX_LEVELS + 1];
    int best = 0;
    double best_t = modelled_for_budget(d, 0, budget, order);
    for (int L = 1; L <= SW_MAX_LEVELS && ((int64_t)1 << L) <= lo; ++L) {
        if ((lo >> L) < 64) break;                              // leaves below half a tile never pay
        const double t = modelled_for_budget(d, L, budget, order);
        if (t >= 0.0 && t < best_t) { best_t = t; best = L; }
    }
    return best;
}
int best_levels(int64_t n, int64_t budget) { return best_levels(Dims{n, n, n}, budget); }

struct Dgemm {
    bool ta, tb;
    int64_t M, N, K;
    double alpha, beta;
    const double* A; int64_t lda;
    const double* B; int64_t ldb;
    double* C; int64_t ldc;
    Dims s;                         // block shape: C blocks s.m x s.n, inner slices of s.k
    int64_t ldp, lda_t, ldb_t;      // pitches of P (s.m x s.n), TA (s.m x s.k), TB (s.k x s.n)
    double *P, *TA, *TB;
    int levels;
    const char* schedule;
    void* rest; int64_t rest_bytes;
    hipStream_t st;
    Profiler* prof;
    hipError_t err = hipSuccess;
    int rc = SW_OK;

    void note(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
    bool ok() const { return err == hipSuccess && rc == SW_OK; }

    // op(A)[i0 .. i0+rows, k0 .. k0+kc) as a row-major block (rows <= s.m, kc <= s.k)
    Mat blockA(int64_t i0, int64_t rows, int64_t k0, int64_t kc)
    {
        if (!ta) return Mat{const_cast<double*>(A) + i0 * lda + k0, lda, 0, false};
        ProfMark pm_;
        prof_begin(prof, st, SW_CLASS_BLAS, 16.0 * rows * kc, &pm_);
        note(launch_transpose(A + k0 * lda + i0, lda, kc, rows, TA, lda_t, st));
        prof_end(prof, st, &pm_);
        return Mat{TA, lda_t, 0, lda_t > kc};
    }
    // op(B)[k0 .. k0+kc, j0 .. j0+cols)  (kc <= s.k, cols <= s.n)
    Mat blockB(int64_t k0, int64_t kc, int64_t j0, int64_t cols)
    {
        if (!tb) return Mat{const_cast<double*>(B) + k0 * ldb + j0, ldb, 0, false};
        ProfMark pm_;
        prof_begin(prof, st, SW_CLASS_BLAS, 16.0 * kc * cols, &pm_);
        note(launch_transpose(B + j0 * ldb + k0, ldb, cols, kc, TB, ldb_t, st));
        prof_end(prof, st, &pm_);
        return Mat{TB, ldb_t, 0, ldb_t > cols};
    }
    void fold(int64_t i0, int64_t rows, int64_t j0, int64_t cols, double b)
    {
        ProfMark pm_;
        prof_begin(prof, st, SW_CLASS_BLAS, 8.0 * rows * cols * (b != 0.0 ? 3.0 : 2.0), &pm_);
        note(launch_axpby(C + i0 * ldc + j0, ldc, P, ldp, rows, cols, alpha, b, st));
        prof_end(prof, st, &pm_);
    }
    void classical(int64_t rows, int64_t cols, int64_t kc, Mat a, Mat b, Mat c, bool accumulate)
    {
        ProfMark pm_;
        prof_begin(prof, st, SW_CLASS_PEEL, 2.0 * rows * cols * kc, &pm_);
        note(launch_gemm(rows, cols, kc, 1, a, b, c, accumulate, st));
        prof_end(prof, st, &pm_);
    }

    // an s.m x s.n block of C through the recursion, one inner slice of s.k after the other
    void fast_block(int64_t i0, int64_t j0)
    {
        const int64_t kb = K / s.k, rK = K - kb * s.k;
        // a single product that needs no scaling and no old C goes straight into C
        const bool direct = alpha == 1.0 && beta == 0.0 && kb == 1;
        const Mat out = direct ? Mat{C + i0 * ldc + j0, ldc, 0, false} : Mat{P, ldp, 0, ldp > s.n};
        for (int64_t k = 0; k < kb && ok(); ++k) {
            const Mat a = blockA(i0, s.m, k * s.k, s.k), b = blockB(k * s.k, s.k, j0, s.n);
            if (!ok()) return;
            rc = gemm_rect_impl(s, a.p, a.ld, b.p, b.ld, out.p, out.ld, levels, schedule, rest, rest_bytes, st);
            if (rc != SW_OK) return;
            if (k == kb - 1 && rK > 0) {
                const Mat ar = blockA(i0, s.m, kb * s.k, rK), br = blockB(kb * s.k, rK, j0, s.n);
                classical(s.m, s.n, rK, ar, br, out, true);
            }
            if (!direct) fold(i0, s.m, j0, s.n, k == 0 ? beta : 1.0);
        }
    }

    // a block of at most s.m x s.n of C through the classical product, K in slices of s.k
    void classical_block(int64_t i0, int64_t rows, int64_t j0, int64_t cols)
    {
        for (int64_t k0 = 0; k0 < K && ok(); k0 += s.k) {
            const int64_t kc = K - k0 < s.k ? K - k0 : s.k;
            const Mat a = blockA(i0, rows, k0, kc), b = blockB(k0, kc, j0, cols);
            classical(rows, cols, kc, a, b, Mat{P, ldp, 0, ldp > cols}, k0 > 0);
        }
        fold(i0, rows, j0, cols, beta);
    }

    void run()
    {
        const int64_t mb = M / s.m, nb = N / s.n, rM = M - mb * s.m, rN = N - nb * s.n;
        for (int64_t i = 0; i < mb && ok(); ++i)
            for (int64_t j = 0; j < nb && ok(); ++j) fast_block(i * s.m, j * s.n);
        if (rN > 0)                                                    // the right strip, all rows
            for (int64_t i0 = 0; i0 < M && ok(); i0 += s.m) classical_block(i0, M - i0 < s.m ? M - i0 : s.m, nb * s.n, rN);
        if (rM > 0)                                                    // the bottom strip left of it
            for (int64_t j = 0; j < nb && ok(); ++j) classical_block(mb * s.m, rM, j * s.n, s.n);
    }
};

// extent / parts, rounded down to a multiple of 2^levels
int64_t block_extent(int64_t extent, int parts, int levels)
{
    const int64_t raw = extent / parts;
    return raw - raw % ((int64_t)1 << levels);
}

// one temporary for a block of C, one more per transposed operand
int64_t fixed_bytes(bool ta, bool tb, Dims s)
{
    return (ws_mat_elems(s.m, s.n) + (ta ? ws_mat_elems(s.m, s.k) : 0) + (tb ? ws_mat_elems(s.k, s.n) : 0)) * (int64_t)sizeof(double);
}

struct Choice { Dims s; int levels; double seconds; };

// The block shape: M, N and K are each cut into 1 .. 4 equal parts (rounded down to a multiple of 2^levels;
// what is left over, less than parts * 2^levels rows, columns or inner indices, goes through the classical
// product).  Among the shapes whose workspace need fits, the one with the least modelled time: block products
// through the recursion at their modelled time plus one fold pass, the rest at the classical rate.
// levels < 0: the depth is chosen per shape as well.  order_out: the step order when the caller gave none.
Choice choose_blocking(int64_t M, int64_t N, int64_t K, int levels, const char* schedule, bool ta, bool tb, int64_t ws_bytes,
                       char* order_out)
{
    Choice best{Dims{0, 0, 0}, 0, 0.0};
    char order[SW_MAX_LEVELS + 1];
    for (int pm = 1; pm <= 4; ++pm)
        for (int pn = 1; pn <= 4; ++pn)
            for (int pk = 1; pk <= 4; ++pk) {
                int L = levels;
                if (L < 0) {
                    const Dims raw{M / pm, N / pn, K / pk};
                    if (raw.m == 0 || raw.n == 0 || raw.k == 0) continue;
                    const int64_t room0 = ws_bytes - fixed_bytes(ta, tb, raw);
                    L = room0 > 0 ? best_levels(raw, room0) : 0;
                }
                const Dims s{block_extent(M, pm, L), block_extent(N, pn, L), block_extent(K, pk, L)};
                if (s.m == 0 || s.n == 0 || s.k == 0) continue;
                const int64_t room = ws_bytes - fixed_bytes(ta, tb, s);
                if (room < 0) continue;
                double tblock = -1.0;
                if (schedule && *schedule) {
                    if (total_need(s, L, schedule) <= room) { tblock = modelled_seconds(s, L, schedule, 0); strcpy(order, schedule); }
                } else {
                    tblock = modelled_for_budget(s, L, room, order);
                }
                if (tblock < 0.0) continue;
                const double blocks = (double)(M / s.m) * (double)(N / s.n) * (double)(K / s.k);
                const double rest = 2.0 * (double)M * N * K - blocks * 2.0 * (double)s.m * s.n * s.k;
                const double t = blocks * (tblock + 3.0 * 8.0 * (double)s.m * s.n / 5.0e12) + rest / 75e12;
                if (best.s.m == 0 || t < best.seconds) {
                    best = Choice{s, L, t};
                    strcpy(order_out, order);
                }
            }
    return best;
}

int check_dims(int64_t M, int64_t N, int64_t K, int levels)
{
    if (M < 0 || N < 0 || K < 0) { set_error("negative dimension"); return SW_EINVAL; }
    if (M > 200000 || N > 200000 || K > 200000) { set_error("a dimension above the supported maximum of 200000"); return SW_EINVAL; }
    if (levels > SW_MAX_LEVELS) { set_error("levels = %d above %d", levels, SW_MAX_LEVELS); return SW_EINVAL; }
    return SW_OK;
}

}  // namespace

double modelled_order(Dims d, int levels, const char* order, int64_t budget, bool overlap, int odd_mode)
{
    return modelled_order_impl(d, levels, order, budget, overlap, odd_mode);
}

int plan_levels(int64_t n, int64_t budget) { return n > 0 ? best_levels(n, budget) : 0; }

}  // namespace sw

using namespace sw;

extern "C" {

int sw_plan_levels(int64_t n, int64_t budget_bytes)
{
    if (n < 0 || n > 200000 || budget_bytes < 0) { set_error("bad argument"); return SW_EINVAL; }
    if (n == 0) return 0;
    return best_levels(n, budget_bytes);
}

double sw_model_seconds_order(int64_t n, int levels, const char* schedule, int64_t budget_bytes, int overlap)
{
    if (check_shape(n, levels) != SW_OK || n <= 0 || budget_bytes < 0 || !schedule || !schedule_ok(schedule, levels)) return -1.0;
    return modelled_order_impl(Dims{n, n, n}, levels, schedule, budget_bytes, overlap != 0, SW_ODD_PAD);
}

double sw_model_seconds(int64_t n, int levels, int64_t budget_bytes)
{
    if (n <= 0 || n > 200000 || levels < 0 || levels > SW_MAX_LEVELS || ((int64_t)1 << levels) > n || budget_bytes < 0) {
        set_error("bad argument");
        return -1.0;
    }
    char order[SW_MAX_LEVELS + 1];
    const double t = modelled_for_budget(Dims{n, n, n}, levels, budget_bytes, order);
    if (t < 0.0) set_error("no step order of depth %d fits %lld bytes", levels, (long long)budget_bytes);
    return t;
}

int64_t sw_plan_memory_dgemm(int transa, int transb, int64_t M, int64_t N, int64_t K, int levels, const char* schedule)
{
    int rc = check_dims(M, N, K, levels);
    if (rc != SW_OK) return rc;
    if (levels < 0) { set_error("sw_plan_memory_dgemm needs an explicit depth (sw_plan_levels gives one)"); return SW_EINVAL; }
    if (M == 0 || N == 0 || K == 0) return 0;
    const Dims s{block_extent(M, 1, levels), block_extent(N, 1, levels), block_extent(K, 1, levels)};
    if (s.m == 0 || s.n == 0 || s.k == 0) { set_error("2^levels = %lld exceeds the smallest dimension", (long long)((int64_t)1 << levels)); return SW_EINVAL; }
    const int64_t inner = sw_plan_memory_rect(s.m, s.n, s.k, levels, schedule);
    if (inner < 0) return inner;
    return fixed_bytes(transa != 0, transb != 0, s) + inner;
}

int sw_dgemm(int transa, int transb, int64_t M, int64_t N, int64_t K, double alpha, const double* A, int64_t lda,
             const double* B, int64_t ldb, double beta, double* C, int64_t ldc, int levels, const char* schedule)
{
    int rc = check_dims(M, N, K, levels);
    if (rc != SW_OK) return rc;
    if (M == 0 || N == 0) return SW_OK;
    const bool ta = transa != 0, tb = transb != 0;
    if (!C || ldc < N) { set_error("C is NULL or ldc < N"); return SW_EINVAL; }
    void* ws = nullptr;
    int64_t ws_bytes = 0;
    hipStream_t st = nullptr;
    library_state(&ws, &ws_bytes, &st);
    Profiler* prof = profiler();
    if (K == 0 || alpha == 0.0) {
        // nothing to multiply: C <- beta * C, the operands are not read
        ProfMark pm_;
        prof_begin(prof, st, SW_CLASS_BLAS, 8.0 * M * N * 2.0, &pm_);
        hipError_t e = launch_axpby(C, ldc, nullptr, 0, M, N, 0.0, beta, st);
        prof_end(prof, st, &pm_);
        return e == hipSuccess ? SW_OK : hip_fail(e, "scaling kernel");
    }
    const int64_t arows = ta ? K : M, acols = ta ? M : K, brows = tb ? N : K, bcols = tb ? K : N;
    if (!A || !B) { set_error("NULL matrix pointer"); return SW_EINVAL; }
    if (lda < acols || ldb < bcols) { set_error("leading dimension smaller than the row length"); return SW_EINVAL; }
    // operands that are not transposed are read by the product kernel as views of the caller's matrices
    if (!gemm_pitches_ok(ta ? 0 : lda, tb ? 0 : ldb)) {
        set_error("leading dimension too large for the product kernel's 32-bit offsets (lda <= 4227329, ldb <= 35791385)");
        return SW_EINVAL;
    }
    const int64_t spanA = (arows - 1) * lda + acols, spanB = (brows - 1) * ldb + bcols, spanC = (M - 1) * ldc + N;
    if (overlaps(C, spanC, A, spanA) || overlaps(C, spanC, B, spanB)) { set_error("C overlaps A or B"); return SW_EINVAL; }
    if (ws && ((uintptr_t)ws & 255u)) { set_error("workspace must be 256-byte aligned"); return SW_EINVAL; }

    if (schedule && *schedule && levels >= 0 && !schedule_ok(schedule, levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", schedule, levels);
        return SW_EINVAL;
    }
    if (levels < 0) schedule = nullptr;
    if (levels >= 0 && (block_extent(M, 1, levels) == 0 || block_extent(N, 1, levels) == 0 || block_extent(K, 1, levels) == 0)) {
        set_error("2^levels = %lld exceeds the smallest dimension", (long long)((int64_t)1 << levels));
        return SW_EINVAL;
    }
    // Block shape (and depth, if left open) by the cost model
    char chosen[SW_MAX_LEVELS + 1] = "";
    const Choice ch = choose_blocking(M, N, K, levels, schedule, ta, tb, ws ? ws_bytes : 0, chosen);
    if (ch.s.m == 0) {
        set_error("workspace of %lld bytes is too small for any block shape of %lld x %lld x %lld", (long long)(ws ? ws_bytes : 0),
                  (long long)M, (long long)N, (long long)K);
        return SW_ENOMEM;
    }
    const Dims s = ch.s;
    levels = ch.levels;
    if (!schedule || !*schedule) schedule = chosen;
    const int64_t fixed = fixed_bytes(ta, tb, s);
    if (overlaps((const double*)ws, ws_bytes / 8, A, spanA) || overlaps((const double*)ws, ws_bytes / 8, B, spanB) ||
        overlaps((const double*)ws, ws_bytes / 8, C, spanC)) {
        set_error("workspace overlaps A, B or C");
        return SW_EINVAL;
    }

    Dgemm g;
    g.ta = ta; g.tb = tb;
    g.M = M; g.N = N; g.K = K;
    g.alpha = alpha; g.beta = beta;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
    g.s = s;
    g.ldp = ws_ld(s.n); g.lda_t = ws_ld(s.k); g.ldb_t = ws_ld(s.n);
    double* w = (double*)ws;
    g.P = w; w += ws_mat_elems(s.m, s.n);
    g.TA = ta ? w : nullptr; if (ta) w += ws_mat_elems(s.m, s.k);
    g.TB = tb ? w : nullptr; if (tb) w += ws_mat_elems(s.k, s.n);
    g.levels = levels;
    g.schedule = schedule;
    g.rest = w;
    g.rest_bytes = ws_bytes - fixed;
    g.st = st;
    g.prof = prof;
    g.run();
    if (g.rc != SW_OK) return g.rc;
    if (g.err != hipSuccess) return hip_fail(g.err, "kernel launch");
    return SW_OK;
}

}  // extern "C"
