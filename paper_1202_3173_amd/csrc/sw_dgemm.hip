// The product as a drop-in general matrix multiply: C <- alpha * op(A) * op(B) + beta * C on rectangular
// row-major operands, op(X) = X or its transpose, and the choice of the recursion depth by a cost model.
//
// The fast recursion works on square blocks.  With s the largest multiple of 2^levels that fits min(M, N, K),
// op(A), op(B), C are cut into s x s blocks; every block product goes through the Strassen-Winograd
// recursion into a temporary P and is folded into C by one pass (C_ij <- alpha * P + beta' * C_ij, beta' =
// beta for the first k block and 1 afterwards).  What is left over in each dimension (less than s rows,
// columns or inner indices) goes through the classical MFMA product, the K remainder being accumulated into P
// before the fold.  Transposed operands are transposed block by block into a workspace buffer, so the
// recursion and the leaf kernel always see row-major blocks.
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
// Leaf products: 7^L classical products of size m = n / 2^L, launched 7^(BFS steps) at a time, at the rate the
// MFMA kernel reaches on m x m (a measured table), times the fill of its 128 x 128 tiles, times the fill of
// the 512 workgroup slots by the tiles of one launch.
// Additions: per parent and step, in half-size matrices moved through HBM: 33 for a BFS step, 48.75 for
// two fused BFS steps (in units of the upper one), 38 for a DFS step with two temporaries, 27 for one that
// keeps its operands; at 5.2 TB/s, plus a few microseconds per launch.  The constants are fitted to
// measurements on one MI355X at n = 2048 .. 94080.
double leaf_rate(double m, double batch)
{
    // rate on full tiles with all workgroup slots busy, TFLOP/s, by leaf size (measured; between the points
    // linear in log2 m): short inner loops leave prologue and epilogue of every tile exposed
    static const double size[] = {64, 128, 256, 512, 1024, 2048, 4096, 8192};
    static const double rate[] = {12, 27, 47, 61, 72, 74, 75.3, 76.4};
    double r = rate[7];
    if (m <= size[0]) r = rate[0] * m / size[0];
    else
        for (int i = 1; i < 8; ++i)
            if (m <= size[i]) {
                const double f = (log2(m) - log2(size[i - 1])) / (log2(size[i]) - log2(size[i - 1]));
                r = rate[i - 1] + f * (rate[i] - rate[i - 1]);
                break;
            }
    const double edge = ceil(m / 128.0);
    const double fill = (m / (edge * 128.0)) * (m / (edge * 128.0));          // tiles that hang over the edge
    const double tiles = batch * edge * edge;
    // 512 workgroup slots (two per CU) are filled in rounds; a last round of at most 256 tiles has every CU
    // to one workgroup, which then runs at 0.89 of the rate of two and finishes in 0.56 of a round
    const double full = floor(tiles / 512.0), rest = tiles - 512.0 * full;
    const double rounds = full + (rest == 0.0 ? 0.0 : (rest <= 256.0 ? 0.56 : 1.0));
    return r * 1e12 * fill * (tiles / 512.0) / rounds;
}

double modelled_seconds(int64_t n, int levels, const char* order, uint32_t rich)
{
    constexpr double HBM = 5.2e12, LAUNCH = 6e-6;
    const int64_t np = padded_n(n, levels);
    const double m = (double)(np >> levels);
    double t = 0.0, parents = 1.0, launches = 1.0, h = (double)np;   // `launches` subtrees in sequence, `parents` in each
    for (int i = 0; i < levels;) {
        h /= 2;
        const double unit = 8.0 * h * h;
        if (fuse_two_bfs(order + i)) {
            t += launches * (parents * 48.75 * unit / HBM + 3 * LAUNCH);
            parents *= 49.0;
            h /= 2;
            i += 2;
        } else if (order[i] == 'B') {
            t += launches * (parents * 33.0 * unit / HBM + 3 * LAUNCH);
            parents *= 7.0;
            i += 1;
        } else {
            const bool keep = (rich >> i) & 1u;
            t += launches * (parents * (keep ? 27.0 : 38.0) * unit / HBM + (keep ? 3 : 9) * LAUNCH);
            launches *= 7.0;
            i += 1;
        }
    }
    // `parents` leaf products per launch, `launches` launches
    t += launches * (parents * 2.0 * m * m * m / leaf_rate(m, parents) + LAUNCH);
    if (np != n) t += 8.0 * (2.0 * (double)n * n + 4.0 * (double)np * np) / HBM;
    return t;
}

double modelled_for_budget(int64_t n, int levels, int64_t budget, char* order)
{
    if (levels == 0) { order[0] = '\0'; return modelled_seconds(n, 0, order, 0); }
    if (plan(n, levels, budget, order) != SW_OK) return -1.0;       // no step order of this depth fits
    uint32_t rich = 0;
    bool dbl = false;
    const int64_t np = padded_n(n, levels);
    const int64_t fixed = total_need(n, levels, order) - ws_need_bytes(np, order, 1);
    choose_options(np, levels, order, budget - fixed, false, &rich, &dbl);
    return modelled_seconds(n, levels, order, rich);
}

int best_levels(int64_t n, int64_t budget)
{
    // below the measured crossover (classical wins at 2048, the recursion by a few percent at 4096) the
    // product is a handful of launch-bound kernels the model does not describe
    if (n < 3072) return 0;
    char order[SW_MAX_LEVELS + 1];
    int best = 0;
    double best_t = modelled_for_budget(n, 0, budget, order);
    for (int L = 1; L <= SW_MAX_LEVELS && ((int64_t)1 << L) <= n; ++L) {
        if ((n >> L) < 64) break;                               // leaves below half a tile never pay
        const double t = modelled_for_budget(n, L, budget, order);
        if (t >= 0.0 && t < best_t) { best_t = t; best = L; }
    }
    return best;
}

struct Dgemm {
    bool ta, tb;
    int64_t M, N, K;
    double alpha, beta;
    const double* A; int64_t lda;
    const double* B; int64_t ldb;
    double* C; int64_t ldc;
    int64_t s, ldp;
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

    // op(A)[i0 .. i0+rows, k0 .. k0+kc) as a row-major block
    Mat blockA(int64_t i0, int64_t rows, int64_t k0, int64_t kc)
    {
        if (!ta) return Mat{const_cast<double*>(A) + i0 * lda + k0, lda, 0, false};
        prof_begin(prof, st, SW_CLASS_BLAS, 16.0 * rows * kc);
        note(launch_transpose(A + k0 * lda + i0, lda, kc, rows, TA, ldp, st));
        prof_end(prof, st);
        return Mat{TA, ldp, 0, ldp > kc};
    }
    // op(B)[k0 .. k0+kc, j0 .. j0+cols)
    Mat blockB(int64_t k0, int64_t kc, int64_t j0, int64_t cols)
    {
        if (!tb) return Mat{const_cast<double*>(B) + k0 * ldb + j0, ldb, 0, false};
        prof_begin(prof, st, SW_CLASS_BLAS, 16.0 * kc * cols);
        note(launch_transpose(B + j0 * ldb + k0, ldb, cols, kc, TB, ldp, st));
        prof_end(prof, st);
        return Mat{TB, ldp, 0, ldp > cols};
    }
    void fold(int64_t i0, int64_t rows, int64_t j0, int64_t cols, double b)
    {
        prof_begin(prof, st, SW_CLASS_BLAS, 8.0 * rows * cols * (b != 0.0 ? 3.0 : 2.0));
        note(launch_axpby(C + i0 * ldc + j0, ldc, P, ldp, rows, cols, alpha, b, st));
        prof_end(prof, st);
    }
    void classical(int64_t rows, int64_t cols, int64_t kc, Mat a, Mat b, bool accumulate)
    {
        prof_begin(prof, st, SW_CLASS_PEEL, 2.0 * rows * cols * kc);
        note(launch_gemm(rows, cols, kc, 1, a, b, Mat{P, ldp, 0, ldp > cols}, accumulate, st));
        prof_end(prof, st);
    }

    // an s x s block of C through the recursion, one k block after the other
    void fast_block(int64_t i0, int64_t j0)
    {
        const int64_t kb = K / s, rK = K - kb * s;
        // a single product that needs no scaling and no old C goes straight into C
        const bool direct = alpha == 1.0 && beta == 0.0 && kb == 1 && rK == 0;
        for (int64_t k = 0; k < kb && ok(); ++k) {
            const Mat a = blockA(i0, s, k * s, s), b = blockB(k * s, s, j0, s);
            if (!ok()) return;
            rc = gemm_impl(s, a.p, a.ld, b.p, b.ld, direct ? C + i0 * ldc + j0 : P, direct ? ldc : ldp, levels, schedule, rest,
                           rest_bytes, st);
            if (rc != SW_OK || direct) return;
            if (k == kb - 1 && rK > 0) {
                const Mat ar = blockA(i0, s, kb * s, rK), br = blockB(kb * s, rK, j0, s);
                classical(s, s, rK, ar, br, true);
            }
            fold(i0, s, j0, s, k == 0 ? beta : 1.0);
        }
    }

    // a block of at most s x s of C through the classical product, K in slices of s
    void classical_block(int64_t i0, int64_t rows, int64_t j0, int64_t cols)
    {
        for (int64_t k0 = 0; k0 < K && ok(); k0 += s) {
            const int64_t kc = K - k0 < s ? K - k0 : s;
            const Mat a = blockA(i0, rows, k0, kc), b = blockB(k0, kc, j0, cols);
            classical(rows, cols, kc, a, b, k0 > 0);
        }
        fold(i0, rows, j0, cols, beta);
    }

    void run()
    {
        const int64_t mb = M / s, nb = N / s, rM = M - mb * s, rN = N - nb * s;
        for (int64_t i = 0; i < mb && ok(); ++i)
            for (int64_t j = 0; j < nb && ok(); ++j) fast_block(i * s, j * s);
        if (rN > 0)                                                    // the right strip, all rows
            for (int64_t i0 = 0; i0 < M && ok(); i0 += s) classical_block(i0, M - i0 < s ? M - i0 : s, nb * s, rN);
        if (rM > 0)                                                    // the bottom strip left of it
            for (int64_t j = 0; j < nb && ok(); ++j) classical_block(mb * s, rM, j * s, s);
    }
};

// largest multiple of 2^levels that fits the smallest dimension
int64_t block_size(int64_t M, int64_t N, int64_t K, int levels)
{
    int64_t d = M < N ? M : N;
    if (K < d) d = K;
    return d - d % ((int64_t)1 << levels);
}

int64_t fixed_bytes(bool ta, bool tb, int64_t s) { return (1 + (ta ? 1 : 0) + (tb ? 1 : 0)) * ws_mat_elems(s) * (int64_t)sizeof(double); }

struct Choice { int64_t s; int levels; double seconds; };

// Among the block sizes floor(min(M, N, K) / j), j = 1 .. 8 (rounded down to a multiple of 2^levels), the one
// with the least modelled time that fits the workspace: block products through the recursion at their
// modelled time, everything else at the classical rate, one fold pass per block product.  levels < 0: the
// depth is chosen per block size as well.  order_out: the step order to use when the caller gave none.
Choice choose_blocking(int64_t M, int64_t N, int64_t K, int levels, const char* schedule, bool ta, bool tb, int64_t ws_bytes,
                       char* order_out)
{
    int64_t d = M < N ? M : N;
    if (K < d) d = K;
    Choice best{0, 0, 0.0};
    char order[SW_MAX_LEVELS + 1];
    for (int j = 1; j <= 8; ++j) {
        const int64_t raw = d / j;
        if (raw == 0) break;
        int L = levels;
        if (L < 0) {
            const int64_t room0 = ws_bytes - fixed_bytes(ta, tb, raw);
            L = room0 > 0 ? best_levels(raw, room0) : 0;
        }
        const int64_t s = raw - raw % ((int64_t)1 << L);
        if (s == 0) continue;
        const int64_t room = ws_bytes - fixed_bytes(ta, tb, s);
        if (room < 0) continue;
        double tb_ = -1.0;
        if (schedule && *schedule) {
            if (total_need(s, L, schedule) <= room) { tb_ = modelled_seconds(s, L, schedule, 0); strcpy(order, schedule); }
        } else {
            tb_ = modelled_for_budget(s, L, room, order);
        }
        if (tb_ < 0.0) continue;
        const double blocks = (double)(M / s) * (double)(N / s) * (double)(K / s);
        const double rest = 2.0 * (double)M * N * K - blocks * 2.0 * (double)s * s * s;
        const double t = blocks * (tb_ + 3.0 * 8.0 * (double)s * s / 5.0e12) + rest / 75e12;
        if (best.s == 0 || t < best.seconds) {
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

double sw_model_seconds(int64_t n, int levels, int64_t budget_bytes)
{
    if (n <= 0 || n > 200000 || levels < 0 || levels > SW_MAX_LEVELS || ((int64_t)1 << levels) > n || budget_bytes < 0) {
        set_error("bad argument");
        return -1.0;
    }
    char order[SW_MAX_LEVELS + 1];
    const double t = modelled_for_budget(n, levels, budget_bytes, order);
    if (t < 0.0) set_error("no step order of depth %d fits %lld bytes", levels, (long long)budget_bytes);
    return t;
}

int64_t sw_plan_memory_dgemm(int transa, int transb, int64_t M, int64_t N, int64_t K, int levels, const char* schedule)
{
    int rc = check_dims(M, N, K, levels);
    if (rc != SW_OK) return rc;
    if (levels < 0) { set_error("sw_plan_memory_dgemm needs an explicit depth (sw_plan_levels gives one)"); return SW_EINVAL; }
    if (M == 0 || N == 0 || K == 0) return 0;
    const int64_t s = block_size(M, N, K, levels);
    if (s == 0) { set_error("2^levels = %lld exceeds the smallest dimension", (long long)((int64_t)1 << levels)); return SW_EINVAL; }
    const int64_t inner = sw_plan_memory(s, levels, schedule);
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
        prof_begin(prof, st, SW_CLASS_BLAS, 8.0 * M * N * 2.0);
        hipError_t e = launch_axpby(C, ldc, nullptr, 0, M, N, 0.0, beta, st);
        prof_end(prof, st);
        return e == hipSuccess ? SW_OK : hip_fail(e, "scaling kernel");
    }
    const int64_t arows = ta ? K : M, acols = ta ? M : K, brows = tb ? N : K, bcols = tb ? K : N;
    if (!A || !B) { set_error("NULL matrix pointer"); return SW_EINVAL; }
    if (lda < acols || ldb < bcols) { set_error("leading dimension smaller than the row length"); return SW_EINVAL; }
    const int64_t spanA = (arows - 1) * lda + acols, spanB = (brows - 1) * ldb + bcols, spanC = (M - 1) * ldc + N;
    if (overlaps(C, spanC, A, spanA) || overlaps(C, spanC, B, spanB)) { set_error("C overlaps A or B"); return SW_EINVAL; }
    if (ws && ((uintptr_t)ws & 255u)) { set_error("workspace must be 256-byte aligned"); return SW_EINVAL; }

    if (schedule && *schedule && levels >= 0 && !schedule_ok(schedule, levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", schedule, levels);
        return SW_EINVAL;
    }
    if (levels < 0) schedule = nullptr;
    if (levels >= 0 && block_size(M, N, K, levels) == 0) {
        set_error("2^levels = %lld exceeds the smallest dimension", (long long)((int64_t)1 << levels));
        return SW_EINVAL;
    }
    // Block size (and depth, if left open) by the cost model: the smallest dimension cut into 1 .. 8 blocks;
    // fewer, larger blocks recurse deeper, more blocks leave less to the classical remainder products.
    char chosen[SW_MAX_LEVELS + 1] = "";
    const Choice ch = choose_blocking(M, N, K, levels, schedule, ta, tb, ws ? ws_bytes : 0, chosen);
    if (ch.s == 0) {
        const int64_t s1 = block_size(M, N, K, levels < 0 ? 0 : levels);
        set_error("workspace of %lld bytes is too small: a block size of %lld needs %lld", (long long)(ws ? ws_bytes : 0), (long long)s1,
                  (long long)(fixed_bytes(ta, tb, s1) + total_need(s1, levels < 0 ? 0 : levels,
                                                                   schedule && *schedule ? schedule : std::string((size_t)(levels < 0 ? 0 : levels), 'D').c_str())));
        return SW_ENOMEM;
    }
    const int64_t s = ch.s;
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
    g.s = s; g.ldp = ws_ld(s);
    double* w = (double*)ws;
    const int64_t e = ws_mat_elems(s);
    g.P = w; w += e;
    g.TA = ta ? w : nullptr; if (ta) w += e;
    g.TB = tb ? w : nullptr; if (tb) w += e;
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
