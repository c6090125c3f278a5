// Batched classical fp64 product for the leaves of the recursion tree (Section 5.4.1: below the cutoff the
// implementation switches to the classical algorithm), written for the CDNA4 matrix cores.
//
//   C_b = A_b * B_b,  b < batch, every matrix m x m, row-major, one launch for the whole batch.
//
// Design (gfx950, 256 CUs, 64-wide wavefronts, v_mfma_f64_16x16x4_f64 = 64 cycles of one SIMD's matrix pipe):
//   * a workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128 tile of one C_b; each wavefront owns
//     64 x 64 of it as 4 x 4 MFMA tiles of 16 x 16, i.e. 64 fp64 accumulators per lane, kept in VGPRs;
//   * K is walked in slabs of 16 = four MFMA k-steps.  Per slab a wavefront issues 64 MFMAs; everything else
//     is threaded between them so the matrix pipe never waits on it:
//       k-step 0: write the NEXT slab (loaded from global memory one slab earlier) into the other LDS buffer
//       k-step 1: issue the global loads of the slab after that into the freed staging registers
//       k-steps 0..2: read the fragments of the following k-step from LDS into the other fragment set
//       one barrier, then k-step 3 runs while the first fragments of the next slab are read;
//   * LDS: A slab as [row][k] with a pitch of 18 doubles, B slab as [k][col] with a pitch of 144 doubles;
//     with these pitches the 8-byte fragment reads of 32 consecutive lanes fall on 32 distinct bank pairs;
//   * two workgroups fit per CU (72 KB of LDS each, < 256 VGPRs), so what one wavefront cannot hide (the
//     barrier itself) is covered by the other workgroup's MFMAs;
//   * workgroup ids are remapped so that each XCD (ids congruent mod 8 share an XCD and its L2) works on a
//     contiguous run of tiles, ordered in groups of 8 tile rows: the ~64 tiles in flight on an XCD then
//     share A row panels and B column panels through that L2;
//   * edges: rows and columns beyond m are clamped to the last valid one on load (their products land in
//     accumulators that are never stored); the K tail is zero-filled; stores are bounds-checked on tiles that
//     reach beyond the matrix and unchecked (one address update per four rows) on tiles inside it.  A cell of the
//     128 x 128 grid that holds at most 64 or 96 rows (columns) of the matrix runs a body with 2 or 3 MFMA tiles
//     per wavefront in that direction instead of 4, so an edge cell issues only the MFMAs its part of the
//     matrix needs (to the next multiple of 32).  16-byte global loads when pointers and leading dimensions
//     allow it (an odd m too, if rows are padded), 8-byte loads otherwise.
#include <type_traits>

#include "sw_internal.h"

namespace sw {
namespace {

typedef double v2d __attribute__((ext_vector_type(2)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16, NT = 256;
constexpr int SA = 18;                 // LDS pitch of an A row (doubles)
constexpr int SB = BN + 16;            // LDS pitch of a B k-row (doubles)
constexpr int A_ELEMS = BM * SA;       // 2304
constexpr int B_ELEMS = BK * SB;       // 2304
constexpr int STAGE = A_ELEMS + B_ELEMS;
constexpr int GROUP_M = 8;             // tile rows per ordering group
constexpr int NUM_XCD = 8;

struct GemmArgs {
    const double* A;
    const double* B;
    double* C;
    int64_t lda, ldb, ldc;
    int64_t sa, sb, sc;   // batch strides
    int M, N, K;
    int tiles_m, tiles_n;
    int accumulate;       // 0: C = A*B, 1: C += A*B
};

// One tile of C.  NI x NJ MFMA tiles of 16 x 16 per wavefront: the workgroup's 2 x 2 wavefronts cover
// (32 NI) x (32 NJ) of the 128 x 128 grid cell, which is all of it for NI = NJ = 4 and the part that holds rows
// and columns of the matrix for a cell on the bottom or right edge (NI, NJ = 2 or 3 when at most 64 or 96 of the
// cell's rows / columns exist): an edge cell then issues NI NJ / 16 of the MFMAs of a full one.
template <int VEC, int NI, int NJ>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, double* smem, const int batch, const int m0, const int n0)
{

    // uniform bases of this tile's A row panel and B column panel
    const double* __restrict__ A = g.A + (int64_t)batch * g.sa + (int64_t)m0 * g.lda;
    const double* __restrict__ B = g.B + (int64_t)batch * g.sb + n0;
    double* __restrict__ C = g.C + (int64_t)batch * g.sc;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global -> register staging: who loads what --------------------------------------------------------
    // VEC == 2: A: row tid/8 + 32 i (i < 4), k (tid%8)*2, +1.        B: k tid/64 + 4 i (i < 4), cols (tid%64)*2, +1
    // VEC == 1: A: row tid/16 + 16 i (i < 8), k tid%16.              B: k tid/128 + 2 i (i < 8), col tid%128
    typedef typename std::conditional<VEC == 2, v2d, double>::type V;
    constexpr int NL = VEC == 2 ? 4 : 8;
    constexpr int A_RSTEP = VEC == 2 ? 32 : 16;
    constexpr int B_KSTEP = VEC == 2 ? 4 : 2;
    const int a_k = VEC == 2 ? (tid & 7) * 2 : (tid & 15);
    const int a_r0 = VEC == 2 ? (tid >> 3) : (tid >> 4);
    const int b_c = VEC == 2 ? (tid & 63) * 2 : (tid & 127);
    const int b_k0 = VEC == 2 ? (tid >> 6) : (tid >> 7);

    // BYTE offsets from the uniform panel bases (rows / columns clamped into the matrix).  They stay below
    // 128 * ld * 8 < 2^32, so every load is "uniform 64-bit base in SGPRs + 32-bit per-lane offset" and
    // the K loop advances the bases with scalar adds only: no vector ALU work competes with the MFMAs.
    // last column (pair) a lane may load: with VEC == 2 and odd N the pair N - 1, N reaches into the padding
    const int b_cmax = (VEC == 2 ? ((g.N - 1) & ~1) : g.N - 1) - n0;
    unsigned offA[NL], offB[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int row = min(a_r0 + i * A_RSTEP, g.M - 1 - m0);
        offA[i] = ((unsigned)((int64_t)row * g.lda) + (unsigned)a_k) * 8u;
        offB[i] = ((unsigned)((int64_t)(b_k0 + i * B_KSTEP) * g.ldb) + (unsigned)min(b_c, b_cmax)) * 8u;
    }

    V ra[NL], rb[NL];

    // a whole slab whose uniform byte bases are pa (A panel at column k0) and pb (B panel at row k0)
    auto gload = [&](const char* __restrict__ pa, const char* __restrict__ pb) __attribute__((always_inline)) {
        // The empty asm keeps each 32-bit offset opaque inside the loop, so that instruction selection
        // sees "scalar base + zero-extended 32-bit lane offset" and emits the SGPR-base form of global_load
        // instead of a 64-bit vector add per load.
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            asm volatile("" : "+v"(offA[i]));
            ra[i] = *reinterpret_cast<const V*>(pa + offA[i]);
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            asm volatile("" : "+v"(offB[i]));
            rb[i] = *reinterpret_cast<const V*>(pb + offB[i]);
        }
    };
    // the last slab when it reaches beyond K: k is clamped for the address and the value zero-filled
    auto gload_tail = [&](int k0) __attribute__((always_inline)) {
        // A: the lane's k (VEC == 2: the pair k, k + 1; with odd K the pair K - 1, K reaches into the row's
        // padding, which the caller guarantees to exist, and that element is zeroed)
        const int k = k0 + a_k;
        const int kc = min(k, VEC == 2 ? ((g.K - 1) & ~1) : g.K - 1);   // last load position inside the row
        const int a_back = (k - kc) * 8;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            V v = *reinterpret_cast<const V*>(reinterpret_cast<const char*>(A + k0) + ((int64_t)offA[i] - a_back));
            if constexpr (VEC == 2) {
                if (k >= g.K) v[0] = 0.0;
                if (k + 1 >= g.K) v[1] = 0.0;
            } else {
                if (k >= g.K) v = 0.0;
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int kb = k0 + b_k0 + i * B_KSTEP;
            const bool ok = kb < g.K;
            const int64_t back = ok ? 0 : (int64_t)(kb - (g.K - 1)) * g.ldb * 8;
            const V v = *reinterpret_cast<const V*>(reinterpret_cast<const char*>(B + (int64_t)k0 * g.ldb) + ((int64_t)offB[i] - back));
            rb[i] = ok ? v : V(0.0);
        }
    };

    auto sstore_a = [&](int buf) __attribute__((always_inline)) {
        double* As = smem + buf * STAGE;
#pragma unroll
        for (int i = 0; i < NL; ++i) *reinterpret_cast<V*>(As + (a_r0 + i * A_RSTEP) * SA + a_k) = ra[i];
    };
    auto sstore_b = [&](int buf) __attribute__((always_inline)) {
        double* Bs = smem + buf * STAGE + A_ELEMS;
#pragma unroll
        for (int i = 0; i < NL; ++i) *reinterpret_cast<V*>(Bs + (b_k0 + i * B_KSTEP) * SB + b_c) = rb[i];
    };
    auto sstore = [&](int buf) __attribute__((always_inline)) { sstore_a(buf); sstore_b(buf); };

    // ---- fragments and accumulators -------------------------------------------------------------------------
    v4d acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    double fa[2][NI], fb[2][NJ];   // two fragment sets: one feeds the MFMAs while the other is being read

    // k-step s of the slab in buffer buf: lane (r16, g4) holds A[16 i + r16][4 s + g4] and B[4 s + g4][16 j + r16]
    auto fread = [&](int buf, int s, int set) __attribute__((always_inline)) {
        const double* As = smem + buf * STAGE + (wm * (16 * NI) + r16) * SA + 4 * s + g4;
        const double* Bs = smem + buf * STAGE + A_ELEMS + (4 * s + g4) * SB + wn * (16 * NJ) + r16;
#pragma unroll
        for (int i = 0; i < NI; ++i) fa[set][i] = As[i * 16 * SA];
#pragma unroll
        for (int j = 0; j < NJ; ++j) fb[set][j] = Bs[j * 16];
    };

    // MFMA tile rows i0 .. i1-1 of one k-step
    auto mfma_rows = [&](int set, int i0, int i1) __attribute__((always_inline)) {
#pragma unroll
        for (int i = i0; i < (i1 < NI ? i1 : NI); ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };
#define SW_FENCE() __builtin_amdgcn_sched_barrier(0)

    const int KT = (g.K + BK - 1) / BK;
    const bool ragged = (g.K % BK) != 0;     // only the last slab can reach beyond K
    const int64_t stepA = (int64_t)BK * 8, stepB = (int64_t)BK * g.ldb * 8;
    const char* pa = reinterpret_cast<const char*>(A);   // uniform bases of the NEXT slab to load
    const char* pb = reinterpret_cast<const char*>(B);

    // One slab held in LDS buffer `cur`.  The scheduling fences pin the order written here: LDS reads for
    // the NEXT k-step are issued before the MFMAs of this one, and stores / global loads are slipped
    // between groups of four MFMAs, whose 256 cycles of matrix-pipe time cover their issue.
    //   store: the next slab is in the staging registers and goes to the other buffer
    //   load:  0 nothing, 1 start the global loads of the slab after next, 2 the same, zero-filling the K tail
    auto slab = [&](int kt, int cur, bool store, int load) __attribute__((always_inline)) {
        // k-step 0: fetch the fragments of k-step 1, publish the next slab
        fread(cur, 1, 1);
        SW_FENCE();
        mfma_rows(0, 0, 1);
        SW_FENCE();
        if (store) sstore_a(cur ^ 1);
        SW_FENCE();
        mfma_rows(0, 1, 2);
        SW_FENCE();
        if (store) sstore_b(cur ^ 1);
        SW_FENCE();
        mfma_rows(0, 2, 4);
        SW_FENCE();
        // k-step 1: start the global loads of the slab after next into the freed staging registers
        fread(cur, 2, 0);
        SW_FENCE();
        mfma_rows(1, 0, 1);
        SW_FENCE();
        if (load == 1) { gload(pa, pb); pa += stepA; pb += stepB; }
        if (load == 2) gload_tail((kt + 2) * BK);
        SW_FENCE();
        mfma_rows(1, 1, 4);
        SW_FENCE();
        // k-step 2
        fread(cur, 3, 1);
        SW_FENCE();
        mfma_rows(0, 0, 4);
        SW_FENCE();
        // every wavefront has stored the next slab and finished reading this one
        __syncthreads();
        // k-step 3, overlapped with the first fragment reads of the next slab
        if (store) fread(cur ^ 1, 0, 0);
        SW_FENCE();
        mfma_rows(1, 0, 4);
        SW_FENCE();
    };

    if (KT == 1 && ragged) gload_tail(0); else { gload(pa, pb); pa += stepA; pb += stepB; }
    sstore(0);
    if (KT > 1) { if (KT == 2 && ragged) gload_tail(BK); else { gload(pa, pb); pa += stepA; pb += stepB; } }
    __syncthreads();
    fread(0, 0, 0);

    // steady state, two slabs per trip so that the LDS buffer index is a compile-time constant and all
    // LDS addresses are "per-lane base + immediate": straight-line code without vector ALU instructions
    int kt = 0;
    for (; kt + 4 < KT; kt += 2) {
        slab(kt, 0, true, 1);
        slab(kt + 1, 1, true, 1);
    }
    // the last (up to four) slabs: nothing more to store or load at the very end, and a ragged K tail.  Two per
    // trip as well (kt is even here), so the buffers stay compile-time constants and only the flags are decided
    // at run time, by scalar branches: with the buffer a run-time value every LDS access of these slabs needed
    // vector-ALU address arithmetic, and they took twice as long as steady ones.
    auto last_slab = [&](int k, auto buf) __attribute__((always_inline)) {
        const bool store = k + 1 < KT;
        const int load = k + 2 < KT ? ((ragged && k + 2 == KT - 1) ? 2 : 1) : 0;
        slab(k, decltype(buf)::value, store, load);
    };
    for (; kt < KT; kt += 2) {
        last_slab(kt, std::integral_constant<int, 0>());
        if (kt + 1 < KT) last_slab(kt + 1, std::integral_constant<int, 1>());
    }

    // ---- store: accumulator v of lane (r16, g4) in MFMA tile (i, j) is C[16 i + g4 + 4 v][16 j + r16] ----
    const int row0 = m0 + wm * (16 * NI) + g4, col0 = n0 + wn * (16 * NJ) + r16;
    if (!g.accumulate && m0 + 32 * NI <= g.M && n0 + 32 * NJ <= g.N) {
        // the whole tile lies inside the matrix: one 64-bit address per lane, advanced by four rows per store
        // group, the columns of a group as immediate offsets -- the fewer vector-ALU instructions here, the
        // sooner the matrix pipe is handed to the next tile (each one queues behind the MFMAs of the other
        // workgroup on this CU)
        char* cp = reinterpret_cast<char*>(C + (int64_t)row0 * g.ldc + col0);
        const int64_t step = 4 * g.ldc * (int64_t)sizeof(double);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) reinterpret_cast<double*>(cp)[j * 16] = acc[i][j][v];
                cp += step;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = row0 + i * 16 + 4 * v;
            if (row < g.M) {
                double* crow = C + (int64_t)row * g.ldc + col0;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    if (col0 + j * 16 < g.N)
                        crow[j * 16] = g.accumulate ? crow[j * 16] + acc[i][j][v] : acc[i][j][v];
            }
        }
    }
}

// how many 16-row (16-column) MFMA tiles per wavefront cover `left` remaining rows (columns) of a 128-wide cell
__device__ __forceinline__ int wave_tiles(int left) { return left > 96 ? 4 : (left > 64 ? 3 : 2); }

template <int VEC>
__global__ void __launch_bounds__(NT, 2)
leaf_gemm_kernel(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) double smem[2 * STAGE];

    // ---- which tile: XCD-aware remap, then grouped order inside a matrix ----
    const int nb = gridDim.x;
    const int bid = blockIdx.x;
    const int xcd = bid % NUM_XCD;
    const int per = nb / NUM_XCD, rem = nb % NUM_XCD;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + bid / NUM_XCD;
    const int tpm = g.tiles_m * g.tiles_n;
    const int batch = logical / tpm;
    const int t = logical - batch * tpm;
    const int grp = t / (GROUP_M * g.tiles_n);
    const int first_m = grp * GROUP_M;
    const int gsz = min(GROUP_M, g.tiles_m - first_m);
    const int tin = t - grp * (GROUP_M * g.tiles_n);
    const int tile_m = first_m + tin % gsz;
    const int tile_n = tin / gsz;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // the shape of this cell's part of the matrix picks the body (uniform over the workgroup)
    const int ni = wave_tiles(g.M - m0), nj = wave_tiles(g.N - n0);
#define SW_TILE(I, J) if (ni == I && nj == J) { gemm_tile<VEC, I, J>(g, smem, batch, m0, n0); return; }
    SW_TILE(4, 4) SW_TILE(4, 3) SW_TILE(3, 4) SW_TILE(3, 3) SW_TILE(4, 2) SW_TILE(2, 4) SW_TILE(3, 2) SW_TILE(2, 3) SW_TILE(2, 2)
#undef SW_TILE
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

// The kernel addresses a tile's operands as "uniform 64-bit panel base + 32-bit BYTE offset per lane": a lane
// reaches up to 127 rows of A (plus 15 more doubles along the row) and 15 rows of B (plus 127 doubles) from
// the base, so (127 lda + 16) * 8 and (15 ldb + 128) * 8 must stay below 2^32.
bool gemm_pitches_ok(int64_t lda, int64_t ldb)
{
    const int64_t lim = (int64_t)1 << 32;
    return lda >= 0 && ldb >= 0 && lda < lim && ldb < lim && (127 * lda + 16) * 8 < lim && (15 * ldb + 128) * 8 < lim;
}

hipError_t launch_gemm(int64_t M, int64_t N, int64_t K, int64_t batch, Mat a, Mat b, Mat c, bool accumulate,
                       hipStream_t s)
{
    if (M == 0 || N == 0 || batch == 0) return hipSuccess;
    if (K == 0) return accumulate ? hipSuccess : hipErrorInvalidValue;   // callers never ask for an empty sum
    if (!gemm_pitches_ok(a.ld, b.ld)) return hipErrorInvalidValue;
    if (Tracer* t = tracer()) {
        if (accumulate) return t->kernel(Tracer::K_GEMM, s, {fp(a, M, K, batch), fp(b, K, N, batch), fp(c, M, N, batch)}, {fp(c, M, N, batch)});
        return t->kernel(Tracer::K_GEMM, s, {fp(a, M, K, batch), fp(b, K, N, batch)}, {fp(c, M, N, batch)});
    }
    GemmArgs g;
    g.A = a.p; g.B = b.p; g.C = c.p;
    g.lda = a.ld; g.ldb = b.ld; g.ldc = c.ld;
    g.sa = a.stride; g.sb = b.stride; g.sc = c.stride;
    g.M = (int)M; g.N = (int)N; g.K = (int)K;
    g.tiles_m = (int)((M + BM - 1) / BM);
    g.tiles_n = (int)((N + BN - 1) / BN);
    g.accumulate = accumulate ? 1 : 0;
    const int64_t blocks = (int64_t)g.tiles_m * g.tiles_n * batch;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    // 16-byte loads need aligned pairs.  An odd K (pairs along A's rows) or an odd N (pairs along B's rows)
    // is fine when one more element behind every row is readable memory: the pair that straddles the edge
    // then stays inside the allocation and its outer half is zeroed (A) or lands in a column never stored (B).
    const bool v2 = aligned16(a.p) && aligned16(b.p) && a.ld % 2 == 0 && b.ld % 2 == 0 && a.stride % 2 == 0 &&
                    b.stride % 2 == 0 && (K % 2 == 0 || a.padded) && (N % 2 == 0 || b.padded);
    if (v2) hipLaunchKernelGGL((leaf_gemm_kernel<2>), dim3((unsigned)blocks), dim3(NT), 0, s, g);
    else    hipLaunchKernelGGL((leaf_gemm_kernel<1>), dim3((unsigned)blocks), dim3(NT), 0, s, g);
    return hipGetLastError();
}

hipError_t launch_leaf_gemm(int64_t m, int64_t batch, Mat a, Mat b, Mat c, hipStream_t s)
{
    return launch_gemm(m, m, m, batch, a, b, c, false, s);
}

}  // namespace sw
