// Batched classical fp64 product for the leaves of the recursion tree (Section 5.4.1: below the cutoff the
// implementation switches to the classical algorithm), written for the CDNA4 matrix cores.
//
//   C_b = A_b * B_b,  b < batch, every matrix m x m, row-major, one launch for the whole batch.
//
// Design (gfx950, 256 CUs, 64-wide wavefronts, v_mfma_f64_16x16x4_f64):
//   * a workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128 tile of one C_b; each wavefront owns
//     64 x 64 of it as 4 x 4 MFMA tiles of 16 x 16, i.e. 64 fp64 accumulators per lane, kept in VGPRs;
//   * K is walked in slabs of 16; a slab of A (128 x 16) and of B (16 x 128) is loaded from global memory
//     into registers while the previous slab is being multiplied, then written to the other half of a
//     double-buffered LDS area: one barrier per slab;
//   * LDS layouts make every fragment read one conflict-free ds_read_b128 that feeds TWO MFMAs: A is kept
//     [row][k] with a row pitch of 18 doubles, B is kept [k/2][col][k%2] so that the two k of a pair sit side
//     by side.  The MFMA of lane group g (= lane / 16) may use any k as long as A and B agree, so group g
//     takes k = 8q + 2g and 8q + 2g + 1 (q = 0, 1) of the slab for its two consecutive MFMAs;
//   * two workgroups fit per CU (70 KB of LDS each, < 256 VGPRs), so one wavefront's barrier or LDS wait is
//     covered by the other's MFMAs;
//   * workgroup ids are remapped so that each XCD (ids congruent mod 8 share an XCD and its L2) works on a
//     contiguous run of tiles, ordered in groups of 8 tile rows: the ~64 tiles in flight on an XCD then
//     share A row panels and B column panels through that L2;
//   * edges (m not a multiple of 128, K not a multiple of 16) are handled by zero-filled loads and
//     bounds-checked stores; 16-byte global loads are used when pointers, leading dimensions and m allow
//     it, 8-byte loads otherwise.
#include "sw_internal.h"

namespace sw {
namespace {

typedef double v2d __attribute__((ext_vector_type(2)));
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16, NT = 256;
constexpr int SA = 18;                 // LDS pitch of an A row (doubles): 16 + 2 keeps b128 reads conflict-free
constexpr int SBP = 2 * BN + 4;        // LDS pitch of a B k-pair row (doubles)
constexpr int A_ELEMS = BM * SA;       // 2304
constexpr int B_ELEMS = (BK / 2) * SBP;  // 2080
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
};

template <int VEC>
__global__ void __launch_bounds__(NT, 2)
leaf_gemm_kernel(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) double smem[2 * STAGE];

    // ---- which tile: XCD-aware remap, then grouped row-major order inside a matrix ----
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

    const double* __restrict__ A = g.A + (int64_t)batch * g.sa;
    const double* __restrict__ B = g.B + (int64_t)batch * g.sb;
    double* __restrict__ C = g.C + (int64_t)batch * g.sc;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- global -> register staging -------------------------------------------------------------------
    // VEC == 2: A: 4 loads of 2 doubles: row tid/8 + 32 i, k (tid%8)*2.   B: k pair tid/64 + 4 i (i < 2),
    //           columns (tid%64)*2, +1; the two k of the pair are two loads.
    // VEC == 1: A: 8 loads: row tid/16 + 16 i, k tid%16.                  B: k pair tid/128 + 2 i (i < 4),
    //           column tid%128.
    constexpr int NA = VEC == 2 ? 4 : 8;
    constexpr int NBP = VEC == 2 ? 2 : 4;
    const int a_k = VEC == 2 ? (tid & 7) * 2 : (tid & 15);
    const int a_r0 = VEC == 2 ? (tid >> 3) : (tid >> 4);
    constexpr int A_RSTEP = VEC == 2 ? 32 : 16;
    const int b_c = VEC == 2 ? (tid & 63) * 2 : (tid & 127);
    const int b_p0 = VEC == 2 ? (tid >> 6) : (tid >> 7);
    constexpr int B_PSTEP = VEC == 2 ? 4 : 2;

    typedef typename std::conditional<VEC == 2, v2d, double>::type V;
    V ra[NA];
    V rb[NBP][2];

    const bool b_col_ok = n0 + b_c < g.N;   // VEC == 2 requires N even, so the pair is in or out together

    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int row = m0 + a_r0 + i * A_RSTEP;
            const int k = k0 + a_k;
            V v = V(0.0);
            if (row < g.M && k < g.K) v = *reinterpret_cast<const V*>(A + (int64_t)row * g.lda + k);
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < NBP; ++i) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int k = k0 + 2 * (b_p0 + i * B_PSTEP) + e;
                V v = V(0.0);
                if (b_col_ok && k < g.K) v = *reinterpret_cast<const V*>(B + (int64_t)k * g.ldb + n0 + b_c);
                rb[i][e] = v;
            }
        }
    };

    auto sstore = [&](int buf) {
        double* As = smem + buf * STAGE;
        double* Bs = As + A_ELEMS;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            *reinterpret_cast<V*>(As + (a_r0 + i * A_RSTEP) * SA + a_k) = ra[i];
#pragma unroll
        for (int i = 0; i < NBP; ++i) {
            double* dst = Bs + (b_p0 + i * B_PSTEP) * SBP + b_c * 2;
            if constexpr (VEC == 2) {
                v2d lo = {rb[i][0][0], rb[i][1][0]};
                v2d hi = {rb[i][0][1], rb[i][1][1]};
                *reinterpret_cast<v2d*>(dst) = lo;
                *reinterpret_cast<v2d*>(dst + 2) = hi;
            } else {
                v2d p = {rb[i][0], rb[i][1]};
                *reinterpret_cast<v2d*>(dst) = p;
            }
        }
    };

    v4d acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (v4d){0.0, 0.0, 0.0, 0.0};

    auto compute = [&](int buf) {
        const double* As = smem + buf * STAGE + (wm * 64 + r16) * SA + 2 * g4;
        const double* Bs = smem + buf * STAGE + A_ELEMS + g4 * SBP + (wn * 64 + r16) * 2;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            v2d a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const v2d*>(As + i * 16 * SA + 8 * q);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const v2d*>(Bs + 4 * q * SBP + j * 32);
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i][e], b[j][e], acc[i][j], 0, 0, 0);
        }
    };

    const int KT = (g.K + BK - 1) / BK;
    gload(0);
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) gload((kt + 1) * BK);
        compute(cur);
        if (more) sstore(cur ^ 1);
        __syncthreads();
    }

    // ---- store: accumulator v of lane (r16, g4) in MFMA tile (i, j) is C[16 i + g4 + 4 v][16 j + r16] ----
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = m0 + wm * 64 + i * 16 + g4 + 4 * v;
            if (row < g.M) {
                double* crow = C + (int64_t)row * g.ldc + n0 + wn * 64 + r16;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n0 + wn * 64 + j * 16 + r16 < g.N) crow[j * 16] = acc[i][j][v];
            }
        }
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t launch_leaf_gemm(int64_t m, int64_t batch, Mat a, Mat b, Mat c, hipStream_t s)
{
    if (m == 0 || batch == 0) return hipSuccess;
    GemmArgs g;
    g.A = a.p; g.B = b.p; g.C = c.p;
    g.lda = a.ld; g.ldb = b.ld; g.ldc = c.ld;
    g.sa = a.stride; g.sb = b.stride; g.sc = c.stride;
    g.M = g.N = g.K = (int)m;
    g.tiles_m = (int)((m + BM - 1) / BM);
    g.tiles_n = (int)((m + BN - 1) / BN);
    const int64_t blocks = (int64_t)g.tiles_m * g.tiles_n * batch;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool v2 = (m % 2 == 0) && aligned16(a.p) && aligned16(b.p) && a.ld % 2 == 0 && b.ld % 2 == 0 &&
                    a.stride % 2 == 0 && b.stride % 2 == 0;
    if (v2) hipLaunchKernelGGL((leaf_gemm_kernel<2>), dim3((unsigned)blocks), dim3(NT), 0, s, g);
    else    hipLaunchKernelGGL((leaf_gemm_kernel<1>), dim3((unsigned)blocks), dim3(NT), 0, s, g);
    return hipGetLastError();
}

}  // namespace sw
