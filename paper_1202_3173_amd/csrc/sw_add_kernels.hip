// Streaming kernels of the Strassen-Winograd step: the pre-additions that form the T and S operands, the
// post-additions that turn the seven products into the four quadrants of C (Appendix A), the element-wise
// pieces of a DFS step, and the zero-padded copy.  All are HBM-bound: every kernel reads each input element
// once and writes each output element once, with 16-byte accesses when alignment allows (8-byte otherwise) and
// non-temporal hints (every operand is far larger than the caches and is next touched by another kernel).
//
// Thread layout, common to all kernels: threadIdx.x walks columns in units of VEC doubles, blockIdx.y walks
// groups of ROWS rows, blockIdx.z is the matrix of the batch.  Adjacent lanes touch adjacent addresses, so a
// wavefront reads and writes whole 512- or 1024-byte row segments.
#include "sw_internal.h"

namespace sw {
namespace {

constexpr int NT = 256;                  // threads per block
constexpr int ROWS = 2;                  // rows per thread (independent loads in flight)
constexpr int POST_ROWS = 2;
constexpr int PAD_ROWS = 8;              // rows per thread of the pad / crop copy

// Every kernel below walks a LOGICAL grid (column chunks x row groups x matrices) with however many
// workgroups it was launched with: workgroup b takes logical blocks b, b + gridDim.x, ...  Launched with the
// full grid this is the ordinary one-block-per-workgroup kernel; launched with a few hundred workgroups it is
// a persistent streaming kernel that leaves most of every CU to the leaf products running beside it.
struct LGrid { unsigned gx, gy, gz; };
#define SW_LOGICAL_BLOCKS(lg)                                                                        \
    for (unsigned long long w_ = blockIdx.x, n_ = (unsigned long long)(lg).gx * (lg).gy * (lg).gz; w_ < n_; \
         w_ += gridDim.x)
#define SW_DECODE_BLOCK(lg)                                       \
    const unsigned bx = (unsigned)(w_ % (lg).gx);                 \
    const unsigned long long t_ = w_ / (lg).gx;                   \
    const unsigned by = (unsigned)(t_ % (lg).gy);                 \
    const unsigned bz = (unsigned)(t_ / (lg).gy);                 \
    (void)bz;

template <int VEC> struct VecT;
template <> struct VecT<1> { typedef double type; };
template <> struct VecT<2> { typedef double __attribute__((ext_vector_type(2))) type; };

template <int VEC>
__device__ __forceinline__ typename VecT<VEC>::type ld(const double* p)
{
    // streaming data: nothing here is read again before it has left every cache
    return __builtin_nontemporal_load(reinterpret_cast<const typename VecT<VEC>::type*>(p));
}
template <int VEC>
__device__ __forceinline__ void st(double* p, typename VecT<VEC>::type v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<typename VecT<VEC>::type*>(p));
}

// ---- BFS pre-additions ------------------------------------------------------------------------------------
// SIDE 0: T0 = A11, T1 = A12, T2 = A21 + A22, T3 = T2 - A11, T4 = A11 - A21, T5 = A12 - T3, T6 = A22
// SIDE 1: S0 = B11, S1 = B21, S2 = B12 - B11, S3 = B22 - S2, S4 = B22 - B12, S5 = B22, S6 = S3 - B21
// copies != 0: all seven operands are written, child j of parent p in slot 7p + j.  copies == 0: only the four
// that need arithmetic (T2, T3, T4, T5 or S2, S3, S4, S6) are written, to slots 4p + 0..3; the plain quadrants
// are then used in place by the caller.
template <int SIDE, int VEC>
__global__ void __launch_bounds__(NT)
pre_add_kernel(const double* __restrict__ parent, int64_t pld, int64_t pstride, int hr, int hc,
               double* __restrict__ child, int64_t cld, int64_t cstride, int copies, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            typedef typename VecT<VEC>::type V;
            const int cx = (bx * NT + threadIdx.x) * VEC;
            if (cx >= hc) return;
            const int r0 = by * ROWS;
            const double* P = parent + (int64_t)bz * pstride;
            double* O = child + (int64_t)bz * (copies ? 7 : 4) * cstride;
    
            V q11[ROWS], q12[ROWS], q21[ROWS], q22[ROWS];
        #pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int row = r0 + r;
                if (row < hr) {
                    const double* top = P + (int64_t)row * pld + cx;
                    const double* bot = P + (int64_t)(row + hr) * pld + cx;
                    q11[r] = ld<VEC>(top);
                    q12[r] = ld<VEC>(top + hc);
                    q21[r] = ld<VEC>(bot);
                    q22[r] = ld<VEC>(bot + hc);
                }
            }
        #pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int row = r0 + r;
                if (row < hr) {
                    double* o = O + (int64_t)row * cld + cx;
                    if (SIDE == 0) {
                        const V t2 = q21[r] + q22[r];
                        const V t3 = t2 - q11[r];
                        const V t4 = q11[r] - q21[r];
                        const V t5 = q12[r] - t3;
                        if (copies) {
                            st<VEC>(o, q11[r]);
                            st<VEC>(o + cstride, q12[r]);
                            st<VEC>(o + 6 * cstride, q22[r]);
                            o += 2 * cstride;
                        }
                        st<VEC>(o, t2);
                        st<VEC>(o + cstride, t3);
                        st<VEC>(o + 2 * cstride, t4);
                        st<VEC>(o + 3 * cstride, t5);
                    } else {
                        const V s2 = q12[r] - q11[r];
                        const V s3 = q22[r] - s2;
                        const V s4 = q22[r] - q12[r];
                        const V s6 = s3 - q21[r];
                        if (copies) {
                            st<VEC>(o, q11[r]);
                            st<VEC>(o + cstride, q21[r]);
                            st<VEC>(o + 2 * cstride, s2);
                            st<VEC>(o + 3 * cstride, s3);
                            st<VEC>(o + 4 * cstride, s4);
                            st<VEC>(o + 5 * cstride, q22[r]);
                            st<VEC>(o + 6 * cstride, s6);
                        } else {
                            st<VEC>(o, s2);
                            st<VEC>(o + cstride, s3);
                            st<VEC>(o + 2 * cstride, s4);
                            st<VEC>(o + 3 * cstride, s6);
                        }
                    }
                }
            }
        }();
    }
}

// ---- BFS post-additions -----------------------------------------------------------------------------------
// U1 = Q0 + Q3, U2 = U1 + Q4, U3 = U1 + Q2, C11 = Q0 + Q1, C12 = U3 + Q5, C21 = U2 - Q6, C22 = U2 + Q2
template <int VEC>
__global__ void __launch_bounds__(NT)
post_add_kernel(const double* __restrict__ Q, int64_t qld, int64_t qstride, int hr, int hc,
                double* __restrict__ parent, int64_t pld, int64_t pstride, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            typedef typename VecT<VEC>::type V;
            constexpr int R = POST_ROWS;
            const int cx = (bx * NT + threadIdx.x) * VEC;
            if (cx >= hc) return;
            const int r0 = by * R;
            const double* q = Q + (int64_t)bz * 7 * qstride;
            double* P = parent + (int64_t)bz * pstride;
    
            V v[R][7];
        #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = r0 + r;
                if (row < hr) {
        #pragma unroll
                    for (int j = 0; j < 7; ++j) v[r][j] = ld<VEC>(q + j * qstride + (int64_t)row * qld + cx);
                }
            }
        #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = r0 + r;
                if (row < hr) {
                    const V u1 = v[r][0] + v[r][3];
                    const V u2 = u1 + v[r][4];
                    const V u3 = u1 + v[r][2];
                    double* top = P + (int64_t)row * pld + cx;
                    double* bot = P + (int64_t)(row + hr) * pld + cx;
                    st<VEC>(top, v[r][0] + v[r][1]);
                    st<VEC>(top + hc, u3 + v[r][5]);
                    st<VEC>(bot, u2 - v[r][6]);
                    st<VEC>(bot + hc, u2 + v[r][2]);
                }
            }
        }();
    }
}

// ---- element-wise pieces of a DFS step ------------------------------------------------------------------------

struct EwOp {
    double* z;
    const double* x;
    const double* y;
    int64_t zld, xld, yld;
    int64_t zstride, xstride, ystride;
    int sign;
};

// NOPS independent operations Z = X + sign * Y; blockIdx.z = op * live + matrix.  Z may alias X or Y
// exactly (same element, same thread), so no __restrict__ here.
template <int VEC, int NOPS>
__global__ void __launch_bounds__(NT)
ew_kernel(EwOp op0, EwOp op1, int live, int hr, int hc, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            typedef typename VecT<VEC>::type V;
            const int cx = (bx * NT + threadIdx.x) * VEC;
            if (cx >= hc) return;
            const int r0 = by * ROWS;
            int b = bz;
            const bool second = NOPS == 2 && b >= live;
            if (second) b -= live;
            const EwOp& op = second ? op1 : op0;
            double* z = op.z + (int64_t)b * op.zstride;
            const double* x = op.x + (int64_t)b * op.xstride;
            const double* y = op.y + (int64_t)b * op.ystride;
            V xv[ROWS], yv[ROWS];
        #pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int row = r0 + r;
                if (row < hr) {
                    xv[r] = ld<VEC>(x + (int64_t)row * op.xld + cx);
                    yv[r] = ld<VEC>(y + (int64_t)row * op.yld + cx);
                }
            }
        #pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int row = r0 + r;
                if (row < hr) st<VEC>(z + (int64_t)row * op.zld + cx, op.sign > 0 ? xv[r] + yv[r] : xv[r] - yv[r]);
            }
        }();
    }
}

// With X = Q0, C12 = Q3, C21 = Q4, C22 = Q2, C11 = Q5:
//   U1 = X + C12, U2 = U1 + C21, U3 = U1 + C22, C22 <- U2 + C22, C12 <- U3 + C11, C21 <- U2
// (Appendix A column 4 in its printed association; C21 still lacks - Q6 and C11 is rewritten later).
template <int VEC>
__global__ void __launch_bounds__(NT)
dfs_post_kernel(const double* x, int64_t xld, int64_t xstride, const double* c11, double* c12, double* c21,
                double* c22, int64_t cld, int64_t cstride, int hr, int hc, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            typedef typename VecT<VEC>::type V;
            constexpr int R = 2;
            const int cx = (bx * NT + threadIdx.x) * VEC;
            if (cx >= hc) return;
            const int r0 = by * R;
            const int64_t boff = (int64_t)bz * cstride;
            const double* xb = x + (int64_t)bz * xstride;
            V q0[R], q5[R], q3[R], q4[R], q2[R];
        #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = r0 + r;
                if (row < hr) {
                    const int64_t o = boff + (int64_t)row * cld + cx;
                    q0[r] = ld<VEC>(xb + (int64_t)row * xld + cx);
                    q5[r] = ld<VEC>(c11 + o);
                    q3[r] = ld<VEC>(c12 + o);
                    q4[r] = ld<VEC>(c21 + o);
                    q2[r] = ld<VEC>(c22 + o);
                }
            }
        #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = r0 + r;
                if (row < hr) {
                    const int64_t o = boff + (int64_t)row * cld + cx;
                    const V u1 = q0[r] + q3[r];
                    const V u2 = u1 + q4[r];
                    const V u3 = u1 + q2[r];
                    st<VEC>(c22 + o, u2 + q2[r]);
                    st<VEC>(c12 + o, u3 + q5[r]);
                    st<VEC>(c21 + o, u2);
                }
            }
        }();
    }
}

// ---- two BFS steps in one pass ------------------------------------------------------------------------------------
// When two BFS steps follow each other, the operands of the 49 grandchildren are formed straight from the
// parent: the parent is a 4 x 4 grid of m x m blocks a[R][C]; the first step's T_j (a 2 x 2 block matrix) has
// blocks T_j[p][q] = f_j(a[p][q], a[p][2+q], a[2+p][q], a[2+p][2+q]) and the second step gives
// T_{j,i} = f_i(T_j[0][0], T_j[0][1], T_j[1][0], T_j[1][1]), with f the seven combinations of Appendix A in
// their printed association.  The 28 intermediate blocks live in registers only, so the values are the same
// bits as two separate steps while the intermediate operands are never written to or read from HBM.
template <int SIDE, typename V>
__device__ __forceinline__ void winograd_pre(const V x11, const V x12, const V x21, const V x22, V (&o)[7])
{
    if (SIDE == 0) {            // T0..T6 from A's quadrants
        const V t2 = x21 + x22;
        const V t3 = t2 - x11;
        o[0] = x11; o[1] = x12; o[2] = t2; o[3] = t3; o[4] = x11 - x21; o[5] = x12 - t3; o[6] = x22;
    } else {                    // S0..S6 from B's quadrants
        const V s2 = x12 - x11;
        const V s3 = x22 - s2;
        o[0] = x11; o[1] = x21; o[2] = s2; o[3] = s3; o[4] = x22 - x12; o[5] = x22; o[6] = s3 - x21;
    }
}

template <int SIDE, int VEC>
__global__ void __launch_bounds__(NT)
pre_add2_kernel(const double* __restrict__ parent, int64_t pld, int64_t pstride, int mr, int mc,
                double* __restrict__ child, int64_t cld, int64_t cstride, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            typedef typename VecT<VEC>::type V;
            const int cx = (bx * NT + threadIdx.x) * VEC;
            const int row = by;
            if (cx >= mc) return;
            const double* P = parent + (int64_t)bz * pstride + (int64_t)row * pld + cx;
            double* O = child + (int64_t)bz * 49 * cstride + (int64_t)row * cld + cx;
    
            V a[4][4];
        #pragma unroll
            for (int R = 0; R < 4; ++R)
        #pragma unroll
                for (int C = 0; C < 4; ++C) a[R][C] = ld<VEC>(P + (int64_t)R * mr * pld + C * mc);
    
            V t[4][7];   // t[2p+q][j] = T_j[p][q]
        #pragma unroll
            for (int p = 0; p < 2; ++p)
        #pragma unroll
                for (int q = 0; q < 2; ++q) winograd_pre<SIDE, V>(a[p][q], a[p][2 + q], a[2 + p][q], a[2 + p][2 + q], t[2 * p + q]);
        #pragma unroll
            for (int j = 0; j < 7; ++j) {
                V o[7];
                winograd_pre<SIDE, V>(t[0][j], t[1][j], t[2][j], t[3][j], o);
        #pragma unroll
                for (int i = 0; i < 7; ++i) st<VEC>(O + (int64_t)(j * 7 + i) * cstride, o[i]);
            }
        }();
    }
}

// The reverse for the products: q[j][i] are the 49 grandchild products; Q_j[p][q] is the post-addition of
// q[j][0..6] (Appendix A, fourth column) and the parent's block c[2X+p][2Y+q] the same post-addition over j.
template <int VEC>
__global__ void __launch_bounds__(NT)
post_add2_kernel(const double* __restrict__ Q, int64_t qld, int64_t qstride, int mr, int mc,
                 double* __restrict__ parent, int64_t pld, int64_t pstride, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            typedef typename VecT<VEC>::type V;
            const int cx = (bx * NT + threadIdx.x) * VEC;
            const int row = by;
            if (cx >= mc) return;
            const double* q = Q + (int64_t)bz * 49 * qstride + (int64_t)row * qld + cx;
            double* P = parent + (int64_t)bz * pstride + (int64_t)row * pld + cx;
    
            // Q_j as four blocks [11, 12, 21, 22] from the seven products of child j
            auto child = [&](int j, V (&out)[4]) __attribute__((always_inline)) {
                V v[7];
        #pragma unroll
                for (int i = 0; i < 7; ++i) v[i] = ld<VEC>(q + (int64_t)(j * 7 + i) * qstride);
                const V u1 = v[0] + v[3];
                const V u2 = u1 + v[4];
                const V u3 = u1 + v[2];
                out[0] = v[0] + v[1];
                out[1] = u3 + v[5];
                out[2] = u2 - v[6];
                out[3] = u2 + v[2];
            };
            // store the four blocks of the parent's quadrant (X, Y)
            auto put = [&](int X, int Y, const V (&c)[4]) __attribute__((always_inline)) {
        #pragma unroll
                for (int pq = 0; pq < 4; ++pq)
                    st<VEC>(P + (int64_t)(2 * X + (pq >> 1)) * mr * pld + (2 * Y + (pq & 1)) * mc, c[pq]);
            };
    
            V q0[4], q3[4], u1[4], u2[4], u3[4], t[4], c[4];
            child(0, q0);
            child(3, q3);
        #pragma unroll
            for (int k = 0; k < 4; ++k) u1[k] = q0[k] + q3[k];          // U1 = Q0 + Q3
            child(1, t);
        #pragma unroll
            for (int k = 0; k < 4; ++k) c[k] = q0[k] + t[k];            // C11 = Q0 + Q1
            put(0, 0, c);
            child(4, t);
        #pragma unroll
            for (int k = 0; k < 4; ++k) u2[k] = u1[k] + t[k];           // U2 = U1 + Q4
            child(2, t);
        #pragma unroll
            for (int k = 0; k < 4; ++k) { u3[k] = u1[k] + t[k]; c[k] = u2[k] + t[k]; }   // U3 = U1 + Q2, C22 = U2 + Q2
            put(1, 1, c);
            child(5, t);
        #pragma unroll
            for (int k = 0; k < 4; ++k) c[k] = u3[k] + t[k];            // C12 = U3 + Q5
            put(0, 1, c);
            child(6, t);
        #pragma unroll
            for (int k = 0; k < 4; ++k) c[k] = u2[k] - t[k];            // C21 = U2 - Q6
            put(1, 0, c);
        }();
    }
}

// ---- zero-padded copy ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NT)
pad_copy_kernel(const double* __restrict__ src, int64_t sld, int rows, int cols, double* __restrict__ dst,
                int64_t dld, int prows, int pcols, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            const int c = bx * NT + threadIdx.x;
            if (c >= pcols) return;
            const int r0 = by * PAD_ROWS;
        #pragma unroll
            for (int r = 0; r < PAD_ROWS; ++r) {
                const int row = r0 + r;
                if (row < prows) {
                    const double v = (row < rows && c < cols) ? src[(int64_t)row * sld + c] : 0.0;
                    dst[(int64_t)row * dld + c] = v;
                }
            }
        }();
    }
}

// ---- dense copies of thin strips ------------------------------------------------------------------------------------
// dst_b (rows x cols, pitch dld) = src_b (pitch sld) for every matrix b of the batch: the peeled column of an A and the
// peeled row of a B are set aside with it, so that the operands themselves are free again before the update that
// uses the strips runs.
__global__ void __launch_bounds__(NT)
strip_copy_kernel(const double* __restrict__ src, int64_t sld, int64_t sstride, int rows, int cols, double* __restrict__ dst,
                  int64_t dld, int64_t dstride, LGrid lg)
{
    SW_LOGICAL_BLOCKS(lg) {
        SW_DECODE_BLOCK(lg)
        [=]() {
            const int c = bx * NT + threadIdx.x;
            if (c >= cols) return;
            const int r0 = by * PAD_ROWS;
            const double* S = src + (int64_t)bz * sstride;
            double* D = dst + (int64_t)bz * dstride;
        #pragma unroll
            for (int r = 0; r < PAD_ROWS; ++r) {
                const int row = r0 + r;
                if (row < rows) D[(int64_t)row * dld + c] = S[(int64_t)row * sld + c];
            }
        }();
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool even(int64_t v) { return (v & 1) == 0; }
inline bool mat_vec2(const Mat& m) { return aligned16(m.p) && even(m.ld) && even(m.stride); }

// logical grid for `batch` matrices of hr x hc: column chunks of NT * vec, groups of `rows` rows
inline LGrid grid_for(int64_t hr, int64_t hc, int vec, int rows, int64_t batch)
{
    const int64_t chunks = (hc + vec - 1) / vec;
    return LGrid{(unsigned)((chunks + NT - 1) / NT), (unsigned)((hr + rows - 1) / rows), (unsigned)batch};
}

// 0: one workgroup per logical block; else at most this many workgroups per launch.  Per host thread, so that
// two threads inside the library at once do not change each other's launches.
static thread_local int g_block_cap = 0;

inline dim3 physical(const LGrid& lg)
{
    const unsigned long long total = (unsigned long long)lg.gx * lg.gy * lg.gz;
    const unsigned long long cap = g_block_cap > 0 ? (unsigned long long)g_block_cap : 0x7fffffffULL;
    return dim3((unsigned)(total < cap ? total : cap));
}

}  // namespace

void set_add_block_cap(int cap) { g_block_cap = cap; }

hipError_t launch_pre_add(int side, Mat parent, int64_t live, int64_t hr, int64_t hc, Mat child, bool copies, hipStream_t s)
{
    if (live == 0 || hr == 0 || hc == 0) return hipSuccess;
    if (Tracer* t = tracer())
        return t->kernel(Tracer::K_PRE_ADD, s, {fp(parent, 2 * hr, 2 * hc, live)}, {fp(child, hr, hc, (copies ? 7 : 4) * live)});
    const bool v2 = even(hc) && mat_vec2(parent) && mat_vec2(child);
    const LGrid lg = grid_for(hr, hc, v2 ? 2 : 1, ROWS, live);
#define SW_LAUNCH(SIDE, VEC)                                                                              \
    hipLaunchKernelGGL((pre_add_kernel<SIDE, VEC>), physical(lg), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, \
                       (int)hr, (int)hc, child.p, child.ld, child.stride, copies ? 1 : 0, lg)
    if (side == 0) { if (v2) SW_LAUNCH(0, 2); else SW_LAUNCH(0, 1); }
    else           { if (v2) SW_LAUNCH(1, 2); else SW_LAUNCH(1, 1); }
#undef SW_LAUNCH
    return hipGetLastError();
}

hipError_t launch_post_add(Mat q, int64_t live, int64_t hr, int64_t hc, Mat parent, hipStream_t s)
{
    if (live == 0 || hr == 0 || hc == 0) return hipSuccess;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_POST_ADD, s, {fp(q, hr, hc, 7 * live)}, {fp(parent, 2 * hr, 2 * hc, live)});
    const bool v2 = even(hc) && mat_vec2(parent) && mat_vec2(q);
    const LGrid lg = grid_for(hr, hc, v2 ? 2 : 1, POST_ROWS, live);
    if (v2)
        hipLaunchKernelGGL((post_add_kernel<2>), physical(lg), dim3(NT), 0, s, q.p, q.ld, q.stride, (int)hr, (int)hc, parent.p,
                           parent.ld, parent.stride, lg);
    else
        hipLaunchKernelGGL((post_add_kernel<1>), physical(lg), dim3(NT), 0, s, q.p, q.ld, q.stride, (int)hr, (int)hc, parent.p,
                           parent.ld, parent.stride, lg);
    return hipGetLastError();
}

hipError_t launch_pre_add2(int side, Mat parent, int64_t live, int64_t mr, int64_t mc, Mat child, hipStream_t s)
{
    if (live == 0 || mr == 0 || mc == 0) return hipSuccess;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_PRE_ADD2, s, {fp(parent, 4 * mr, 4 * mc, live)}, {fp(child, mr, mc, 49 * live)});
    const bool v2 = even(mc) && mat_vec2(parent) && mat_vec2(child);
    const LGrid lg = grid_for(mr, mc, v2 ? 2 : 1, 1, live);
#define SW_LAUNCH(SIDE, VEC)                                                                               \
    hipLaunchKernelGGL((pre_add2_kernel<SIDE, VEC>), physical(lg), dim3(NT), 0, s, parent.p, parent.ld, parent.stride, \
                       (int)mr, (int)mc, child.p, child.ld, child.stride, lg)
    if (side == 0) { if (v2) SW_LAUNCH(0, 2); else SW_LAUNCH(0, 1); }
    else           { if (v2) SW_LAUNCH(1, 2); else SW_LAUNCH(1, 1); }
#undef SW_LAUNCH
    return hipGetLastError();
}

hipError_t launch_post_add2(Mat q, int64_t live, int64_t mr, int64_t mc, Mat parent, hipStream_t s)
{
    if (live == 0 || mr == 0 || mc == 0) return hipSuccess;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_POST_ADD2, s, {fp(q, mr, mc, 49 * live)}, {fp(parent, 4 * mr, 4 * mc, live)});
    const bool v2 = even(mc) && mat_vec2(parent) && mat_vec2(q);
    const LGrid lg = grid_for(mr, mc, v2 ? 2 : 1, 1, live);
    if (v2)
        hipLaunchKernelGGL((post_add2_kernel<2>), physical(lg), dim3(NT), 0, s, q.p, q.ld, q.stride, (int)mr, (int)mc, parent.p,
                           parent.ld, parent.stride, lg);
    else
        hipLaunchKernelGGL((post_add2_kernel<1>), physical(lg), dim3(NT), 0, s, q.p, q.ld, q.stride, (int)mr, (int)mc, parent.p,
                           parent.ld, parent.stride, lg);
    return hipGetLastError();
}

static EwOp make_op(Mat z, Mat x, Mat y, int sign)
{
    return EwOp{z.p, x.p, y.p, z.ld, x.ld, y.ld, z.stride, x.stride, y.stride, sign};
}

hipError_t launch_ew(Mat z, Mat x, Mat y, int sign, int64_t live, int64_t hr, int64_t hc, hipStream_t s)
{
    if (live == 0 || hr == 0 || hc == 0) return hipSuccess;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_EW, s, {fp(x, hr, hc, live), fp(y, hr, hc, live)}, {fp(z, hr, hc, live)});
    const bool v2 = even(hc) && mat_vec2(z) && mat_vec2(x) && mat_vec2(y);
    const LGrid lg = grid_for(hr, hc, v2 ? 2 : 1, ROWS, live);
    const EwOp op = make_op(z, x, y, sign);
    if (v2) hipLaunchKernelGGL((ew_kernel<2, 1>), physical(lg), dim3(NT), 0, s, op, op, (int)live, (int)hr, (int)hc, lg);
    else    hipLaunchKernelGGL((ew_kernel<1, 1>), physical(lg), dim3(NT), 0, s, op, op, (int)live, (int)hr, (int)hc, lg);
    return hipGetLastError();
}

hipError_t launch_ew2(Mat z0, Mat x0, Mat y0, int sign0, Mat z1, Mat x1, Mat y1, int sign1, int64_t live,
                      int64_t hr, int64_t hc, hipStream_t s)
{
    if (live == 0 || hr == 0 || hc == 0) return hipSuccess;
    if (Tracer* t = tracer())
        return t->kernel(Tracer::K_EW, s, {fp(x0, hr, hc, live), fp(y0, hr, hc, live), fp(x1, hr, hc, live), fp(y1, hr, hc, live)},
                         {fp(z0, hr, hc, live), fp(z1, hr, hc, live)});
    const bool v2 = even(hc) && mat_vec2(z0) && mat_vec2(x0) && mat_vec2(y0) && mat_vec2(z1) && mat_vec2(x1) &&
                    mat_vec2(y1);
    const LGrid lg = grid_for(hr, hc, v2 ? 2 : 1, ROWS, 2 * live);
    const EwOp a = make_op(z0, x0, y0, sign0), b = make_op(z1, x1, y1, sign1);
    if (v2) hipLaunchKernelGGL((ew_kernel<2, 2>), physical(lg), dim3(NT), 0, s, a, b, (int)live, (int)hr, (int)hc, lg);
    else    hipLaunchKernelGGL((ew_kernel<1, 2>), physical(lg), dim3(NT), 0, s, a, b, (int)live, (int)hr, (int)hc, lg);
    return hipGetLastError();
}

hipError_t launch_dfs_post(Mat x, Mat c11, Mat c12, Mat c21, Mat c22, int64_t live, int64_t hr, int64_t hc, hipStream_t s)
{
    if (live == 0 || hr == 0 || hc == 0) return hipSuccess;
    if (Tracer* t = tracer())
        return t->kernel(Tracer::K_DFS_POST, s,
                         {fp(x, hr, hc, live), fp(c11, hr, hc, live), fp(c12, hr, hc, live), fp(c21, hr, hc, live), fp(c22, hr, hc, live)},
                         {fp(c12, hr, hc, live), fp(c21, hr, hc, live), fp(c22, hr, hc, live)});
    // the four quadrants share ld and stride by construction
    const bool v2 = even(hc) && mat_vec2(x) && mat_vec2(c11) && mat_vec2(c12) && mat_vec2(c21) && mat_vec2(c22);
    const LGrid lg = grid_for(hr, hc, v2 ? 2 : 1, 2, live);
    if (v2)
        hipLaunchKernelGGL((dfs_post_kernel<2>), physical(lg), dim3(NT), 0, s, x.p, x.ld, x.stride, c11.p, c12.p, c21.p,
                           c22.p, c11.ld, c11.stride, (int)hr, (int)hc, lg);
    else
        hipLaunchKernelGGL((dfs_post_kernel<1>), physical(lg), dim3(NT), 0, s, x.p, x.ld, x.stride, c11.p, c12.p, c21.p,
                           c22.p, c11.ld, c11.stride, (int)hr, (int)hc, lg);
    return hipGetLastError();
}

hipError_t launch_pad_copy(const double* src, int64_t src_ld, int64_t rows, int64_t cols, double* dst,
                           int64_t dst_ld, int64_t prows, int64_t pcols, hipStream_t s)
{
    if (prows == 0 || pcols == 0) return hipSuccess;
    if (Tracer* t = tracer()) {
        const int64_t r = rows < prows ? rows : prows, c = cols < pcols ? cols : pcols;
        const Footprint out{dst, prows, pcols, dst_ld, 1, 0};
        if (r > 0 && c > 0) return t->kernel(Tracer::K_PAD_COPY, s, {Footprint{src, r, c, src_ld, 1, 0}}, {out});
        return t->kernel(Tracer::K_PAD_COPY, s, {}, {out});
    }
    const LGrid lg{(unsigned)((pcols + NT - 1) / NT), (unsigned)((prows + PAD_ROWS - 1) / PAD_ROWS), 1u};
    hipLaunchKernelGGL(pad_copy_kernel, physical(lg), dim3(NT), 0, s, src, src_ld, (int)rows, (int)cols, dst, dst_ld,
                       (int)prows, (int)pcols, lg);
    return hipGetLastError();
}

hipError_t launch_strip_copy(Mat src, int64_t rows, int64_t cols, Mat dst, int64_t live, hipStream_t s)
{
    if (live == 0 || rows == 0 || cols == 0) return hipSuccess;
    if (Tracer* t = tracer()) return t->kernel(Tracer::K_PAD_COPY, s, {fp(src, rows, cols, live)}, {fp(dst, rows, cols, live)});
    const LGrid lg{(unsigned)((cols + NT - 1) / NT), (unsigned)((rows + PAD_ROWS - 1) / PAD_ROWS), (unsigned)live};
    hipLaunchKernelGGL(strip_copy_kernel, physical(lg), dim3(NT), 0, s, src.p, src.ld, src.stride, (int)rows, (int)cols, dst.p, dst.ld,
                       dst.stride, lg);
    return hipGetLastError();
}

}  // namespace sw
