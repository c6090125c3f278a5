/*
 * sw_gemm.h -- C ABI of the MI355X (gfx950) Strassen-Winograd fp64 matrix multiply.
 *
 * The library computes C = A*B (Algorithm 1: Require A, B n x n; Ensure C = A*B)
 * by walking the 7-way recursion tree of the Strassen-Winograd step (Appendix A)
 * with a caller-chosen or planned order of BFS steps (all seven subproblems in
 * flight, Section 3.3) and DFS steps (subproblems in sequence, Section 3.4), and
 * classical fp64 leaf products below the cutoff (Section 5.4.1).
 *
 * Conventions for every call
 *   - matrices are fp64, row-major; pointers named A, B, C, T, S, Q, X, ... are
 *     DEVICE pointers; `const char*`, `char*`, `int64_t*`, `double* ms` are HOST pointers;
 *   - the caller owns every buffer, the library never allocates or frees device memory;
 *   - work is enqueued on the stream given to sw_set_stream (default: the null
 *     stream) without host synchronisation; results are valid after the caller
 *     synchronises that stream;
 *   - return value 0 = SW_OK, negative = error; sw_last_error() gives the text of
 *     the calling thread's last failure.
 *   - a schedule is a string of `levels` characters, 'B' (BFS step) or 'D' (DFS
 *     step), top level of the tree first; NULL or "" asks the planner.
 * Calls that share one workspace must not overlap in time; see sw_gemm_ex for what concurrent host threads may do.
 */
#ifndef SW_GEMM_H
#define SW_GEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SW_OK 0
#define SW_EINVAL (-1) /* bad argument: n < 0, levels < 0 or > SW_MAX_LEVELS, 2^levels > n, NULL pointer,
                          schedule of wrong length or with a character other than B/D, C overlapping A or B */
#define SW_ENOMEM (-2) /* workspace missing or smaller than sw_plan_memory says; no schedule fits the budget */
#define SW_EHIP (-3)   /* a HIP call failed; text in sw_last_error() */

#define SW_MAX_LEVELS 16

/* ---- the product (Algorithm 1; Appendix A; Sections 3.3, 3.4) ------------------------------------------- */

/* C = A*B, all n x n with leading dimension n.  `levels` Strassen-Winograd steps, then classical leaves of
 * size ceil(n / 2^levels).  levels = 0 is one classical product; levels < 0 leaves the depth to the library
 * (sw_plan_levels for the workspace that is set; schedule is then ignored).  If n is not a multiple of 2^levels the
 * operands are zero-padded into workspace copies of the next multiple (Section 3.1 allows padding).
 * A and B are read only; C is overwritten; C must not overlap A or B.  Uses the workspace and stream set by
 * sw_set_workspace / sw_set_stream.  schedule NULL or "": the planner's choice for the current workspace
 * size (sw_plan_schedule with budget = workspace bytes). */
int sw_gemm(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule);

/* Same with explicit leading dimensions, workspace and stream.  Of the library's state only the process-wide
 * settings are read, once on entry: sw_set_overlap, sw_set_odd_mode, sw_profile_enable (a setter called meanwhile
 * affects later calls only).  Host threads may call concurrently with distinct workspaces and distinct streams:
 * every call takes its own set of internal streams and events for its duration, the workgroup cap of the
 * addition kernels belongs to the calling thread, and the profiling record is locked.  (sw_gemm and the other
 * calls that use sw_set_workspace / sw_set_stream share that one workspace and are not for concurrent use.)
 * lda <= 4227329 and ldb <= 35791385 (the product kernel addresses a tile with 32-bit byte offsets); beyond:
 * SW_EINVAL.  workspace: DEVICE pointer, 256-byte aligned, workspace_bytes >= sw_plan_memory(n, levels, schedule). */
int sw_gemm_ex(int64_t n, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
               int levels, const char* schedule, void* workspace, int64_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): sw_gemm_ex with the workspace taken from an array of SW_STATIC_SCRATCH_BYTES that is part
 * of the library's device image (every GPU the library runs on holds its own copy until the process ends).  The
 * call allocates nothing: no hipMalloc or hipFree, no streams, no events.  Everything runs on `hip_stream` (the
 * one-stream executor); sw_set_overlap, sw_set_odd_mode and sw_profile_enable do not apply (odd n is zero-padded
 * inside the scratch).  schedule NULL or "": the planner's choice for SW_STATIC_SCRATCH_BYTES; levels < 0: the
 * depth by the cost model for that size.  Same arguments, results (bit for bit) and errors as sw_gemm_ex;
 * SW_ENOMEM, before anything is enqueued, when the product at this depth and step order needs more than the
 * scratch holds (the all-DFS order of sw_plan_memory is the least: n = 4096 at three levels takes 90 MB).
 * All calls on one GPU share that GPU's array: nothing in it needs clearing between calls (every buffer is
 * written before it is read), but two calls that overlap in time on one GPU race, whatever their streams. */
#define SW_STATIC_SCRATCH_BYTES (128 * 1024 * 1024)
int sw_gemm_static(int64_t n, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                   int levels, const char* schedule, void* hip_stream);

/* The same recursion on a rectangular product: C (M x N) = A (M x K) * B (K x N), row-major with leading
 * dimensions lda >= K, ldb >= N, ldc >= N.  Every step halves all three extents: the operands T are
 * M/2 x K/2, S are K/2 x N/2, the products Q are M/2 x N/2 (Appendix A holds for any conformal 2 x 2
 * blocking).  Extents that 2^levels does not divide are zero-padded into workspace copies or, with
 * sw_set_odd_mode(SW_ODD_PEEL), peeled (recursion on the previous multiples, up to three thin classical
 * products for the rest).  Otherwise as sw_gemm_ex; workspace_bytes >= sw_plan_memory_rect.
 * Errors as sw_gemm_ex; SW_EINVAL also when 2^levels exceeds the smallest extent or K == 0 with M, N > 0. */
int sw_gemm_rect(int64_t M, int64_t N, int64_t K, const double* A, int64_t lda, const double* B, int64_t ldb, double* C,
                 int64_t ldc, int levels, const char* schedule, void* workspace, int64_t workspace_bytes, void* hip_stream);
int64_t sw_plan_memory_rect(int64_t M, int64_t N, int64_t K, int levels, const char* schedule);

/* The product with diagonal scaling (Section 6.1): D1 C D3 = (D1 A D2)(D2^-1 B D3) with D1, D2, D3 diagonal
 * powers of two (scaling and unscaling are exact).  scaling: SW_SCALE_OUTSIDE (D1, D3: every row of A and
 * column of B gets a largest entry in [1, 2); the error of entry (i, j) then relates to ||A(i,:)|| ||B(:,j)||
 * instead of ||A|| ||B||), SW_SCALE_INSIDE (D2: column k of A and row k of B get largest entries of equal
 * size), or both (outside first); 0 = plain sw_gemm.  A and B stay untouched: scaled copies live in the
 * workspace, which must hold sw_plan_memory_scaled(n, levels, schedule) bytes.  Same state and rules as sw_gemm. */
#define SW_SCALE_OUTSIDE 1
#define SW_SCALE_INSIDE 2
int sw_gemm_scaled(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule,
                   int scaling);
int64_t sw_plan_memory_scaled(int64_t n, int levels, const char* schedule);

/* ---- other recursive algorithms on the same BFS/DFS machinery (Section 6.6) ------------------------------- */

/* C = A*B by a recursion built on another block scheme: a way to multiply n0 x n0 block matrices with q block
 * products (Section 6.6.2: exponent w0 = log_n0 q).  q combinations of the blocks of A and of B are multiplied
 * pairwise (recursively) and combined into the blocks of C.  A BFS step keeps T, S, Q of all q subproblems of
 * every parent (3q buffers of 1/n0 the size), a DFS step solves them in sequence (3 buffers).
 * scheme: SW_SCHEME_WINOGRAD = sw_gemm itself; SW_SCHEME_STRASSEN = Strassen's original algorithm (2 x 2 blocks,
 * 7 products, 18 additions per step, the count behind the constants of Section 3.3.2); SW_SCHEME_CLASSICAL = the
 * classical algorithm written recursively on 2 x 2 blocks (8 products, 4 additions; Section 6.6.1), whose
 * rounding errors obey the classical component-wise bound; SW_SCHEME_LADERMAN = Laderman's algorithm on 3 x 3
 * blocks (23 products); SW_SCHEME_CLASSICAL3 = the classical algorithm on 3 x 3 blocks (27 products).  Every
 * combination is summed left to right over the blocks 11, 12, .. (over the products in their order), so all
 * step orders give the same bits.  Same arguments, state (workspace, stream) and errors as sw_gemm; n that the
 * levels' block counts do not divide is zero-padded to the next multiple of their product; the workspace must
 * hold sw_plan_memory_bilinear bytes; additionally SW_EINVAL for an unknown scheme, when the levels cut n into
 * more parts than it has rows, or when the leaf products of one launch (q per BFS step) do not fit one
 * launch.  Runs on one stream. */
#define SW_SCHEME_WINOGRAD 0
#define SW_SCHEME_STRASSEN 1
#define SW_SCHEME_CLASSICAL 2
#define SW_SCHEME_LADERMAN 3
#define SW_SCHEME_CLASSICAL3 4
int sw_gemm_bilinear(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule,
                     int scheme);
/* The same with one scheme per level: schemes is a HOST array of `levels` scheme numbers, top level first (any but
 * SW_SCHEME_WINOGRAD), so steps on 2 x 2 and on 3 x 3 blocks mix: n = 94080 = 2^7 * 3 * 5 * 7^2 takes four Strassen
 * steps and one Laderman step without padding. */
int sw_gemm_bilinear_levels(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule,
                            const int* schemes);
/* Workspace bytes of sw_gemm_bilinear / sw_gemm_bilinear_levels (schedule NULL or "": all-DFS, the minimum).
 * Host arithmetic only. */
int64_t sw_plan_memory_bilinear(int64_t n, int levels, const char* schedule, int scheme);
int64_t sw_plan_memory_bilinear_levels(int64_t n, int levels, const char* schedule, const int* schemes);
/* Floating-point operations of the scheme's recursion, n a multiple of n0^levels (classical leaves 2m^3 - m^2,
 * one operation per element and block addition); -1.0 for bad arguments.  Host arithmetic only. */
double sw_flop_count_bilinear(int64_t n, int levels, int scheme);

/* ---- the product as a general matrix multiply ------------------------------------------------------------- */

/* C <- alpha * op(A) * op(B) + beta * C, the operation the fast algorithm replaces (Section 1), on row-major
 * rectangular operands: op(A) is M x K, op(B) is K x N, C is M x N; transa / transb != 0 take the transpose,
 * the stored matrix then being K x M (lda >= M) or N x K (ldb >= K).  The product is cut into blocks of
 * s_m x s_n x s_k: M, N and K each into 1 .. 4 equal parts, rounded down to a multiple of 2^levels.  Every
 * block product runs through the Strassen-Winograd recursion on rectangular operands (sw_gemm_rect: `levels`
 * steps, `schedule` as for that call) into a temporary and is folded into C in one pass (or is written
 * straight into C when alpha = 1, beta = 0 and K is one part); a transposed operand is transposed block by
 * block into a temporary; the rows, columns and inner indices left over (fewer than 4 * 2^levels each) go
 * through the classical MFMA product.  Among the block shapes whose need the workspace holds, the one with
 * the least modelled time is taken.  levels < 0: the depth is chosen with the block shape by the same model
 * (schedule is then ignored).  beta == 0: C is not read; alpha == 0 or K == 0: A and B are not read.  alpha,
 * beta are passed by value.  Uses the workspace and stream of sw_set_workspace / sw_set_stream; a workspace
 * of sw_plan_memory_dgemm bytes (the whole product as one block: a temporary for C, one more per transposed
 * operand, and the recursion's own) always suffices, smaller ones work with smaller blocks.  C must not
 * overlap A or B.
 * Errors: SW_EINVAL (negative or > 200000 dimension, 2^levels > min(M, N, K), short leading dimension, NULL
 * pointer, overlap, bad schedule), SW_ENOMEM, SW_EHIP. */
int sw_dgemm(int transa, int transb, int64_t M, int64_t N, int64_t K, double alpha, const double* A, int64_t lda,
             const double* B, int64_t ldb, double beta, double* C, int64_t ldc, int levels, const char* schedule);
/* Workspace bytes that suffice for sw_dgemm at an explicit depth (schedule NULL or "": all-DFS): the need of
 * the largest block size it considers.  Host arithmetic only. */
int64_t sw_plan_memory_dgemm(int transa, int transb, int64_t M, int64_t N, int64_t K, int levels,
                             const char* schedule);
/* The recursion depth for an n x n product with `budget_bytes` of workspace (the cutoff question of Section
 * 5.4.1, where five or six steps were best): the depth whose modelled time is least among those some step
 * order fits -- leaf products at the measured rate of the MFMA kernel for the leaf size (tile fill
 * included), additions at the measured HBM rate of the fused kernels.  0 = the classical product.  Host
 * arithmetic only; negative = error code. */
int sw_plan_levels(int64_t n, int64_t budget_bytes);
/* The modelled time in seconds behind sw_plan_levels for one depth (step order: the planner's for the
 * budget); -1.0 for bad arguments or when no step order of that depth fits.  Host arithmetic only. */
double sw_model_seconds(int64_t n, int levels, int64_t budget_bytes);
/* The same model for one explicit step order, with what the executor makes of `budget_bytes` of workspace (rich
 * DFS steps; with overlap != 0 the second set of leaf-side buffers, whose additions then run beside the leaf
 * products: a launch costs the longer of the two, the products stretched by 7 %).  -1.0 for bad arguments or
 * when the order does not fit.  Host arithmetic only. */
double sw_model_seconds_order(int64_t n, int levels, const char* schedule, int64_t budget_bytes, int overlap);

/* ---- the planner (Section 3.1: pick the step order that uses the memory there is; Sections 3.3.1, 3.4.1) - */

/* Bytes of workspace sw_gemm needs beyond A, B, C for this n, depth and step order (what THIS library
 * allocates from the workspace: 21 half-size buffers per parent at a BFS step -- or 147 quarter-size ones for
 * two fused BFS steps --, 2 at a DFS step, padded leading dimensions, plus padded copies of A, B, C when
 * 2^levels does not divide n).  schedule NULL or "":
 * the all-DFS order (the minimum).  Pure host arithmetic; needs no GPU.  Negative = error code. */
int64_t sw_plan_memory(int64_t n, int levels, const char* schedule);

/* Bytes of workspace (>= sw_plan_memory, <= budget_bytes) that sw_gemm can make use of for this step order:
 * with more than the minimum, first the buffers next to the leaves exist twice (consecutive leaf launches
 * alternate, so additions overlap products; only with sw_set_overlap on and a DFS step above), then DFS steps
 * -- deepest first -- keep their four non-trivial T, four S and seven Q
 * (the storage of a BFS step, Section 3.3.1, without the plain copies) while still solving the seven
 * subproblems in sequence (Section 3.4), so their additions become the one-pass kernels.  sw_gemm decides the
 * same way from the size of the workspace it is given.  SW_ENOMEM if the minimum exceeds the budget. */
int64_t sw_plan_workspace(int64_t n, int levels, const char* schedule, int64_t budget_bytes);

/* Choose the step order for n and levels under a workspace budget.  The candidates are the Limited-Memory
 * shapes of Section 3.4 -- l DFS steps followed by levels - l BFS steps -- that fit the budget; each is scored
 * with the cost model of sw_model_seconds_order; among the candidates within the model's error (6 %) of the best
 * score, one whose BFS steps come in fused pairs below a DFS step (so that their additions run beside the leaf
 * products; only with sw_set_overlap on) is preferred, then the lower score; an order whose leaf launches would
 * not fill the machine's workgroup slots three times is left out while another remains.  On sweeps of all step
 * orders at n = 4096 .. 47040 the choice is within 0.3 % of the fastest order.  out: HOST buffer of levels + 1
 * chars.  SW_ENOMEM if not even the all-DFS order fits. */
int sw_plan_schedule(int64_t n, int levels, int64_t budget_bytes, char* out);

/* The paper's memory model for a step order, in words: sum over levels i = 0..levels of 3 * live_i * n_i^2
 * (i = 0 is A, B, C; live multiplies by 7 at a BFS step).  Equals P * Mem_UM (Section 3.3.1) for all-BFS
 * and P * Mem_LM (Section 3.4.1) for DFS-then-BFS.  n must be a multiple of 2^levels. */
int64_t sw_model_words(int64_t n, int levels, const char* schedule);

/* Number of DFS steps of the Limited-Memory scheme, l = max(0, ceil(log2(4 n / (P^(1/w0) sqrt(M))))),
 * w0 = log2 7 (Section 3.4, the equation that sets l; valid when 3 n^2 / P <= M / 3).  M in words. */
int sw_lm_dfs_steps(double n, double P, double M_words);

/* Actual arithmetic of one product: 7^levels * (2 m^3 - m^2) + 15 * sum_i 7^i (n_i / 2)^2 with
 * m = n / 2^levels, i.e. F(n) = c_s n^w0 - 5 n^2 of Appendix A.  n must be a multiple of 2^levels. */
double sw_flop_count(int64_t n, int levels);

/* ---- library state -------------------------------------------------------------------------------------- */

int sw_set_workspace(void* dev_ptr, int64_t bytes); /* caller-owned; NULL/0 clears it                    */
int sw_set_stream(void* hip_stream);                /* hipStream_t; NULL = the null stream               */

/* on != 0 (default): inside one product the kernels that form operands, the leaf products and the kernels
 * that fold products into C run on three streams (the caller's and two of the library's), ordered by events
 * from the address ranges each kernel reads and writes, so HBM-bound additions overlap MFMA-bound products;
 * towards the caller the call still behaves as if everything ran on the caller's stream.  on == 0: one
 * stream.  The results are the same bits either way.  Step orders without a DFS step form one chain of
 * kernels and always run on one stream.  While overlapping, the addition kernels next to the leaves (those
 * that run beside the leaf products when the leaf-side buffers exist twice) are launched as persistent
 * streaming kernels with a limited number of workgroups, so that they take little of the machine away from
 * the products: on == 1 (default) sizes that number to the work (enough to move their bytes in two thirds of
 * the time of the leaf launch beside them, at least 32; uncapped when more than 256 would be needed),
 * on > 1 fixes it to `on`.  All other addition kernels lie on the critical path and get the whole machine. */
int sw_set_overlap(int on);

/* What sw_gemm, sw_plan_memory and sw_plan_schedule do when 2^levels does not divide n (Section 3.1:
 * "padding or dynamic peeling").  SW_ODD_PAD (default): zero-padded workspace copies of A, B, C of the next
 * multiple.  SW_ODD_PEEL: the recursion runs in place on the leading blocks of the previous multiple n0 and
 * the n - n0 < 2^levels peeled rows and columns are finished by thin classical products (C11 += A12*B21,
 * C12 = [A11 A12]*[B12;B22], [C21 C22] = [A21 A22]*B); no copies, so it also works when three more matrices
 * do not fit. */
#define SW_ODD_PAD 0
#define SW_ODD_PEEL 1
/* SW_ODD_PEEL_LEVELS ("dynamic" peeling): no copies and no rounding of n either; whenever the size at some level of
 * the recursion is odd, the last row, column and inner index are peeled off there, the step runs on the even
 * part and the peeled parts are finished by thin classical products (C11 += a12*b21, c12 = [A11 a12]*[b12;b22],
 * [c21 c22] = [a21 a22]*B) for all problems of that level at once; the children may be odd again.  Needs only
 * 2^levels <= n.  Two BFS steps are fused only where the level between them is even.  Workspace: what the halved
 * (rounded-down) extents need, plus a copy of the peeled column of A and row of B per problem of a level whose
 * inner extent is odd (sw_plan_memory counts it). */
#define SW_ODD_PEEL_LEVELS 2
int sw_set_odd_mode(int mode);
const char* sw_last_error(void);                    /* HOST string, valid until the thread's next call  */

/* ---- the steps of the path, one call each (used by sw_gemm; exported so each can be tested and timed) ---- */

/* Pre-additions of one BFS step (Appendix A, first and second column).  side 0: from each of `live` parents
 * P (n x n, h = n/2) write T0..T6 = A11, A12, A21+A22, T2-A11, A11-A21, A12-T3, A22.  side 1: S0..S6 = B11,
 * B21, B12-B11, B22-S2, B22-B12, B22, S3-B21.  Parent p starts at parent + p*parent_stride; child j of
 * parent p starts at child + (7p + j)*child_stride and has leading dimension child_ld >= h.  Strides and
 * leading dimensions in elements.  One pass: each input element read once, each output written once. */
int sw_pre_add(int side, const double* parent, int64_t parent_ld, int64_t parent_stride, int64_t live,
               int64_t h, double* child, int64_t child_ld, int64_t child_stride, void* hip_stream);

/* Post-additions of one BFS step (Appendix A, fourth column): U1 = Q0+Q3, U2 = U1+Q4, U3 = U1+Q2,
 * C11 = Q0+Q1, C12 = U3+Q5, C21 = U2-Q6, C22 = U2+Q2, in this association, for `live` parents. */
int sw_post_add(const double* Q, int64_t q_ld, int64_t q_stride, int64_t live, int64_t h,
                double* parent, int64_t parent_ld, int64_t parent_stride, void* hip_stream);

/* Two consecutive BFS steps in one pass (what sw_gemm uses when the step order has "BB"): each parent
 * (4m x 4m) gives the operands of its 49 grandchildren (m x m), grandchild (j, i) = T_i of (T_j of the
 * parent), stored at child + (49 p + 7 j + i) * child_stride; the values are bit-identical to two sw_pre_add
 * calls, the 28 intermediate blocks never reach memory.  sw_post_add2 is the reverse for the products. */
int sw_pre_add2(int side, const double* parent, int64_t parent_ld, int64_t parent_stride, int64_t live,
                int64_t m, double* child, int64_t child_ld, int64_t child_stride, void* hip_stream);
int sw_post_add2(const double* Q, int64_t q_ld, int64_t q_stride, int64_t live, int64_t m,
                 double* parent, int64_t parent_ld, int64_t parent_stride, void* hip_stream);

/* Classical leaf products (Section 5.4.1): C_b = A_b * B_b for b < batch, each m x m, fp64 MFMA
 * (v_mfma_f64_16x16x4_f64), one launch for the whole batch.  Operand b starts at base + b*stride. */
int sw_leaf_gemm(int64_t m, int64_t batch, const double* A, int64_t lda, int64_t stride_a,
                 const double* B, int64_t ldb, int64_t stride_b, double* C, int64_t ldc, int64_t stride_c,
                 void* hip_stream);

/* The leaf kernel on general shapes: C (M x N) = A (M x K) * B (K x N), or C += A * B if accumulate != 0.
 * Used by peeling; any M, N, K >= 0 (K = 0 with accumulate == 0 zeroes C). */
int sw_gemm_classical(int64_t M, int64_t N, int64_t K, const double* A, int64_t lda, const double* B, int64_t ldb,
                      double* C, int64_t ldc, int accumulate, void* hip_stream);

/* Zero-padded copy (rows x cols of src into the top-left of a prows x pcols dst, rest zero) and its
 * inverse crop are the same call: the region copied is min(rows, prows) x min(cols, pcols). */
int sw_pad_copy(const double* src, int64_t src_ld, int64_t rows, int64_t cols,
                double* dst, int64_t dst_ld, int64_t prows, int64_t pcols, void* hip_stream);

/* ---- measurement ---------------------------------------------------------------------------------------- */

/* Kernel classes for sw_profile_read. */
#define SW_CLASS_PRE_ADD 0  /* BFS pre-additions                        */
#define SW_CLASS_POST_ADD 1 /* BFS post-additions                       */
#define SW_CLASS_LEAF 2     /* batched leaf GEMM                        */
#define SW_CLASS_DFS_ADD 3  /* element-wise kernels of DFS steps        */
#define SW_CLASS_PAD 4      /* pad / crop copies                        */
#define SW_CLASS_PEEL 5     /* classical products of peeling and of sw_dgemm's remainders (work = flops) */
#define SW_CLASS_SCALE 6    /* diagonal scaling: maxima, scaled copies, unscaling */
#define SW_CLASS_BLAS 7     /* sw_dgemm: block transposes and the alpha/beta folds into C */
#define SW_NUM_CLASSES 8

/* on != 0: bracket every kernel launch of sw_gemm with HIP events on the launch stream (no host sync).
 * sw_profile_read synchronises those events, adds up per class the elapsed milliseconds, the launches and
 * the algorithmic bytes (add kernels: distinct elements read + written, times 8) or flops (leaf: 2 m^3 per
 * product) into HOST arrays of SW_NUM_CLASSES entries, and clears the record. */
int sw_profile_enable(int on);
int sw_profile_read(double* ms, int64_t* launches, double* work);

/* ---- verification of the executor's ordering, on the host (no GPU needed) ---------------------------------- */

/* A record-only run of sw_gemm_rect: the executor walks the same recursion (Algorithm 2, procedures BFS and DFS)
 * for this shape, step order, workspace size and settings, but launches nothing and makes no HIP call.  It
 * writes down, in submission order, every kernel it would launch with the memory that kernel touches -- taken
 * from the launch arguments, not from what the executor declared to its dependency tracker --, every event it
 * would record, every stream wait it would issue and every buffer it takes from the workspace.  A checker can
 * rebuild happens-before from the record and look for conflicting accesses that no chain of waits orders.
 * Operands have synthetic addresses: A at 2^40, B at 2 * 2^40, C at 3 * 2^40, the workspace at 4 * 2^40.
 * overlap, odd_mode: as sw_set_overlap / sw_set_odd_mode would set them (the process-wide settings are not read).
 * withhold: -1, or the number (counted over the call, reads before writes) of ONE range that is kept from the
 * dependency tracker although its kernel still touches it: a planted mistake for testing the checker.
 * log: HOST buffer of log_words 64-bit words, may be NULL.  Returns the number of words of the whole record
 * (only the first log_words are written) or a negative error code.  Records:
 *   1, stream, kernel kind, nr, nw, then nr read and nw written footprints of 6 words each:
 *      address, rows, cols, leading dimension, count, stride (count matrices of rows x cols doubles, in elements)
 *   2, stream, slot                 an event is recorded on `stream` (slot -1: the entry event)
 *   3, stream, event stream, slot   `stream` waits for the event (event stream, slot) as last recorded
 *   4, offset, bytes                a buffer is taken from the workspace stack
 *   5, offset                       the stack is cut back to `offset`
 *   6, tracked                      the tracker held `tracked` unsettled accesses and fell back to ordering every
 *                                   stream after every other (the waits follow as records of kind 3)
 * Streams: 0 the caller's, 1 and 2 the library's.  Kernel kinds: 0 pre-addition, 1 post-addition, 2 and 3 the
 * fused two-step forms, 4 element-wise, 5 DFS post block, 6 pad copy, 7 product. */
int64_t sw_trace_gemm(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int levels, const char* schedule,
                      int64_t workspace_bytes, int overlap, int odd_mode, int64_t withhold, int64_t* log, int64_t log_words);

#ifdef __cplusplus
}
#endif
#endif /* SW_GEMM_H */
