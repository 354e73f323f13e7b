/*
 * ecgemm: error-corrected single-precision GEMM for AMD MI355X (gfx950).
 *
 * C-ABI of the split-and-correct SGEMM of Ootomo & Yokota, "Recovering single precision
 * accuracy from Tensor Cores while surpassing the FP32 theoretical peak performance".
 * Every FP32 input is split into low-precision parts, the product is formed from the
 * leading product plus the first-order correction products on the matrix units, the
 * corrections are summed in an accumulator of their own and merged once at the end.
 *
 * All matrix pointers are DEVICE pointers owned by the caller.  The library only reads A
 * and B, writes C, keeps no pointer after a call returns, and never frees caller memory.
 * All work is enqueued on the handle's stream and the calls return without waiting for it, with the
 * exceptions stated at the functions concerned: a handle-owned workspace that has to grow (below),
 * ecgemm_exponent_range, ecgemm_choose_mode, ecgemm_auto_choice and ecgemm_get_timing.
 * Every function returns an ecgemm_status_t and never throws or aborts.  Enumeration arguments are read as plain
 * integers: a value that is not one of the enumerators is refused like any other bad argument.  Arguments and sizes are checked before
 * anything is enqueued: ECGEMM_ERR_INVALID_ARG, ECGEMM_ERR_UNSUPPORTED and ECGEMM_ERR_ALLOC mean that the call has
 * enqueued nothing and left C untouched.  ECGEMM_ERR_HIP means that the HIP runtime refused a launch or an event in
 * the middle of the call: kernels enqueued before that point still run, and the contents of C and of the workspace
 * are then unspecified.  A handle may be used by one host thread at a time.
 *
 * Workspace.  A product needs device memory for the split operands (ecgemm_workspace_size; a small product, which
 * runs as a single kernel that reads A and B itself, needs none in the modes of the method).  Either the caller
 * provides it (ecgemm_set_workspace), or the handle allocates it on first need and keeps it; whenever a call needs
 * more than the handle holds, that call waits for the handle's stream, frees the old buffer and allocates a larger
 * one (hipStreamSynchronize, hipFree, hipMalloc) before it enqueues anything.  With a caller-provided workspace and
 * timing off, ecgemm_sgemm and ecgemm_product only launch kernels (no allocation, no memset, no wait), so they can be
 * recorded into a HIP graph; ecgemm_sgemm_noalloc does the same on a workspace built into the library.
 * All calls on a handle share its workspace and nothing orders them but the stream: after ecgemm_set_stream has
 * changed the stream, the caller makes the new stream wait for the work enqueued on the old one before the next
 * product (or uses one handle per stream).
 *
 * Results are bitwise reproducible for equal inputs and equal settings
 * (no floating-point atomics; the sums of tiles cut along K are added in a fixed order).
 *
 * This header is the production surface.  The knobs and diagnostics that only tests, tuning sweeps and the
 * accuracy experiments use (forcing a kernel shape, the paper's comparison methods, bare matrix instructions) are
 * declared in ecgemm_debug.h.
 */
#ifndef ECGEMM_H
#define ECGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ecgemm_context *ecgemm_handle_t;

typedef enum { ECGEMM_OP_N = 0, ECGEMM_OP_T = 1 } ecgemm_op_t;

typedef enum {
    /* "halfhalf" (Eqs. corr-1-1024 .. corr-4-1024 and corr-5-1024-reduce): v ~ v16 + dv16 * 2^-11 with
     * two FP16 parts, three matrix-unit products.  FP32 accuracy for inputs of magnitude 2^-14 .. 2^16;
     * precision tapers below and nothing is left under 2^-35 (section "Effect of the exponent range"). */
    ECGEMM_MODE_FP16_SPLIT = 0,
    /* Full FP32 exponent range.  The paper uses TF32 pairs (section "Reducing the underflow ...", tf32tf32);
     * gfx950 has no TF32 matrix instruction, so each value is split exactly into three BF16 terms and the
     * six products of relative size >= 2^-16 are kept (same argument as section "Removing negligible
     * error correction"). */
    ECGEMM_MODE_BF16_FULL = 1,
    /* 2 .. 9: the methods the paper compares against, run through the same kernels so that its error curves can be
     * redrawn on this hardware.  Not meant for production use; each is described in ecgemm_debug.h (they are
     * enumerators here because a C enumeration cannot be extended from a second header). */
    ECGEMM_MODE_FP16_MARKIDIS = 2,
    ECGEMM_MODE_FP16_UNSCALED = 3,
    ECGEMM_MODE_FP16_PLAIN = 4,
    ECGEMM_MODE_BF16_PLAIN = 5,
    ECGEMM_MODE_FP16_OUTSIDE_ACC = 6,
    ECGEMM_MODE_FP32_MFMA = 7,
    ECGEMM_MODE_FP16_OUTSIDE_ACC_4 = 8,
    ECGEMM_MODE_FP16_OUTSIDE_ACC_16 = 9,
    /* ecgemm_sgemm, ecgemm_sgemm_noalloc and ecgemm_workspace_size only: ECGEMM_MODE_FP16_SPLIT if the FP16 pair
     * represents both operands well enough, as they are or after scaling their rows and columns by powers of two, else
     * ECGEMM_MODE_BF16_FULL, decided on the GPU during the split pass (see "Automatic mode" below).  The trade the paper leaves to the user (section "Effect of the exponent range of input
     * matrices": halfhalf is faster, tf32tf32 covers the range) made from the data. */
    ECGEMM_MODE_AUTO = 10
} ecgemm_mode_t;

typedef enum {
    ECGEMM_OK = 0,
    ECGEMM_ERR_INVALID_ARG = 1, /* bad enum, negative size, leading dimension too small, null pointer */
    ECGEMM_ERR_ALLOC = 2,       /* device workspace could not be allocated, or the caller's is too small */
    ECGEMM_ERR_HIP = 3,         /* a HIP runtime call failed; see ecgemm_last_error_string */
    ECGEMM_ERR_UNSUPPORTED = 4  /* device is not gfx950, or the forced kernel shape does not exist for the mode */
} ecgemm_status_t;

/* Creates a handle bound to the current HIP device.  Allocates no device memory.  The device must
 * be a gfx950; otherwise ECGEMM_ERR_UNSUPPORTED.  `handle` is a host pointer. */
ecgemm_status_t ecgemm_create(ecgemm_handle_t *handle);

/* Frees the handle and the workspace it allocated itself (never a caller-provided one).  Work already
 * enqueued must have finished: the caller synchronises the stream first. */
ecgemm_status_t ecgemm_destroy(ecgemm_handle_t handle);

/* Stream (a hipStream_t passed as void*) on which every later call enqueues its kernels.
 * Default: the null stream. */
ecgemm_status_t ecgemm_set_stream(ecgemm_handle_t handle, void *hip_stream);

/* Bytes of device workspace ecgemm_sgemm needs for this problem: the split operands in matrix-unit fragment order,
 * zero-padded to whole tiles, plus at most 128 MiB of partial sums for output tiles that are cut into slices along K.
 * (Small products run as one launch that needs no packed operands, and partial sums only where deep products of few
 * tiles are cut into slices along K; the size returned for them is the larger of that and what ecgemm_product needs.)
 * The plan behind it is made for the 256 compute units of the MI355X, so the size depends on the problem, the mode and
 * the kernel shape only; `handle` supplies the shape forced with ecgemm_set_shape (ecgemm_debug.h) and may be NULL
 * (automatic choice).  transA and transB are checked and otherwise do not matter: the split pass absorbs the
 * transposes, so all four combinations need the same workspace.  `bytes` is a host pointer. */
ecgemm_status_t ecgemm_workspace_size(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                                      int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode, size_t *bytes);

/* How ecgemm_sgemm would run this problem (host logic only; no GPU work, `handle` as in ecgemm_workspace_size):
 * the kernel shape, the output tiles, how many of them are one work item over the whole depth and how many are cut
 * into how many slices along K, whether the product kernel is launched as a persistent grid, in which order the tiles
 * go to the XCDs, its grid size on a 256-CU device, and the workspace bytes.  `info` is a host pointer. */
typedef struct {
    int shape;          /* kernel shape used: 1 = block tile 256 x 128, 2 = 128 x 128 two per compute unit, 3 and 4 = one
                           launch that splits for itself, block tile 64 x 64 and 32 x 32 (the ecgemm_shape_t values of
                           ecgemm_debug.h; never 0 = automatic) */
    int tile_m, tile_n; /* block tile */
    int tiles_m, tiles_n;
    int whole_tiles;    /* tiles that are one work item */
    int sliced_tiles;   /* tiles cut into `slices` work items each; their sums are added by a second kernel */
    int slices;         /* 1 if sliced_tiles == 0 */
    int persistent;     /* 1: one workgroup per CU walks through several work items */
    int group_m;        /* tile rows per group of the order in which tiles are handed out (groups are walked along N) */
    int column_bands;   /* n: the tile order takes the grid in n bands of columns one after the other; each XCD takes a
                           contiguous run of the order, so the 8 XCDs lie (8 / n) x n over the tile grid */
    int64_t grid;       /* workgroups of the product (or fused) kernel */
    size_t workspace_bytes;
    double estimated_us; /* the cost estimate by which this plan was preferred to the others (product and reduce kernels,
                            microseconds on a power-limited MI355X; for the one-launch shapes, the whole call) */
} ecgemm_plan_info_t;
ecgemm_status_t ecgemm_plan_info(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode,
                                 ecgemm_plan_info_t *info);

/* Hands the library a caller-owned device buffer (256-byte aligned) to use as workspace from now on;
 * (NULL, 0) returns to the handle-owned workspace, which is allocated on first need and only ever
 * grows (the call that makes it grow waits for the stream and allocates, see the top of this file).  With a caller
 * buffer the library never allocates: a too small one makes ecgemm_sgemm return ECGEMM_ERR_ALLOC.  The workspace must
 * not overlap A, B or C, and stays the caller's: ecgemm_destroy does not free it. */
ecgemm_status_t ecgemm_set_workspace(ecgemm_handle_t handle, void *device_buffer, size_t bytes);

/*
 * C <- alpha * op(A) * op(B) + beta * C        (BLAS sgemm semantics, column-major)
 *
 *   op(A) is M x K, op(B) is K x N, C is M x N; op(X) = X or X^T per transA / transB.
 *   A: device, FP32, column-major, leading dimension lda >= (transA == N ? M : K)
 *   B: device, FP32, column-major, leading dimension ldb >= (transB == N ? K : N)
 *   C: device, FP32, column-major, ldc >= M; read only when beta != 0 (so NaN/Inf already in C do
 *      not propagate when beta == 0), written for all M x N elements.  C must not overlap A or B.
 *   alpha, beta: host scalars.
 *
 * Steps (each a kernel on the handle's stream; for a small product, up to about 1024^3, one kernel does all three:
 * it reads A and B itself and forms the parts in registers, as the paper's own kernel does, with the same result):
 *   1. split: A and B are read once and written to the workspace as FP16 (v16, dv16 = (v - v16) * 2^11;
 *      Eqs. corr-1-1024 .. corr-4-1024) or as three BF16 terms, round to nearest even, K-contiguous,
 *      in the lane order the matrix instruction wants, zero-padded to tile multiples.  A finite input
 *      never produces an infinite part: conversions saturate at the largest finite FP16 / BF16 value.
 *   2. product: A16 B16 goes to one FP32 accumulator; the correction products (dA16 B16 + A16 dB16, or
 *      the five lower BF16 products) go to a second FP32 accumulator that is never mixed with the first
 *      inside the loop; dA16 dB16 and the BF16 products below 2^-16 are left out (Eq. corr-5-1024-reduce).
 *   3. epilogue: c = main + correction * 2^-11 (FP16 mode) or main + correction (BF16 mode), then
 *      C <- alpha * c + beta * C in FP32.
 *
 * Sizes: a packed row block (K / 16 * parts KiB) must stay below 4 GiB, i.e. K < 2^25 for two parts, 2^24.4 for three.
 * M == 0 or N == 0: nothing is done.  K == 0 or alpha == 0: C <- beta * C (C <- 0 when beta == 0).
 * Inf / NaN inputs give Inf / NaN outputs but not necessarily in IEEE-exact positions.
 */
ecgemm_status_t ecgemm_sgemm(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                             int64_t M, int64_t N, int64_t K, float alpha,
                             const float *A, int64_t lda, const float *B, int64_t ldb,
                             float beta, float *C, int64_t ldc, ecgemm_mode_t mode);

/*
 * ecgemm_sgemm for callers that cannot allocate device memory and have no workspace to hand over: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bitwise the same result as ecgemm_sgemm, but the workspace is a fixed array of ECGEMM_NOALLOC_WORKSPACE_BYTES that
 * is part of the library's device code (each GPU the library runs on holds its copy until the process ends; its
 * address on the handle's device is looked up once, in ecgemm_create).  The call only launches kernels: no hipMalloc,
 * no hipFree, no memset, no event, no wait; the handle's workspace setting and its timing switch are ignored.
 * A problem whose workspace (ecgemm_workspace_size) exceeds the array returns ECGEMM_ERR_ALLOC and enqueues nothing;
 * 64 MiB hold, for example, 2048^3 in either mode or 1024 x 1024 x 8192 in FP16 mode.
 * Every call on a GPU, from any handle, uses that GPU's one array, which keeps the previous call's contents (nothing
 * in it needs clearing: every byte a product reads has been written by the same call's split pass or slices before).
 * Calls that overlap in time on one GPU - two streams, two handles, two host threads - therefore race; calls on one
 * stream are ordered by it.
 */
#define ECGEMM_NOALLOC_WORKSPACE_BYTES ((size_t)64 << 20)
ecgemm_status_t ecgemm_sgemm_noalloc(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                                     int64_t M, int64_t N, int64_t K, float alpha,
                                     const float *A, int64_t lda, const float *B, int64_t ldb,
                                     float beta, float *C, int64_t ldc, ecgemm_mode_t mode);

/*
 * Automatic mode (mode == ECGEMM_MODE_AUTO).  The call enqueues, without ever waiting for the GPU:
 *   1. the FP16 pair split of A and B (after the handle's pre-scaling, if any), whose kernels also sum, in FP64 and in
 *      a fixed order, |x|^2 and |x - (v16 + dv16 * 2^-11)|^2 over each operand;
 *   2. a one-workgroup kernel that chooses the FP16 mode if for both operands the second sum is at most 2^-48 times the
 *      first, that is, if the pair represents each operand to a relative error of 2^-24 (the unit roundoff of FP32) in
 *      the Frobenius norm, and if at least one operand spreads the weight of a row over 16 elements or more, measured by
 *      (sum |x|)^2 / (rows * sum x^2) (the kernels sum |x| as well): the pair holds 22.75 of FP32's 24 bits, which
 *      matches an FP32 product only where that product's own summation error outweighs the missing bit, not for dot
 *      products carried by a handful of terms (very short K, or exponents spread so widely that a few elements dominate
 *      each row);
 *   3. otherwise: the scaling exponents of ecgemm_row_scales for the rows of op(A) and the columns of op(B) (largest
 *      binade of each to 2^14), the FP16 pair split of the operands scaled by them with the same sums, and a second
 *      choice by the same rule: the FP16 mode on the scaled operands, with the factors divided out element by element
 *      as in ecgemm_sgemm_scaled (a row-wise and column-wise guarantee: the error of element (m, n) is then bounded
 *      relative to |row m of op(A)| |column n of op(B)|), or else the BF16 mode (an operand holds a NaN or an infinity, or
 *      the rows are too short in the sense of step 2);
 *   4. the three-term BF16 split and the three products, each of which reads the choice from device memory when it
 *      starts and returns at once if it is not the one chosen.
 * The result is bitwise that of ecgemm_sgemm in FP16 mode, of ecgemm_row_scales (target 14) + ecgemm_sgemm_scaled in
 * FP16 mode, or of ecgemm_sgemm in BF16 mode.  The criterion is about the inputs, so it holds for any product of them:
 * with Delta A, Delta B the parts the pair loses, |Delta A B + A Delta B| is bounded by
 * (|Delta A| / |A| + |Delta B| / |B|) |A| |B| in the Frobenius norm.  Uniform(-1, 1) and the paper's Type 1 inputs
 * choose the plain FP16 mode; Types 2 to 4 and inputs spread over the whole FP32 exponent range choose the scaled one
 * and run at the FP16 mode's speed.  What the scaled FP16 mode does not give is element-wise accuracy for elements far
 * below their row's or column's largest: a caller who needs every element of A and B honoured to 24 bits whatever its
 * size asks for ECGEMM_MODE_BF16_FULL.  Cost over calling the chosen arrangement directly: the statistics in the split
 * (it stays bound by memory traffic), seven to a dozen kernel launches, most of which do nothing, and for the later candidates the
 * splits that are thrown away.  Workspace: that of the BF16 mode plus 24 bytes per 64 x 32 block of each operand, 4 (M + N)
 * bytes and 256 (ecgemm_workspace_size with ECGEMM_MODE_AUTO).  Not available with caller-given scaling vectors,
 * ecgemm_split / ecgemm_product, ecgemm_plan_info or a forced one-launch kernel shape (ECGEMM_ERR_UNSUPPORTED or
 * ECGEMM_ERR_INVALID_ARG for the mode).
 *
 * ecgemm_auto_choice reports what the handle's last ecgemm_sgemm / ecgemm_sgemm_noalloc call chose: the mode, and
 * whether it ran on row / column scaled operands (1) or not (0).  It waits for the handle's stream (the only part of
 * the automatic mode that does), so it is for tests and logs, not for inner loops.  ECGEMM_ERR_INVALID_ARG
 * (argument 1) if that call was not in automatic mode, did nothing (M, N or K zero, alpha zero), or the workspace has
 * been replaced since.  `mode` and `scaling_vectors` are host pointers.
 */
ecgemm_status_t ecgemm_auto_choice(ecgemm_handle_t handle, ecgemm_mode_t *mode, int *scaling_vectors);

/*
 * Power-of-two pre-scaling: the remedy the paper names, at the end of section "Effect of the exponent range of input
 * matrices", for inputs whose elements are all too small for the FP16 pair.  From now on
 * ecgemm_sgemm on this handle splits op(A) * 2^log2_scale_a and op(B) * 2^log2_scale_b and multiplies the product by
 * 2^-(log2_scale_a + log2_scale_b) before alpha / beta.  Multiplying by a power of two is exact, so this only moves
 * the inputs inside the exponent window of the FP16 pair (2^-14 .. 2^16); the caller must pick exponents that neither
 * overflow nor underflow FP32.  Each exponent and their sum must lie in [-126, 126].  (0, 0) switches it off.
 * ecgemm_split and ecgemm_product are not affected.
 */
ecgemm_status_t ecgemm_set_scaling(ecgemm_handle_t handle, int log2_scale_a, int log2_scale_b);

/*
 * Per-row / per-column power-of-two pre-scaling, for matrices whose rows (of op(A)) or columns (of op(B)) differ in
 * magnitude by more than the exponent window of the FP16 pair lets one global factor absorb: the same remedy as
 * ecgemm_set_scaling (end of section "Effect of the exponent range of input matrices"), applied vector-wise.
 *
 * ecgemm_sgemm_scaled is ecgemm_sgemm with row m of op(A) multiplied by 2^row_log2_scale_a[m] and column n of op(B) by
 * 2^col_log2_scale_b[n] before the split (exact), and element (m, n) of the product multiplied by
 * 2^-(row_log2_scale_a[m] + col_log2_scale_b[n]) (exact unless the result leaves the normal FP32 range; the two
 * exponents are added first, so one of them alone may be far outside what the product could bear) before alpha / beta.  The vectors
 * are device arrays of M and N 32-bit integers in [-126, 126], read during the call and not kept; both NULL gives
 * ecgemm_sgemm.  The handle's global scaling, if any, is applied as well.
 *
 * ecgemm_row_scales writes such a vector: for each row r of X = op(src) (rows x depth; op and ld as in ecgemm_split)
 * the exponent that moves the row's largest non-zero finite element into the binade 2^target_exponent, 0 for a row
 * without one.  For the columns of op(B) pass B the way ecgemm_split takes it: op = T if B is stored K x N
 * (transB == N), op = N if stored N x K, rows = N, depth = K.  Runs on the handle's stream without waiting for it.
 * A target of 14 puts every row's largest binade at the top of the window in which the FP16 pair is fully precise.
 */
ecgemm_status_t ecgemm_row_scales(ecgemm_handle_t handle, ecgemm_op_t op, int64_t rows, int64_t depth, const float *src,
                                  int64_t ld, int target_exponent, int32_t *log2_scale);
ecgemm_status_t ecgemm_sgemm_scaled(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                                    int64_t M, int64_t N, int64_t K, float alpha,
                                    const float *A, int64_t lda, const float *B, int64_t ldb,
                                    float beta, float *C, int64_t ldc, ecgemm_mode_t mode,
                                    const int32_t *row_log2_scale_a, const int32_t *col_log2_scale_b);

/*
 * Helper for choosing a mode or a pre-scaling: binary exponents (floor(log2 |x|)) of the smallest and the largest
 * non-zero finite element of a column-major rows x cols FP32 matrix (src: device, ld >= rows).  Subnormals count as
 * -127; a matrix without such elements gives (INT_MAX, INT_MIN).  Unlike the other calls this one waits for the
 * stream: the two results are host integers.
 */
ecgemm_status_t ecgemm_exponent_range(ecgemm_handle_t handle, int64_t rows, int64_t cols, const float *src, int64_t ld,
                                      int *min_exponent, int *max_exponent);

/*
 * Picks settings for a product from the data (synchronous, reads A and B once): if the non-zero elements of each operand
 * span at most 29 binades, ECGEMM_MODE_FP16_SPLIT with the pre-scaling exponents that put each operand's largest binade
 * at 2^14 (every element then sits in the window where the FP16 pair is fully precise, the paper's Type 1 situation);
 * otherwise ECGEMM_MODE_BF16_FULL with no scaling (Types 2 to 4).  The caller passes the
 * exponents to ecgemm_set_scaling and the mode to ecgemm_sgemm.  Conservative: inputs with a few tiny elements (such
 * as uniform(-1, 1) draws) also do well in FP16 mode, because the residual of Eq. eval-matmul is dominated by the
 * large ones.  A, B, lda, ldb, transA, transB, M, N, K as in ecgemm_sgemm; mode and the two exponents are host pointers.
 */
ecgemm_status_t ecgemm_choose_mode(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N,
                                   int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                                   ecgemm_mode_t *mode, int *log2_scale_a, int *log2_scale_b);

/*
 * Step 1 alone (Eqs. corr-1-1024 .. corr-4-1024 / the BF16 three-term split), for inspection and tests.
 * Splits the `rows` x `depth` matrix X = op(src) into `packed`, a device buffer of
 * ecgemm_split_size(rows, depth, mode) bytes, laid out as
 *     packed[row_block][k_step][part][lane][8]   (16-bit elements)
 * with row_block = r / 32, k_step = k / 16, lane = ((k % 16) / 8) * 32 + r % 32, element k % 8;
 * part 0 is the high part; there are 2 parts in the FP16 pair modes, 3 in ECGEMM_MODE_BF16_FULL, 1 in the plain
 * modes.  Rows are padded to a multiple of 256 and depth to a multiple of 32, with zeros.  src: device, FP32,
 * column-major with leading dimension ld; op == N means X(r, k) = src[r + k * ld] (ld >= rows), op == T means
 * X(r, k) = src[k + r * ld] (ld >= depth).
 */
ecgemm_status_t ecgemm_split(ecgemm_handle_t handle, ecgemm_op_t op, int64_t rows, int64_t depth,
                             const float *src, int64_t ld, ecgemm_mode_t mode, void *packed);

/*
 * Steps 2 and 3 alone (Eq. corr-5-1024-reduce and the merge at the end of the paper's listing), for callers that keep
 * an operand split across many products:  C <- alpha * op(A) op(B) + beta * C  with op(A) (M x K) and op(B)^T (N x K)
 * given as the outputs of ecgemm_split(handle, ..., rows = M or N, depth = K, ..., mode, packed) for the SAME mode.
 * For op(B) that means: ecgemm_split(op = T if B is stored K x N (transB == N), op = N if stored N x K).  packedA,
 * packedB: device, read only.  C, ldc, alpha, beta as in ecgemm_sgemm.  Uses the workspace only for the partial sums
 * of tiles sliced along K.  The result is bitwise what ecgemm_sgemm returns for the same operands and kernel shape
 * (with the automatic shape, ecgemm_sgemm may run a small product as one launch, which slices along K differently
 * from this function or not at all: then the two agree to FP32 rounding).
 */
ecgemm_status_t ecgemm_product(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, float alpha,
                               const void *packedA, const void *packedB, float beta, float *C, int64_t ldc,
                               ecgemm_mode_t mode);

/* Bytes ecgemm_split writes for a rows x depth operand.  `bytes` is a host pointer. */
ecgemm_status_t ecgemm_split_size(int64_t rows, int64_t depth, ecgemm_mode_t mode, size_t *bytes);

/* When enabled, every ecgemm_sgemm brackets its split kernels and its product kernel with HIP events on
 * the handle's stream so that their device durations can be read back; off by default. */
ecgemm_status_t ecgemm_set_timing(ecgemm_handle_t handle, int enabled);

/* Synchronises with the events of the calls made since timing was enabled (or since the last call of
 * this function) and returns the number of ecgemm_sgemm calls seen and the summed device milliseconds
 * of their split kernels and of their product kernel.  All three outputs are host pointers. */
ecgemm_status_t ecgemm_get_timing(ecgemm_handle_t handle, int *calls, float *split_ms, float *product_ms);

/* Human-readable text for the last failure on this handle (host string owned by the handle). */
const char *ecgemm_last_error_string(ecgemm_handle_t handle);

/* Position (1 = the handle, 2 = the next parameter, ...) in the failing function's parameter list of the first
 * argument that the last failed call on this handle found invalid; 0 when that failure was not about one argument
 * (a HIP error, a workspace that is too small) or when no call has failed yet.  -1 for a NULL handle. */
int ecgemm_last_error_argument(ecgemm_handle_t handle);

/* Static name of a status code. */
const char *ecgemm_status_string(ecgemm_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* ECGEMM_H */
