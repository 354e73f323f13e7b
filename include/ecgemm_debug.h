/*
 * ecgemm: the part of the C-ABI that production callers do not need.
 *
 * Knobs and diagnostics used by the tests, the tuning sweeps and the accuracy experiments: forcing a kernel shape,
 * the comparison methods of the paper (run through the same kernels so that its error curves can be redrawn on this
 * hardware), and two kernels that execute bare matrix instructions.  Conventions as in ecgemm.h.
 */
#ifndef ECGEMM_DEBUG_H
#define ECGEMM_DEBUG_H

#include "ecgemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The comparison methods among the ecgemm_mode_t values (the enumerators themselves are in ecgemm.h):
 *
 *   ECGEMM_MODE_FP16_MARKIDIS (2)     Markidis' method: unscaled residual dv16 = toFP16(v - v16) (Eqs. corr-1 .. corr-4),
 *                                     all four products dA dB + dA B + A dB + A B summed in one accumulator (Eq. corr-5,
 *                                     listing "Markidis' error correction method").
 *   ECGEMM_MODE_FP16_UNSCALED (3)     the method's three products and separate correction accumulator, but on Markidis'
 *                                     unscaled residual: isolates what the 2^11 scaling of section "Reducing the
 *                                     underflow ..." buys.
 *   ECGEMM_MODE_FP16_PLAIN (4)        toFP16(A) toFP16(B), one product, no correction (listing "A simple matrix-matrix
 *                                     multiplication ...").
 *   ECGEMM_MODE_BF16_PLAIN (5)        toBF16(A) toBF16(B), one product, no correction.
 *   ECGEMM_MODE_FP16_OUTSIDE_ACC (6)  ECGEMM_MODE_FP16_SPLIT exactly as the paper's listing has it: A16 B16 is multiplied
 *                                     into a zeroed temporary and added to the running sum outside the matrix unit, every
 *                                     k step (section "Avoiding RZ during Tensor Core accumulation").  On this hardware
 *                                     the matrix unit already rounds to nearest, so this only costs time; kept to show that.
 *   ECGEMM_MODE_FP32_MFMA (7)         no splitting at all: A B in FP32 on the matrix unit (v_mfma_f32_32x32x2_f32), through
 *                                     the same repacking pass and the same product kernel.  The FP32 GEMM that the paper
 *                                     sets its method against (its cuBLAS SGEMM column), on this hardware and in this code
 *                                     base, for throughput, energy and error comparisons.
 *
 *   ECGEMM_MODE_FP16_OUTSIDE_ACC_4 (8), ECGEMM_MODE_FP16_OUTSIDE_ACC_16 (9)
 *                                     between that listing and the default: A16 B16 stays in the matrix unit's accumulator
 *                                     for 4 or 16 k steps of 16 (64 or 256 deep) and only then joins the running sum kept
 *                                     outside, which shows how much of the listing's small accuracy gain a longer interval
 *                                     keeps, and at what cost.
 *
 * They exist in one kernel shape each (block tile 256 x 128; the three "outside" modes 128 x 128, one block per unit),
 * addressed as ECGEMM_SHAPE_256x128_W4.
 */

/*
 * Kernel shape of the product (steps 2 and 3 of ecgemm_sgemm); a tuning and test knob.  The paper's counterpart are the
 * block and warp tile sizes that it picks for each matrix size by grid search (section "Parameter tuning of CUTLASS").
 * ECGEMM_SHAPE_AUTO (the default) picks per call from the mode and the problem size.  The others force one shape for
 * every later ecgemm_sgemm / ecgemm_product / ecgemm_workspace_size on the handle:
 *   256x128_W4     block tile 256 x 128, 4 waves of 128 x 64, one block per compute unit (every mode);
 *   128x128_X2     block tile 128 x 128, 4 waves of 64 x 64, two blocks per compute unit (the two modes of the method);
 *   64x64_FUSED    the paper's own arrangement (last paragraph of section "Incorporating our method into CUTLASS"):
 *                  one kernel reads the FP32 operands, splits them in registers and multiplies; no split pass, no
 *                  packed operands in the workspace, one launch (the two modes of the method; ecgemm_sgemm,
 *                  ecgemm_sgemm_scaled and ecgemm_sgemm_noalloc only).  Block tile 64 x 64: eight waves that fetch
 *                  and split, four that multiply 32 x 32 each; every block splits the rows of A and columns of B that
 *                  it uses again, so this is for small products, where launches and latencies decide the time.  A
 *                  block takes the whole depth, unless the tiles are so few that slices of it (at least 512 deep, a
 *                  block each, all blocks in one round of the compute units) are estimated to be faster: then every
 *                  tile is cut, the blocks leave partial sums in the workspace and a second launch adds them up.
 *   32x32_FUSED    the same with block tile 32 x 32: eight waves fetch and split, one multiplies.  Four times the
 *                  blocks with half the split work each: for products so small that 64 x 64 tiles leave most
 *                  compute units idle.
 * All shapes form the same products in the same per-element order; results agree bit for bit between shapes unless
 * output tiles are sliced along K differently.  A call whose mode has no kernel of the forced shape returns
 * ECGEMM_ERR_UNSUPPORTED.
 */
typedef enum {
  ECGEMM_SHAPE_AUTO = 0,
  ECGEMM_SHAPE_256x128_W4 = 1,
  ECGEMM_SHAPE_128x128_X2 = 2,
  ECGEMM_SHAPE_64x64_FUSED = 3,
  ECGEMM_SHAPE_32x32_FUSED = 4
} ecgemm_shape_t;
ecgemm_status_t ecgemm_set_shape(ecgemm_handle_t handle, ecgemm_shape_t shape);

/*
 * Experiment knob for the order in which output tiles are handed to the compute units (it decides what the eight XCDs'
 * L2 caches share; the defaults are what measurements picked).  xcd_remap = 1 (default): each XCD owns a contiguous run
 * of the tile order; 0: tiles go to workgroups in launch order and the hardware's round-robin spreads neighbours over all
 * XCDs.  group_m > 0 forces the number of tile rows per group of the order (default 0: 4, or 8 for the 128 x 128 shape
 * on shallow products; a value of at least the number of tile rows gives plain column-major order).  column_bands in
 * 1 .. 8 forces the number of column bands (default 0: chosen from the size of the operand panels).  Every element is
 * still summed in the same order, so results do not change - except that the tiles which are cut into slices along K
 * are the last of the order, whichever those are, and a tile sums differently (to FP32 rounding) sliced than whole.
 * Affects later ecgemm_sgemm / ecgemm_product / ecgemm_plan_info on the handle.
 */
ecgemm_status_t ecgemm_debug_set_tile_order(ecgemm_handle_t handle, int xcd_remap, int group_m, int column_bands);

/*
 * Host only, for tests: the coordinates of output tile number 0, 1, ... in the order in which ecgemm_sgemm on this
 * handle would hand the tiles of this problem out (ecgemm_plan_info gives tiles_m x tiles_n, the size the two host
 * arrays must have; `handle` may be NULL as there).  The kernels find a tile's coordinates with multiplications by
 * reciprocals that the host prepares; `disagreements` (host pointer) receives the number of tiles for which that
 * arithmetic and plain integer division give different coordinates, which must be 0.  ECGEMM_ERR_UNSUPPORTED for a
 * problem that ecgemm_sgemm runs as one launch (the one-launch shapes number their tiles with plain divisions).
 */
ecgemm_status_t ecgemm_debug_tile_order(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode,
                                        int32_t *tile_m, int32_t *tile_n, int64_t *disagreements);

/*
 * Diagnostic: executes `count` independent v_mfma_f32_32x32x16_f16 (bf16 == 0) or _bf16 (bf16 != 0) instructions,
 * D = A B + C with A 32 x 16, B 16 x 32, C and D 32 x 32, on registers given lane by lane, so that tests can state what
 * the matrix unit does (the method's accumulation discipline, section "Avoiding RZ during Tensor Core accumulation",
 * depends on it).  For problem p and lane l (0..63): a[(p*64 + l)*8 + e] = A(l % 32, 8*(l/32) + e),
 * b[(p*64 + l)*8 + e] = B(8*(l/32) + e, l % 32), c and d [(p*64 + l)*16 + v] = element (8*(v/4) + 4*(l/32) + v%4, l % 32).
 * a, b: device, 16-bit patterns, 16-byte aligned; c, d: device FP32, 64-byte aligned; d may equal c.
 */
ecgemm_status_t ecgemm_debug_mfma(ecgemm_handle_t handle, int bf16, int64_t count, const void *a, const void *b,
                                  const float *c, float *d);

/*
 * Diagnostic: enqueues a kernel of `blocks` workgroups x 4 waves that does nothing but `iters` x 24 matrix
 * instructions per wave (FP16 if bf16 == 0, else BF16) on operands read once from `operands` (device, 12 x 256 x 8
 * 16-bit values = 48 KiB, 16-byte aligned).  `sink`: device, blocks x 256 floats, receives a checksum.  `flops`
 * (host pointer) receives the floating-point operations the kernel performs; timing it (the caller brackets it with
 * events on the handle's stream) gives the rate the matrix pipes sustain for that operand content on this device,
 * against which the product kernel's rate can be read.
 */
ecgemm_status_t ecgemm_debug_mfma_rate(ecgemm_handle_t handle, int bf16, const void *operands, float *sink, int blocks,
                                       int iters, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* ECGEMM_DEBUG_H */
