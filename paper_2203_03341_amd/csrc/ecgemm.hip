// Host side of the ecgemm C-ABI (see include/ecgemm.h): argument checks, workspace, kernel launches.
#include "../../include/ecgemm.h"
#include "../../include/ecgemm_debug.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "helper_kernels.hpp"
#include "kernel_list.hpp"

using namespace ecgemm;

struct TimedCall {
  hipEvent_t start, split_done, product_done;
};

struct ecgemm_context {
  int device = 0;
  int compute_units = 256;
  hipStream_t stream = nullptr;
  void* own_workspace = nullptr;
  size_t own_bytes = 0;
  void* user_workspace = nullptr;
  size_t user_bytes = 0;
  bool timing = false;
  int log2_scale_a = 0, log2_scale_b = 0;
  ecgemm_shape_t shape = ECGEMM_SHAPE_AUTO;
  int xcd_remap = 1, forced_group_m = 0, forced_column_bands = 0;  // ecgemm_debug_set_tile_order
  int* range_buffer = nullptr;  // two ints of device memory for ecgemm_exponent_range
  char* builtin_workspace = nullptr;  // this device's copy of the library's built-in workspace (ecgemm_sgemm_noalloc)
  int last_error_argument = 0;
  const int* auto_choice = nullptr;  // device: where the last ecgemm_sgemm call, if ECGEMM_MODE_AUTO, leaves its choice
  std::vector<TimedCall> timed;
  std::vector<hipEvent_t> free_events;
  std::string last_error;
};

namespace {

typedef void (*reduce_fn_t)(const float*, int, int, int, int, int, int, int, int64_t, int64_t, float, float, float*, int64_t,
                            const int*, int, int);
struct FusedKernels {
  void (*kernel[3][3])(FusedParams);  // [FusedLayout of A][FusedLayout of B]
};
template <int METHOD, int TILE>
constexpr FusedKernels fused_kernels_of() {
  return FusedKernels{{{fused_kernel<METHOD, 0, 0, TILE>, fused_kernel<METHOD, 0, 1, TILE>, fused_kernel<METHOD, 0, 2, TILE>},
                       {fused_kernel<METHOD, 1, 0, TILE>, fused_kernel<METHOD, 1, 1, TILE>, fused_kernel<METHOD, 1, 2, TILE>},
                       {fused_kernel<METHOD, 2, 0, TILE>, fused_kernel<METHOD, 2, 1, TILE>, fused_kernel<METHOD, 2, 2, TILE>}}};
}
const FusedKernels kFusedFp16Tile64 = fused_kernels_of<kMethodFp16Split, 64>(), kFusedFp16Tile32 = fused_kernels_of<kMethodFp16Split, 32>(),
                   kFusedBf16Tile64 = fused_kernels_of<kMethodBf16Full, 64>(), kFusedBf16Tile32 = fused_kernels_of<kMethodBf16Full, 32>();
struct Shape {
  void (*product)(ProductParams);  // steps 2 to 5 on packed operands, or
  void (*product_scaled)(ProductParams);  // the instance to prefer for calls with scaling vectors, if the mode has one
  const FusedKernels* fused;       // steps 1 to 5 on the FP32 operands: one kernel per pair of operand layouts
  reduce_fn_t reduce;
  int bm, bn, bk, threads, blocks_per_cu;
  // Deepest K for which the kernel runs as a persistent grid: one block per CU, each walking through several items
  // with the next item's first loads in flight during its epilogue.  Beyond it, one block per item, handed out in
  // order by the hardware as CUs free up, which keeps the tiles an XCD works on at any time next to each other: blocks
  // of a persistent grid drift apart over long items and lose L2 hits (72 % instead of 82 % at 16384^3).
  // Two co-resident X2 blocks already cover each other's epilogue and never gain.
  int persistent_max_k;
};
template <class Cfg, bool WITH_SCALED = false>
constexpr Shape shape_of(int persistent_max_k) {
  void (*scaled)(ProductParams) = nullptr;
  if constexpr (WITH_SCALED) scaled = product_kernel<Cfg, true>;
  return Shape{product_kernel<Cfg, false>, scaled, nullptr, reduce_tail_kernel<Cfg::BM, Cfg::BN>, Cfg::BM, Cfg::BN, Cfg::BK,
               Cfg::THREADS, Cfg::BLOCKS_PER_CU, persistent_max_k};
}
template <int TILE>
inline Shape fused_shape(const FusedKernels* kernels) {  // (the reduction only for plans that slice the depth)
  return Shape{nullptr, nullptr, kernels, reduce_tail_kernel<TILE, TILE>, TILE, TILE, 32, fused_threads(TILE), 1, 0};
}
constexpr Shape kNoShape{nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, 0, 0};
constexpr int kShapeCount = 4;
// [mode][ecgemm_shape_t - 1]
constexpr int kPersistentMaxK = 4096;
const Shape kShapes[kMethods][kShapeCount] = {
    {shape_of<Fp16W4, true>(kPersistentMaxK), shape_of<Fp16X2, true>(0), fused_shape<64>(&kFusedFp16Tile64), fused_shape<32>(&kFusedFp16Tile32)},
    {shape_of<Bf16W4, true>(kPersistentMaxK), shape_of<Bf16X2, true>(0), fused_shape<64>(&kFusedBf16Tile64), fused_shape<32>(&kFusedBf16Tile32)},
    {shape_of<MarkidisConfig>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<UnscaledConfig>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<PlainFp16Config>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<PlainBf16Config>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<OutsideConfig>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<Fp32Config>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<Outside4Config>(4096), kNoShape, kNoShape, kNoShape},
    {shape_of<Outside16Config>(4096), kNoShape, kNoShape, kNoShape},
};

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
// the ecgemm_mode_t values are the ProductMethod values
inline int parts_of(ecgemm_mode_t mode) { return parts_of_split(split_kind_of((int)mode)); }
inline bool valid_mode(int mode) { return mode >= 0 && mode < kMethods; }  // a mode with kernels of its own
inline bool valid_mode_or_auto(int mode) { return valid_mode(mode) || mode == (int)ECGEMM_MODE_AUTO; }
static_assert((int)ECGEMM_MODE_FP16_SPLIT == (int)kMethodFp16Split && (int)ECGEMM_MODE_BF16_FULL == (int)kMethodBf16Full &&
              (int)ECGEMM_MODE_FP16_MARKIDIS == (int)kMethodFp16Markidis &&
              (int)ECGEMM_MODE_FP16_UNSCALED == (int)kMethodFp16Unscaled &&
              (int)ECGEMM_MODE_FP16_PLAIN == (int)kMethodFp16Plain && (int)ECGEMM_MODE_BF16_PLAIN == (int)kMethodBf16Plain &&
              (int)ECGEMM_MODE_FP16_OUTSIDE_ACC == (int)kMethodFp16Outside && (int)ECGEMM_MODE_FP32_MFMA == (int)kMethodFp32 &&
                  (int)ECGEMM_MODE_FP16_OUTSIDE_ACC_4 == (int)kMethodFp16Outside4 &&
                  (int)ECGEMM_MODE_FP16_OUTSIDE_ACC_16 == (int)kMethodFp16Outside16,
              "mode numbering");
inline bool valid_shape(int shape) { return shape >= ECGEMM_SHAPE_AUTO && shape <= ECGEMM_SHAPE_32x32_FUSED; }
inline bool valid_op(int op) { return op == ECGEMM_OP_N || op == ECGEMM_OP_T; }

size_t packed_bytes(int64_t rows, int64_t depth, ecgemm_mode_t mode) {
  return (size_t)round_up(rows, kRowPad) * (size_t)round_up(depth, kDepthPad) * 2 * parts_of(mode);
}

struct Plan {
  const Shape* shape;  // null: the requested shape does not exist for the mode, or (too_many_tiles) cannot count this problem's tiles
  bool too_many_tiles = false;
  int64_t Kp;
  int tiles_m, tiles_n, k_tiles;
  int full_tiles, tail_tiles, tail_splits;  // see ProductParams
  size_t a_bytes, b_bytes, partial_bytes, total_bytes;
  int64_t items() const { return (int64_t)full_tiles + (int64_t)tail_tiles * tail_splits; }
};

// The plan is made for the 256 compute units of the MI355X whatever device the handle is on, so that the workspace
// size is a function of the problem (and the shape, if the caller fixed one) alone.
constexpr int kPlanComputeUnits = 256;

// Tiles of one shape, and how they become work items.  As many tiles as fill every workgroup slot of the chip a whole
// number of times are one item each.  The tiles left over would occupy only part of the chip for the time of a whole
// tile; each of them can be cut into `splits` slices along K, which leave partial sums for a second kernel to add up
// in a fixed order.  splits == 1: nothing is sliced.
Plan plan_with(int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode, ecgemm_shape_t shape, int splits) {
  Plan pl;
  pl.Kp = round_up(K, kDepthPad);
  pl.shape = &kShapes[(int)mode][(int)shape - 1];
  if (pl.shape->product == nullptr && pl.shape->fused == nullptr) {
    pl.shape = nullptr;
    return pl;
  }
  const int bm = pl.shape->bm, bn = pl.shape->bn;
  // (check_sizes bounds the tiles of 128 x 128; the smaller tiles of the one-launch shapes must fit 32 bits as well)
  if (((M + bm - 1) / bm) * ((N + bn - 1) / bn) > ((int64_t)1 << 30)) {
    pl.shape = nullptr;
    pl.too_many_tiles = true;
    return pl;
  }
  pl.tiles_m = (int)((M + bm - 1) / bm);
  pl.tiles_n = (int)((N + bn - 1) / bn);
  pl.k_tiles = (int)(pl.Kp / pl.shape->bk);
  const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
  const int64_t slots = (int64_t)kPlanComputeUnits * pl.shape->blocks_per_cu;
  // (a one-launch plan slices every tile or none: its blocks take the whole depth unless the caller asks for slices)
  const int64_t tail = pl.shape->fused ? (splits > 1 ? tiles : 0) : tiles % slots;
  if (tail == 0) splits = 1;
  pl.tail_splits = splits;
  pl.tail_tiles = splits > 1 ? (int)tail : 0;
  pl.full_tiles = (int)(tiles - pl.tail_tiles);
  pl.a_bytes = pl.shape->fused ? 0 : align256(packed_bytes(M, K, mode));
  pl.b_bytes = pl.shape->fused ? 0 : align256(packed_bytes(N, K, mode));
  pl.partial_bytes = splits > 1 ? align256((size_t)splits * tail * bm * bn * sizeof(float)) : 0;
  pl.total_bytes = pl.a_bytes + pl.b_bytes + pl.partial_bytes;
  return pl;
}

// Estimated time of the product (and reduce) kernels of a plan in microseconds, to rank the plans of one problem.
// Items are handed out in rounds (one per compute unit for the 256 x 128 shape, two for the 128 x 128 shape); a round
// of n equal items takes the larger of two times per 1024 of depth: what one compute unit needs for its share at its
// own pace (kW4Unit for a 256 x 128 tile; 2 kX2Pair for two co-resident 128 x 128 tiles; kX2Lone, growing with depth,
// for one that has the unit to itself: it cannot hide all of the latency alone), and what the chip as a
// whole, which is power-limited, needs for the round's work (kChip per 128 x 128 tile and unit when all are busy,
// falling with the filled fraction of the round to the power kFillExponent; the 256 x 128 shape needs kW4Work of that
// per flop).  Every round adds a pipeline fill and an epilogue, sliced tiles a
// pass over their partial sums.  Work scales with the mode's matrix instructions per element.  The constants are a
// least-squares fit to 1300 timings: both shapes with every admissible slice count on 174 problems (squares from
// 512 to 5632, random M, N in 512..10000 and K in 256..23000, both modes).  Picking the cheapest plan is within 0.6 %
// of the best measured plan on average over these problems, 3 of them more than 5 % off (worst 11 %).
constexpr double kW4Unit = 22.03, kW4Work = 0.954, kX2Pair = 14.74, kX2Lone = 10.08, kX2LonePerDepth = 0.277, kChip = 17.46;
constexpr double kFillExponent = 0.906, kW4RoundUs = 7.88, kX2RoundUs = 4.70, kReduceUs = 1.01, kReduceUsPerMB = 0.142;

double mode_work(ecgemm_mode_t mode) {  // matrix-pipe time per element relative to the three FP16 products
  switch (mode) {
    case ECGEMM_MODE_FP16_SPLIT:
    case ECGEMM_MODE_FP16_UNSCALED: return 1.0;
    case ECGEMM_MODE_BF16_FULL:
    case ECGEMM_MODE_FP16_OUTSIDE_ACC: return 2.0;
    case ECGEMM_MODE_FP16_OUTSIDE_ACC_4:
    case ECGEMM_MODE_FP16_OUTSIDE_ACC_16: return 1.2;
    case ECGEMM_MODE_FP16_MARKIDIS: return 4.0 / 3.0;
    case ECGEMM_MODE_FP32_MFMA: return 3.0;
    default: return 1.0 / 3.0;  // one product
  }
}

double rounds_us(int64_t items, double depth, bool w4, double work) {  // `items` equal items, each `depth` x 1024 deep
  const int64_t per_round = w4 ? kPlanComputeUnits : 2 * kPlanComputeUnits;
  double us = 0.0;
  for (int64_t left = items; left > 0; left -= per_round) {
    const double n = (double)std::min(left, per_round);
    const double unit = w4 ? kW4Unit : n > kPlanComputeUnits ? 2.0 * kX2Pair : kX2Lone + kX2LonePerDepth * std::min(depth, 20.0);
    const double chip = 2.0 * (w4 ? kW4Work : 1.0) * std::pow(n / per_round, kFillExponent) * kChip;
    us += depth * work * std::max(unit, chip) + (w4 ? kW4RoundUs : kX2RoundUs);
    if (left > 64 * per_round) {  // many equal rounds: no need to walk them one by one
      const int64_t whole_rounds = left / per_round - 1;
      us += whole_rounds * (depth * work * std::max(unit, chip) + (w4 ? kW4RoundUs : kX2RoundUs));
      left -= whole_rounds * per_round;
    }
  }
  return us;
}

double estimated_us(const Plan& pl, ecgemm_mode_t mode) {
  const bool w4 = pl.shape->bm == 256;
  const double work = mode_work(mode);
  const int64_t sliced = pl.tail_splits > 1 ? (int64_t)pl.tail_tiles * pl.tail_splits : 0;
  const double slice_depth = pl.tail_splits > 1 ? (double)((pl.k_tiles + pl.tail_splits - 1) / pl.tail_splits) * pl.shape->bk / 1024.0 : 0.0;
  double us = rounds_us(pl.full_tiles, pl.Kp / 1024.0, w4, work) + rounds_us(sliced, slice_depth, w4, work);
  if (sliced > 0)
    us += kReduceUs + kReduceUsPerMB * (pl.tail_splits + 1.0) * pl.tail_tiles * pl.shape->bm * pl.shape->bn * 4.0 / 1e6;
  return us;
}

// The cheapest way to slice the leftover tiles of one shape: slices at least 512 deep, none of them empty, at most
// 1024 of them in all (128 MiB of partial sums).
// How a caller wants the one-launch shapes: not at all (it needs packed operands), with every block over the whole
// depth (the automatic mode, whose kernels look at the choice themselves), or also with the depth in slices.
enum OneLaunch { kOneLaunchNever = 0, kOneLaunchWhole = 1, kOneLaunchSliced = 2 };
double one_launch_us(const Plan& pl, int64_t K, ecgemm_mode_t mode);
// Chunks of 64 per slice of a one-launch plan: equal shares rounded up to whole in-register slices (512 deep).
int64_t fused_chunks_per_slice(int64_t K, int splits) {
  const int64_t chunks = (K + 63) / 64;
  return round_up((chunks + splits - 1) / splits, (int64_t)kFusedSliceChunks);
}
Plan plan_with_shape(int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode, ecgemm_shape_t shape, OneLaunch one_launch) {
  Plan best = plan_with(M, N, K, mode, shape, 1);
  if (best.shape == nullptr) return best;
  const int64_t slots = (int64_t)kPlanComputeUnits * best.shape->blocks_per_cu;
  const int64_t tiles = (int64_t)best.tiles_m * best.tiles_n;
  if (best.shape->fused) {
    // Deep products of few tiles: slices at least 512 deep, none empty, all blocks in one round.
    if (one_launch != kOneLaunchSliced) return best;
    double best_us = one_launch_us(best, K, mode);
    for (int splits = 2; splits <= 64 && splits * tiles <= kPlanComputeUnits && splits <= K / 512; ++splits) {
      if (fused_chunks_per_slice(K, splits) * (splits - 1) >= (K + 63) / 64) continue;  // the last slice would be empty
      const Plan pl = plan_with(M, N, K, mode, shape, splits);
      const double us = one_launch_us(pl, K, mode);
      if (us < best_us) best = pl, best_us = us;
    }
    return best;
  }
  const int64_t tail = tiles % slots;
  if (tail == 0) return best;
  double best_us = estimated_us(best, mode);
  for (int splits = 2; splits <= 64 && splits <= best.Kp / 512 && splits * tail <= 1024; ++splits) {
    const int per_slice = (best.k_tiles + splits - 1) / splits;
    if ((int64_t)per_slice * (splits - 1) >= best.k_tiles) continue;  // the last slice would be empty
    const Plan pl = plan_with(M, N, K, mode, shape, splits);
    const double us = estimated_us(pl, mode);
    if (us < best_us) best = pl, best_us = us;
  }
  return best;
}

// Estimated time of a whole call in microseconds, for the choice between splitting first and the one-launch shapes.
// Both are fits to timings of back-to-back calls on one MI355X (squares from 64 to 1536 and a dozen other small
// shapes, both modes).
//   split first: the product estimate above, the launches (5.6 us), and the split pass, which costs about 1 us per MB
//   of FP32 operands (1.4 us with three BF16 parts to write) up to 8.5 us, and 0.45 (0.55) us per MB beyond: operands
//   much larger than the product (deep products of small matrices) are a pass at the memory's pace.
//   one launch: 4.4 us, then the blocks in rounds of one per compute unit (a block's 9 or 12 waves leave no registers
//   for a second one beside it).  A round is what a block needs per 64-deep chunk (0.33 / 0.58 us for 32 / 64 tiles in
//   FP16 mode, 0.46 / 0.76 in BF16 mode; a fifth more for 64 x 64 BF16 blocks once nearly every unit has one) plus
//   its first loads and its stores, which are nearly free in a single round (0.4 to 1.1 us) and cost 1.6 to 3 us per
//   round when rounds follow each other.  A last chunk that is not whole takes the slower, general split (three
//   chunks' worth).
double split_first_us(const Plan& pl, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode) {
  const double operand_mb = 4.0 * ((double)M + (double)N) * (double)K / 1e6;
  // (beyond 8.5 us the pass runs at the memory's pace: 8 or 10 bytes moved per element)
  const bool bf16 = mode == ECGEMM_MODE_BF16_FULL;
  const double small_pass = (bf16 ? 1.4 : 1.0) * operand_mb;
  return estimated_us(pl, mode) + 5.6 + (small_pass <= 8.5 ? small_pass : 8.5 + (bf16 ? 0.55 : 0.45) * (operand_mb - 8.5 / (bf16 ? 1.4 : 1.0)));
}
double one_launch_us(const Plan& pl, int64_t K, ecgemm_mode_t mode) {
  const bool bf16 = mode == ECGEMM_MODE_BF16_FULL, small = pl.shape->bm == 32;
  const double per_chunk = small ? (bf16 ? 0.46 : 0.33) : (bf16 ? 0.76 : 0.58);
  const double blocks_per_unit = (double)pl.tiles_m * pl.tiles_n / kPlanComputeUnits;
  const double rounds = std::max(1.0, std::ceil(blocks_per_unit - 1e-9));
  if (pl.tail_splits > 1) {
    // slices of the depth (one round by construction): a block's share, then the kernel that adds the slices up
    // (2.2 us behind the first kernel, and a pass over the partial sums)
    const double share = (double)fused_chunks_per_slice(K, pl.tail_splits), partial_mb = pl.partial_bytes / 1e6;
    return 4.4 + (small ? (bf16 ? 0.7 : 0.4) : (bf16 ? 1.1 : 0.8)) + share * per_chunk + 2.2 + 0.35 * partial_mb;
  }
  const double chunks = (double)(K / 64) + (K % 64 ? 3.0 : 0.0);
  if (rounds == 1.0) {
    const double nearly_full = (!small && bf16 && blocks_per_unit > 0.9) ? 1.2 : 1.0;
    return 4.4 + (small ? (bf16 ? 0.7 : 0.4) : (bf16 ? 1.1 : 0.8)) + chunks * per_chunk * nearly_full;
  }
  const double per_round = small ? (bf16 ? 2.7 : 1.6) : (bf16 ? 3.0 : 2.0);
  return 4.4 + rounds * (per_round + chunks * per_chunk);
}

// The plan of a call.  With a shape forced by the caller, that shape.  Otherwise the cheaper of the two product shapes
// by the product estimate (the comparison methods have the 256 x 128 shape only), unless a one-launch shape is
// allowed (ecgemm_sgemm and what describes it; not for callers that need the packed operands) and estimated to take
// less than 0.85 of the time: the estimates know nothing of the operands' layouts, which move either by a tenth.
Plan choose_plan(int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode, ecgemm_shape_t shape, OneLaunch one_launch) {
  if (shape != ECGEMM_SHAPE_AUTO) return plan_with_shape(M, N, K, mode, shape, one_launch);
  const Plan w4 = plan_with_shape(M, N, K, mode, ECGEMM_SHAPE_256x128_W4, one_launch);
  if (mode != ECGEMM_MODE_FP16_SPLIT && mode != ECGEMM_MODE_BF16_FULL) return w4;
  const Plan x2 = plan_with_shape(M, N, K, mode, ECGEMM_SHAPE_128x128_X2, one_launch);
  const Plan split_first = estimated_us(x2, mode) < estimated_us(w4, mode) ? x2 : w4;
  // (a one-launch block walks the whole depth, or its slice of it, and an operand is split once per block row or
  // column: beyond these bounds it never wins, and its tile count stays far inside 32 bits)
  if (one_launch == kOneLaunchNever || M > 16384 || N > 16384 || (K > 8192 && one_launch != kOneLaunchSliced)) return split_first;
  const Plan tile64 = plan_with_shape(M, N, K, mode, ECGEMM_SHAPE_64x64_FUSED, one_launch);
  const Plan tile32 = plan_with_shape(M, N, K, mode, ECGEMM_SHAPE_32x32_FUSED, one_launch);
  // (near a tie the larger tile, which is less at the mercy of the operands' layout)
  if (K > 8192 && tile64.tail_splits == 1 && tile32.tail_splits == 1) return split_first;  // too many tiles for slices
  const Plan one = one_launch_us(tile32, K, mode) < 0.95 * one_launch_us(tile64, K, mode) ? tile32 : tile64;
  return one_launch_us(one, K, mode) < 0.85 * split_first_us(split_first, M, N, K, mode) ? one : split_first;
}

// A plan is a pure function of its arguments, and loops call the library with the same ones over and over: the last
// few plans of each thread are kept (ranking up to 128 candidate plans costs a few microseconds, which matters next to
// a 12 us call; the automatic mode needs two plans per call).
Plan make_plan(int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode, ecgemm_shape_t shape, OneLaunch one_launch) {
  struct Entry {
    int64_t M = -1, N = -1, K = -1;
    int mode = -1, shape = -1;
    int one_launch = -1;
    Plan plan;
  };
  constexpr int kEntries = 4;
  thread_local Entry cache[kEntries];
  thread_local int next = 0;
  for (const Entry& e : cache)
    if (e.M == M && e.N == N && e.K == K && e.mode == (int)mode && e.shape == (int)shape && e.one_launch == (int)one_launch)
      return e.plan;
  Entry& e = cache[next];
  next = (next + 1) % kEntries;
  e.plan = choose_plan(M, N, K, mode, shape, one_launch);
  e.M = M, e.N = N, e.K = K, e.mode = (int)mode, e.shape = (int)shape, e.one_launch = (int)one_launch;
  return e.plan;
}

// ECGEMM_MODE_AUTO: both candidate plans, and a workspace that serves either.  The statistics arrays have one entry per
// 64 x 32 block of the padded operand, the most any split kernel variant launches (which variant runs depends on the
// operands' alignment, and the workspace size must not).
constexpr double kAutoTolerance = 0x1p-24;
constexpr double kAutoMinTerms = 16.0;  // see choose_mode_kernel
struct AutoPlan {
  Plan fp16, bf16;
  bool exists;
  size_t packed_bytes, partial_bytes, stats_a_bytes, stats_b_bytes, scales_a_bytes, scales_b_bytes, total_bytes;
};
AutoPlan make_auto_plan(int64_t M, int64_t N, int64_t K, ecgemm_shape_t shape) {
  AutoPlan ap;
  ap.fp16 = make_plan(M, N, K, ECGEMM_MODE_FP16_SPLIT, shape, kOneLaunchNever);
  ap.bf16 = make_plan(M, N, K, ECGEMM_MODE_BF16_FULL, shape, kOneLaunchNever);
  ap.exists = ap.fp16.shape && ap.bf16.shape && !ap.fp16.shape->fused && !ap.bf16.shape->fused;
  if (!ap.exists) return ap;
  const size_t blocks_per_row_block = (size_t)(round_up(K, kDepthPad) / 32);
  ap.packed_bytes = std::max(ap.fp16.a_bytes + ap.fp16.b_bytes, ap.bf16.a_bytes + ap.bf16.b_bytes);
  ap.partial_bytes = std::max(ap.fp16.partial_bytes, ap.bf16.partial_bytes);
  // (a candidate that ecgemm_sgemm would run as one launch runs so here too, with its own partial sums if it slices)
  ap.partial_bytes = std::max(ap.partial_bytes, std::max(make_plan(M, N, K, ECGEMM_MODE_FP16_SPLIT, shape, kOneLaunchSliced).partial_bytes,
                                                         make_plan(M, N, K, ECGEMM_MODE_BF16_FULL, shape, kOneLaunchSliced).partial_bytes));
  const size_t per_block = kStatsPerBlock * sizeof(double);
  ap.stats_a_bytes = align256(per_block * blocks_per_row_block * (size_t)(round_up(M, kRowPad) / 64));
  ap.stats_b_bytes = align256(per_block * blocks_per_row_block * (size_t)(round_up(N, kRowPad) / 64));
  ap.scales_a_bytes = align256(sizeof(int32_t) * (size_t)M);
  ap.scales_b_bytes = align256(sizeof(int32_t) * (size_t)N);
  ap.total_bytes = ap.packed_bytes + ap.partial_bytes + ap.stats_a_bytes + ap.stats_b_bytes + ap.scales_a_bytes +
                   ap.scales_b_bytes + 256;
  return ap;
}

ecgemm_status_t fail(ecgemm_handle_t h, ecgemm_status_t st, const std::string& what, int argument = 0) {
  if (h) h->last_error = what, h->last_error_argument = argument;
  return st;
}
// the refusal of a problem for which make_plan returned no shape
ecgemm_status_t no_plan(ecgemm_handle_t h, const Plan& pl, const char* function) {
  return fail(h, ECGEMM_ERR_UNSUPPORTED,
              std::string(function) + (pl.too_many_tiles ? ": M x N has more than 2^30 tiles of the handle's kernel shape"
                                                         : ": the handle's kernel shape does not exist for this mode"));
}

// ECGEMM_ERR_INVALID_ARG for the argument at `position` of the failing function's parameter list (1 = the handle)
ecgemm_status_t bad_arg(ecgemm_handle_t h, int position, const char* what) {
  return fail(h, ECGEMM_ERR_INVALID_ARG, what, position);
}

ecgemm_status_t hip_fail(ecgemm_handle_t h, hipError_t e, const char* where) {
  return fail(h, ECGEMM_ERR_HIP, std::string(where) + ": " + hipGetErrorString(e));
}

#define ECGEMM_HIP(h, call)                                   \
  do {                                                        \
    hipError_t e_ = (call);                                   \
    if (e_ != hipSuccess) return hip_fail((h), e_, #call);    \
  } while (0)

// X = op(src) is rows x depth.  op == N: X(r, k) = src[r + k * ld]; op == T: X(r, k) = src[k + r * ld].
ecgemm_status_t make_split_job(ecgemm_handle_t h, ecgemm_op_t op, int64_t rows, int64_t depth, const float* src, int64_t ld,
                               void* packed, int log2_prescale, const int* row_log2_scale, SplitJob* job) {
  const int64_t Rp = round_up(rows, kRowPad), Kp = round_up(depth, kDepthPad);
  const int64_t blocks64 = (Kp / 32) * (Rp / 64);
  if (blocks64 > 0x7fffffff) return fail(h, ECGEMM_ERR_INVALID_ARG, "operand has more than 2^42 elements");
  const bool k_contiguous = op == ECGEMM_OP_T;
  const bool vec = (ld % 4 == 0) && ((uintptr_t)src % 16 == 0);
  job->src = src;
  job->ld = ld;
  job->rows = rows;
  job->depth = depth;
  job->k_steps_total = Kp / 16;
  job->prescale = std::ldexp(1.0f, log2_prescale);
  job->row_log2_scale = row_log2_scale;
  job->packed = static_cast<unsigned short*>(packed);
  job->stats = nullptr;
  job->gate = nullptr;
  job->gate_value = 0;
  job->row_max = nullptr;
  job->variant = k_contiguous ? (vec ? kSplitKContiguousVec : kSplitKContiguous) : (vec ? kSplitRContiguousWide : kSplitRContiguous);
  // blocks are 64 rows x 32 k, except 256 x 32 (wide) and 64 x 64 (k contiguous, unaligned)
  switch (job->variant) {
    case kSplitRContiguousWide: job->fast_tiles = (unsigned)(Rp / 256), job->blocks = (unsigned)(blocks64 / 4); break;
    case kSplitRContiguous: job->fast_tiles = (unsigned)(Rp / 64), job->blocks = (unsigned)blocks64; break;
    case kSplitKContiguousVec: job->fast_tiles = (unsigned)(Kp / 32), job->blocks = (unsigned)blocks64; break;
    default: job->fast_tiles = (unsigned)((Kp + 63) / 64), job->blocks = (unsigned)((Kp + 63) / 64 * (Rp / 64)); break;
  }
  return ECGEMM_OK;
}

template <int KIND, bool STATS>
void launch_split_job(hipStream_t stream, const SplitJob& job) {
  const dim3 grid(job.blocks), block(256);
  switch (job.variant) {
    case kSplitRContiguousWide: hipLaunchKernelGGL((split_kernel<KIND, kSplitRContiguousWide, STATS>), grid, block, 0, stream, job); break;
    case kSplitRContiguous: hipLaunchKernelGGL((split_kernel<KIND, kSplitRContiguous, STATS>), grid, block, 0, stream, job); break;
    case kSplitKContiguousVec: hipLaunchKernelGGL((split_kernel<KIND, kSplitKContiguousVec, STATS>), grid, block, 0, stream, job); break;
    default: hipLaunchKernelGGL((split_kernel<KIND, kSplitKContiguous, STATS>), grid, block, 0, stream, job); break;
  }
}

template <int KIND, bool STATS = false>
void launch_split_kind(hipStream_t stream, const SplitJob& a, const SplitJob* b) {
  if (b != nullptr && (uint64_t)a.blocks + b->blocks <= 8192) {  // small pairs go out as one launch
    hipLaunchKernelGGL((split_pair_kernel<KIND, STATS>), dim3(a.blocks + b->blocks), dim3(256), 0, stream, a, *b);
  } else {
    launch_split_job<KIND, STATS>(stream, a);
    if (b) launch_split_job<KIND, STATS>(stream, *b);
  }
}

// Step 1 for one operand, or (b != nullptr) for both operands of a product.  `measuring` (FP16 pair only): the kernels
// also leave the statistics of the automatic mode choice in a.stats and b->stats.
ecgemm_status_t launch_split(ecgemm_handle_t h, ecgemm_mode_t mode, const SplitJob& a, const SplitJob* b = nullptr,
                             bool measuring = false) {
  switch (split_kind_of((int)mode)) {
    case kSplitFp16Scaled:
      if (measuring) launch_split_kind<kSplitFp16Scaled, true>(h->stream, a, b);
      else launch_split_kind<kSplitFp16Scaled>(h->stream, a, b);
      break;
    case kSplitBf16x3: launch_split_kind<kSplitBf16x3>(h->stream, a, b); break;
    case kSplitFp16Unscaled: launch_split_kind<kSplitFp16Unscaled>(h->stream, a, b); break;
    case kSplitFp16Plain: launch_split_kind<kSplitFp16Plain>(h->stream, a, b); break;
    case kSplitFp32: launch_split_kind<kSplitFp32>(h->stream, a, b); break;
    default: launch_split_kind<kSplitBf16Plain>(h->stream, a, b); break;
  }
  ECGEMM_HIP(h, hipGetLastError());
  return ECGEMM_OK;
}

// Workgroups of the product kernel: one per item (every XCD's list padded to the same length), or one per workgroup
// slot when the shape runs this depth as a persistent grid and there are more items than slots.
int64_t product_grid(const Plan& pl, int compute_units, bool* persistent_out) {
  const int64_t tail_items = (int64_t)pl.tail_tiles * pl.tail_splits;
  const int64_t one_block_per_item = 8 * ((pl.full_tiles + 7) / 8 + (tail_items + 7) / 8);
  const int64_t slots = (int64_t)compute_units * pl.shape->blocks_per_cu;
  const bool persistent = pl.Kp <= pl.shape->persistent_max_k && one_block_per_item > slots;
  if (persistent_out) *persistent_out = persistent;
  return persistent ? slots : one_block_per_item;
}

// Column bands of the tile order (ProductParams::column_bands), which decide how the 8 XCDs lie over the tile grid:
// each XCD takes a contiguous run of the order, so with n bands the XCDs are laid out (8 / n) x n, each walking its
// own part of the grid along N.  Each XCD has its own L2, and what misses there is served by the memory-side cache
// that all XCDs share (256 MiB), else by HBM.  With xm = 8 / n rows of XCDs, xm panels of A (group_m tile rows x K
// each) are live at a time; they are re-used by every patch of the walk while B streams past once per xm panels.  So
// xm should be as large as lets the live panels of A stay in that cache: measured best when they take at most half of
// it (16384^3: 2 x 4 and 4 x 2 are 2.2 % ahead of 8 x 1; 8192^3: 4 x 2 by 2.2 %; 16384 x 16384 x 4096, where 8 panels
// are 128 MiB: 8 x 1 is 2 % ahead of 2 x 4).  A band is at least as wide as the patch of tiles an XCD works on at one
// time.
int column_bands(const Plan& pl, int group_m, ecgemm_mode_t mode, int forced = 0) {
  if (forced > 0) return std::max(1, std::min(forced, pl.tiles_n));
  const int patch_n = 32 * pl.shape->blocks_per_cu / group_m;
  const int64_t panel_bytes = (int64_t)group_m * pl.shape->bm * pl.Kp * 2 * parts_of(mode);
  const int groups = (pl.tiles_m + group_m - 1) / group_m;
  int best = 1;
  for (int n = 1; n <= 8; n *= 2) {
    if (n > 1 && pl.tiles_n / n < patch_n) break;
    best = n;
    const int live_panels = std::min(8 / n, groups);
    if (live_panels == 1 || live_panels * panel_bytes <= (128ll << 20)) break;
  }
  return best;
}

// Tile rows per group of the tile order.  The 32 compute units of an XCD work on consecutive tiles, and the nearer to
// square the patch of C these cover, the fewer distinct panel rows they request per k step: 4 x 8 tiles of 256 x 128.
// For the 128 x 128 shape (64 tiles at a time) 8 x 8 is ahead only on the shallow products the shape is chosen for
// (2.5 % at 16384 x 16384 x 256 and x 512; 4 x 16 is 4 % ahead at 8192^3).
int group_m_of(const Plan& pl, int forced = 0) {
  if (forced > 0) return forced;
  return (pl.shape->bm == 128 && pl.Kp <= 512) ? 8 : 4;
}

// Steps 2 and 3 on operands already in fragment order (padded as ecgemm_split pads them, or tighter).
ecgemm_status_t launch_product(ecgemm_handle_t h, const Plan& pl, int64_t M, int64_t N, float alpha, const void* a_packed,
                               const void* b_packed, float beta, float* C, int64_t ldc, ecgemm_mode_t mode, float* partials,
                               int log2_out_scale = 0, const int* row_log2_scale = nullptr, const int* col_log2_scale = nullptr,
                               const int* gate = nullptr, int gate_value = 0) {
  ProductParams pp;
  pp.gate = gate;
  pp.gate_value = gate_value;
  pp.a_packed = static_cast<const char*>(a_packed);
  pp.b_packed = static_cast<const char*>(b_packed);
  pp.row_block_bytes = (pl.Kp / 16) * parts_of(mode) * 1024;
  pp.k_tiles = pl.k_tiles;
  pp.full_tiles = pl.full_tiles;
  pp.tail_tiles = pl.tail_tiles;
  pp.tail_splits = pl.tail_splits;
  pp.kt_per_split = (pl.k_tiles + pl.tail_splits - 1) / pl.tail_splits;
  pp.by_tail_tiles = fast_divisor(pl.tail_tiles);
  const int group_m = group_m_of(pl, h->forced_group_m);
  const int bands = column_bands(pl, group_m, mode, h->forced_column_bands);
  pp.order = make_tile_order(pl.tiles_m, pl.tiles_n, group_m, bands);
  pp.xcd_remap = h->xcd_remap;
  pp.M = M;
  pp.N = N;
  pp.ldc = ldc;
  pp.alpha = alpha;
  pp.beta = beta;
  pp.out_scale = std::ldexp(1.0f, log2_out_scale);
  pp.row_log2_scale = row_log2_scale;
  pp.col_log2_scale = col_log2_scale;
  pp.C = C;
  pp.partials = partials;
  // Grid, always a multiple of the 8 XCDs: one block per item, or a persistent grid (see Shape::persistent_max_k).
  const dim3 grid((unsigned)product_grid(pl, h->compute_units, nullptr));
  void* args[] = {&pp};
  const void* kernel = reinterpret_cast<const void*>(row_log2_scale && pl.shape->product_scaled ? pl.shape->product_scaled : pl.shape->product);
  ECGEMM_HIP(h, hipLaunchKernel(kernel, grid, dim3(pl.shape->threads), args, 0, h->stream));
  if (pl.tail_splits > 1) {
    const dim3 rgrid((unsigned)pl.tail_tiles, (unsigned)(pl.shape->bm * pl.shape->bn / 1024));
    hipLaunchKernelGGL(pl.shape->reduce, rgrid, dim3(256), 0, h->stream, partials, pl.tail_splits, pl.tail_tiles,
                       pl.full_tiles, pl.tiles_m, pl.tiles_n, group_m, bands, M, N, alpha, beta, C, ldc, gate, gate_value, gate_value);
    ECGEMM_HIP(h, hipGetLastError());
  }
  return ECGEMM_OK;
}

// Steps 1 to 5 in one kernel, on the caller's FP32 operands (small products).
ecgemm_status_t launch_fused(ecgemm_handle_t h, const Plan& pl, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N,
                             int64_t K, float alpha, const float* A, int64_t lda, const float* B, int64_t ldb, float beta,
                             float* C, int64_t ldc, const int* row_log2_scale, const int* col_log2_scale, float* partials = nullptr,
                             const int* gate = nullptr, int gate_value = 0, int gate_value_scaled = 0) {
  if (pl.tail_splits > 1 && partials == nullptr)
    return fail(h, ECGEMM_ERR_UNSUPPORTED, "ecgemm_sgemm: a sliced one-launch plan without room for its partial sums");
  FusedParams fp;
  fp.k_slices = pl.tail_splits;
  fp.chunks_per_slice = (int)fused_chunks_per_slice(K, pl.tail_splits);
  fp.partials = partials;
  fp.gate = gate;  // (with a gate: gate_value runs without the scaling vectors, gate_value_scaled with them)
  fp.gate_value = gate_value;
  fp.gate_value_scaled = gate_value_scaled;
  fp.row_log2_scale = row_log2_scale;
  fp.col_log2_scale = col_log2_scale;
  fp.A = A;
  fp.B = B;
  fp.lda = lda;
  fp.ldb = ldb;
  // op(A)(m, k) = A[k + m lda] if transA == T; op(B)(k, n) = B[k + n ldb] if transB == N
  auto layout_of = [K](bool k_contiguous, const float* base, int64_t ld) {
    return !k_contiguous ? kFusedRows : (ld % 4 == 0 && (uintptr_t)base % 16 == 0 && K % 4 == 0) ? kFusedDepthVec : kFusedDepth;
  };
  const int layout_a = layout_of(transA == ECGEMM_OP_T, A, lda), layout_b = layout_of(transB == ECGEMM_OP_N, B, ldb);
  fp.prescale_a = std::ldexp(1.0f, h->log2_scale_a);
  fp.prescale_b = std::ldexp(1.0f, h->log2_scale_b);
  fp.M = M;
  fp.N = N;
  fp.K = K;
  fp.ldc = ldc;
  fp.tiles_m = pl.tiles_m;
  fp.tiles_n = pl.tiles_n;
  fp.alpha = alpha;
  fp.beta = beta;
  fp.out_scale = std::ldexp(1.0f, -(h->log2_scale_a + h->log2_scale_b));
  fp.C = C;
  const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
  void* args[] = {&fp};
  ECGEMM_HIP(h, hipLaunchKernel(reinterpret_cast<const void*>(pl.shape->fused->kernel[layout_a][layout_b]),
                                dim3((unsigned)(tiles * pl.tail_splits)), dim3((unsigned)pl.shape->threads), args, 0, h->stream));
  if (pl.tail_splits > 1) {  // the slices in ascending order, then alpha / beta (tiles in the order of the kernel above)
    const dim3 rgrid((unsigned)tiles, (unsigned)(pl.shape->bm * pl.shape->bn / 1024));
    hipLaunchKernelGGL(pl.shape->reduce, rgrid, dim3(256), 0, h->stream, partials, pl.tail_splits, (int)tiles, 0, pl.tiles_m,
                       pl.tiles_n, 4, 1, M, N, alpha, beta, C, ldc, gate, gate_value, gate_value_scaled);
    ECGEMM_HIP(h, hipGetLastError());
  }
  return ECGEMM_OK;
}

// Device memory for this call: the caller's workspace if one is set (never allocating), else the handle's own,
// grown on demand; or the library's built-in one (never allocating either).
enum WorkspaceKind { kWorkspaceOfHandle, kWorkspaceBuiltIn };
ecgemm_status_t acquire_workspace(ecgemm_handle_t h, size_t bytes, char** out, WorkspaceKind kind = kWorkspaceOfHandle) {
  *out = nullptr;
  if (bytes == 0) return ECGEMM_OK;
  if (kind == kWorkspaceBuiltIn) {
    if (bytes > ECGEMM_NOALLOC_WORKSPACE_BYTES)
      return fail(h, ECGEMM_ERR_ALLOC, "ecgemm_sgemm_noalloc: the problem needs " + std::to_string(bytes) +
                                           " bytes of workspace, the built-in one has " +
                                           std::to_string(ECGEMM_NOALLOC_WORKSPACE_BYTES));
    *out = h->builtin_workspace;
    return ECGEMM_OK;
  }
  if (h->user_workspace) {
    if (h->user_bytes < bytes) return fail(h, ECGEMM_ERR_ALLOC, "caller workspace too small");
    *out = static_cast<char*>(h->user_workspace);
    return ECGEMM_OK;
  }
  if (h->own_bytes < bytes) {
    // the old buffer may still be in use by earlier calls on the stream
    ECGEMM_HIP(h, hipStreamSynchronize(h->stream));
    if (h->own_workspace) ECGEMM_HIP(h, hipFree(h->own_workspace));
    h->own_workspace = nullptr;
    h->own_bytes = 0;
    if (hipMalloc(&h->own_workspace, bytes) != hipSuccess) {
      h->own_workspace = nullptr;
      (void)hipGetLastError();
      return fail(h, ECGEMM_ERR_ALLOC, "hipMalloc of the workspace failed");
    }
    h->own_bytes = bytes;
  }
  *out = static_cast<char*>(h->own_workspace);
  return ECGEMM_OK;
}

// `m_position`: where M stands in the calling function's parameter list (N and K follow it)
ecgemm_status_t check_sizes(ecgemm_handle_t h, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode, int m_position) {
  // tile indices are 32-bit and the byte offset along K inside a row block is a 32-bit vector offset
  if (M > (int64_t)1 << 36) return bad_arg(h, m_position, "M too large");
  if (N > (int64_t)1 << 36) return bad_arg(h, m_position + 1, "N too large");
  // work items are counted in 32 bits: at most 2^30 output tiles of 128 x 128 (C would hold 2^44 elements)
  if (((M + 127) / 128) * ((N + 127) / 128) > ((int64_t)1 << 30)) return bad_arg(h, m_position, "M x N too large");
  if (K > ((int64_t)1 << 26) || (round_up(K, kDepthPad) / 16) * parts_of(mode) * 1024 >= ((int64_t)1 << 32))
    return bad_arg(h, m_position + 2, "K too large: a packed row block must stay below 4 GiB");
  return ECGEMM_OK;
}

// ---- the workspace built into the library, for ecgemm_sgemm_noalloc.  In host code `scratch` is only a stand-in for
// the device array: its device address, one per GPU, comes from hipGetSymbolAddress with that GPU current, and that
// address is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[ECGEMM_NOALLOC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_address[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device.
hipError_t builtin_workspace_of(int device, char** out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_address[device] == nullptr) {
    void* address = nullptr;
    const hipError_t e = hipGetSymbolAddress(&address, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (address == nullptr) return hipErrorInvalidSymbol;
    g_scratch_address[device] = address;
  }
  *out = static_cast<char*>(g_scratch_address[device]);
  return hipSuccess;
}

// One operand's part of ecgemm_row_scales.  INVALID_ARG (positions as in ecgemm_row_scales) if the operand has more
// rows or more depth than the kernels' grids hold.
ecgemm_status_t make_row_scale_job(ecgemm_handle_t handle, ecgemm_op_t op, int64_t rows, int64_t depth, const float* src,
                                   int64_t ld, int target_exponent, int32_t* log2_scale, RowScaleJob* job) {
  const bool k_contiguous = op == ECGEMM_OP_T;
  const int slab = (!k_contiguous && depth <= 128 * 65535) ? 128 : 2048;  // k per workgroup (see the kernel)
  const int64_t grid_x = k_contiguous ? (rows + 3) / 4 : (rows + 255) / 256, slabs = (depth + slab - 1) / slab;
  if (rows > 0x1fffffffLL) return bad_arg(handle, 3, "ecgemm_row_scales: too many rows");
  if (slabs > 65535 || grid_x * slabs > 0x3fffffffLL) return bad_arg(handle, 4, "ecgemm_row_scales: operand too large");
  *job = RowScaleJob{src, ld, rows, depth, slab, (int)k_contiguous, target_exponent, (unsigned)grid_x,
                     (unsigned)(grid_x * slabs), log2_scale};
  return ECGEMM_OK;
}

// The kernels of ecgemm_row_scales for one job or two (b.rows == 0: one), optionally gated: step 1 (clear), step 2
// (largest exponents) and step 3 (exponents to scaling exponents), or a subset of them.
enum RowScaleSteps { kRowScaleClear = 1, kRowScaleMax = 2, kRowScaleFinish = 4, kRowScaleAll = 7 };
ecgemm_status_t launch_row_scales(ecgemm_handle_t handle, const RowScaleJob& a, const RowScaleJob& b, const int* gate,
                                  int gate_value, int steps = kRowScaleAll) {
  const unsigned per_row = (unsigned)((a.rows + b.rows + 255) / 256);
  if (steps & kRowScaleClear)
    hipLaunchKernelGGL(row_scales_clear_kernel, dim3(per_row), dim3(256), 0, handle->stream, a, b, gate, gate_value);
  if ((steps & kRowScaleMax) && a.blocks + b.blocks > 0)
    hipLaunchKernelGGL(row_max_exponent_kernel, dim3(a.blocks + b.blocks), dim3(256), 0, handle->stream, a, b, gate, gate_value);
  if (steps & kRowScaleFinish)
    hipLaunchKernelGGL(row_scales_finish_kernel, dim3(per_row), dim3(256), 0, handle->stream, a, b, gate, gate_value);
  ECGEMM_HIP(handle, hipGetLastError());
  return ECGEMM_OK;
}

hipEvent_t take_event(ecgemm_handle_t h) {
  if (!h->free_events.empty()) {
    hipEvent_t e = h->free_events.back();
    h->free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

extern "C" {

const char* ecgemm_status_string(ecgemm_status_t status) {
  switch (status) {
    case ECGEMM_OK: return "ECGEMM_OK";
    case ECGEMM_ERR_INVALID_ARG: return "ECGEMM_ERR_INVALID_ARG";
    case ECGEMM_ERR_ALLOC: return "ECGEMM_ERR_ALLOC";
    case ECGEMM_ERR_HIP: return "ECGEMM_ERR_HIP";
    case ECGEMM_ERR_UNSUPPORTED: return "ECGEMM_ERR_UNSUPPORTED";
  }
  return "ECGEMM_ERR_UNKNOWN";
}

const char* ecgemm_last_error_string(ecgemm_handle_t handle) {
  return handle ? handle->last_error.c_str() : "null handle";
}

int ecgemm_last_error_argument(ecgemm_handle_t handle) { return handle ? handle->last_error_argument : -1; }

ecgemm_status_t ecgemm_create(ecgemm_handle_t* handle) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  *handle = nullptr;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return ECGEMM_ERR_HIP;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return ECGEMM_ERR_HIP;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return ECGEMM_ERR_UNSUPPORTED;
  char* builtin = nullptr;
  if (builtin_workspace_of(device, &builtin) != hipSuccess) {
    (void)hipGetLastError();
    return ECGEMM_ERR_HIP;
  }
  ecgemm_context* ctx = new (std::nothrow) ecgemm_context();
  if (!ctx) return ECGEMM_ERR_ALLOC;
  ctx->device = device;
  ctx->compute_units = prop.multiProcessorCount > 8 ? prop.multiProcessorCount / 8 * 8 : 8;
  ctx->builtin_workspace = builtin;
  *handle = ctx;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_destroy(ecgemm_handle_t handle) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  ecgemm_status_t st = ECGEMM_OK;
  if (handle->own_workspace && hipFree(handle->own_workspace) != hipSuccess) st = ECGEMM_ERR_HIP;
  if (handle->range_buffer && hipFree(handle->range_buffer) != hipSuccess) st = ECGEMM_ERR_HIP;
  for (TimedCall& t : handle->timed) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.split_done);
    (void)hipEventDestroy(t.product_done);
  }
  for (hipEvent_t e : handle->free_events) (void)hipEventDestroy(e);
  delete handle;
  return st;
}

ecgemm_status_t ecgemm_set_stream(ecgemm_handle_t handle, void* hip_stream) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  handle->stream = static_cast<hipStream_t>(hip_stream);
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_set_shape(ecgemm_handle_t handle, ecgemm_shape_t shape) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_shape(shape)) return bad_arg(handle, 2, "ecgemm_set_shape: unknown shape");
  handle->shape = shape;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_debug_set_tile_order(ecgemm_handle_t handle, int xcd_remap, int group_m, int column_bands) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (xcd_remap != 0 && xcd_remap != 1) return bad_arg(handle, 2, "ecgemm_debug_set_tile_order: xcd_remap is 0 or 1");
  if (group_m < 0 || group_m > (1 << 20)) return bad_arg(handle, 3, "ecgemm_debug_set_tile_order: bad group_m");
  if (column_bands < 0 || column_bands > 8) return bad_arg(handle, 4, "ecgemm_debug_set_tile_order: 0 to 8 column bands");
  handle->xcd_remap = xcd_remap;
  handle->forced_group_m = group_m;
  handle->forced_column_bands = column_bands;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_debug_tile_order(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode,
                                        int32_t* tile_m, int32_t* tile_n, int64_t* disagreements) {
  if (M <= 0) return bad_arg(handle, 2, "ecgemm_debug_tile_order: M must be positive");
  if (N <= 0) return bad_arg(handle, 3, "ecgemm_debug_tile_order: N must be positive");
  if (K <= 0) return bad_arg(handle, 4, "ecgemm_debug_tile_order: K must be positive");
  if (!valid_mode(mode)) return bad_arg(handle, 5, "ecgemm_debug_tile_order: unknown mode");
  if (!tile_m) return bad_arg(handle, 6, "ecgemm_debug_tile_order: null output");
  if (!tile_n) return bad_arg(handle, 7, "ecgemm_debug_tile_order: null output");
  if (!disagreements) return bad_arg(handle, 8, "ecgemm_debug_tile_order: null output");
  const ecgemm_status_t st = check_sizes(handle, M, N, K, mode, 2);
  if (st != ECGEMM_OK) return st;
  const Plan pl = make_plan(M, N, K, mode, handle ? handle->shape : ECGEMM_SHAPE_AUTO, kOneLaunchSliced);  // as ecgemm_plan_info
  if (!pl.shape || pl.shape->fused) return fail(handle, ECGEMM_ERR_UNSUPPORTED, "ecgemm_debug_tile_order: no product kernel of this shape and mode");
  const int group_m = group_m_of(pl, handle ? handle->forced_group_m : 0);
  const int bands = column_bands(pl, group_m, mode, handle ? handle->forced_column_bands : 0);
  const TileOrder order = make_tile_order(pl.tiles_m, pl.tiles_n, group_m, bands);
  *disagreements = 0;
  for (int pid = 0; pid < pl.tiles_m * pl.tiles_n; ++pid) {
    int m = -1, n = -1, m_plain = -1, n_plain = -1;
    tile_coordinates(pid, order, m, n);
    tile_coordinates(pid, pl.tiles_m, pl.tiles_n, group_m, bands, m_plain, n_plain);
    if (m != m_plain || n != n_plain) *disagreements += 1;
    tile_m[pid] = m, tile_n[pid] = n;
  }
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_workspace_size(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N,
                                      int64_t K, ecgemm_mode_t mode, size_t* bytes) {
  if (!valid_op(transA)) return bad_arg(handle, 2, "ecgemm_workspace_size: bad transA");
  if (!valid_op(transB)) return bad_arg(handle, 3, "ecgemm_workspace_size: bad transB");
  if (M < 0) return bad_arg(handle, 4, "ecgemm_workspace_size: negative M");
  if (N < 0) return bad_arg(handle, 5, "ecgemm_workspace_size: negative N");
  if (K < 0) return bad_arg(handle, 6, "ecgemm_workspace_size: negative K");
  if (!valid_mode_or_auto(mode)) return bad_arg(handle, 7, "ecgemm_workspace_size: unknown mode");
  if (!bytes) return bad_arg(handle, 8, "ecgemm_workspace_size: null output");
  *bytes = 0;
  if (M == 0 || N == 0 || K == 0) return ECGEMM_OK;
  const ecgemm_status_t st = check_sizes(handle, M, N, K, mode == ECGEMM_MODE_AUTO ? ECGEMM_MODE_BF16_FULL : mode, 4);
  if (st != ECGEMM_OK) return st;
  if (mode == ECGEMM_MODE_AUTO) {
    const AutoPlan ap = make_auto_plan(M, N, K, handle ? handle->shape : ECGEMM_SHAPE_AUTO);
    if (!ap.exists) return fail(handle, ECGEMM_ERR_UNSUPPORTED, "ecgemm_workspace_size: ECGEMM_MODE_AUTO does not run with the fused kernel shape");
    *bytes = ap.total_bytes;
    return ECGEMM_OK;
  }
  const ecgemm_shape_t shape = handle ? handle->shape : ECGEMM_SHAPE_AUTO;
  const Plan pl = make_plan(M, N, K, mode, shape, kOneLaunchSliced);
  if (!pl.shape) return no_plan(handle, pl, "ecgemm_workspace_size");
  *bytes = pl.total_bytes;
  // (ecgemm_product on the same problem never takes a one-launch shape by itself and may need room for partial sums)
  if (pl.shape->fused && shape == ECGEMM_SHAPE_AUTO) *bytes = std::max(*bytes, make_plan(M, N, K, mode, shape, kOneLaunchNever).partial_bytes);
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_plan_info(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode,
                                 ecgemm_plan_info_t* info) {
  if (M <= 0) return bad_arg(handle, 2, "ecgemm_plan_info: M must be positive");
  if (N <= 0) return bad_arg(handle, 3, "ecgemm_plan_info: N must be positive");
  if (K <= 0) return bad_arg(handle, 4, "ecgemm_plan_info: K must be positive");
  if (!valid_mode(mode)) return bad_arg(handle, 5, "ecgemm_plan_info: unknown mode");
  if (!info) return bad_arg(handle, 6, "ecgemm_plan_info: null output");
  const ecgemm_status_t st = check_sizes(handle, M, N, K, mode, 2);
  if (st != ECGEMM_OK) return st;
  const Plan pl = make_plan(M, N, K, mode, handle ? handle->shape : ECGEMM_SHAPE_AUTO, kOneLaunchSliced);
  if (!pl.shape) return no_plan(handle, pl, "ecgemm_plan_info");
  info->shape = (int)(pl.shape - &kShapes[(int)mode][0]) + 1;
  info->tile_m = pl.shape->bm;
  info->tile_n = pl.shape->bn;
  info->tiles_m = pl.tiles_m;
  info->tiles_n = pl.tiles_n;
  info->whole_tiles = pl.full_tiles;
  info->sliced_tiles = pl.tail_tiles;
  info->slices = pl.tail_splits;
  bool persistent = false;
  info->grid = pl.shape->fused ? (int64_t)pl.tiles_m * pl.tiles_n * pl.tail_splits : product_grid(pl, kPlanComputeUnits, &persistent);
  info->persistent = persistent ? 1 : 0;
  info->group_m = pl.shape->fused ? 4 : group_m_of(pl, handle ? handle->forced_group_m : 0);
  info->column_bands = pl.shape->fused ? 1 : column_bands(pl, info->group_m, mode, handle ? handle->forced_column_bands : 0);
  info->workspace_bytes = pl.total_bytes;
  info->estimated_us = pl.shape->fused ? one_launch_us(pl, K, mode) : estimated_us(pl, mode);
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_set_workspace(ecgemm_handle_t handle, void* device_buffer, size_t bytes) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (((uintptr_t)device_buffer % 256) != 0) return bad_arg(handle, 2, "ecgemm_set_workspace: buffer must be 256-byte aligned");
  if ((device_buffer == nullptr) != (bytes == 0)) return bad_arg(handle, 3, "ecgemm_set_workspace: a buffer with its size, or (NULL, 0)");
  handle->user_workspace = device_buffer;
  handle->user_bytes = bytes;
  handle->auto_choice = nullptr;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_split_size(int64_t rows, int64_t depth, ecgemm_mode_t mode, size_t* bytes) {
  if (!bytes || rows < 0 || depth < 0 || !valid_mode(mode)) return ECGEMM_ERR_INVALID_ARG;
  *bytes = packed_bytes(rows, depth, mode);
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_split(ecgemm_handle_t handle, ecgemm_op_t op, int64_t rows, int64_t depth,
                             const float* src, int64_t ld, ecgemm_mode_t mode, void* packed) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_op(op)) return bad_arg(handle, 2, "ecgemm_split: bad op");
  if (rows < 0) return bad_arg(handle, 3, "ecgemm_split: negative rows");
  if (depth < 0) return bad_arg(handle, 4, "ecgemm_split: negative depth");
  if (!valid_mode(mode)) return bad_arg(handle, 7, "ecgemm_split: unknown mode");
  if (rows == 0 || depth == 0) return ECGEMM_OK;
  if (!src) return bad_arg(handle, 5, "ecgemm_split: null source");
  if (ld < (op == ECGEMM_OP_N ? rows : depth)) return bad_arg(handle, 6, "ecgemm_split: leading dimension too small");
  if (!packed || ((uintptr_t)packed % 16) != 0) return bad_arg(handle, 8, "ecgemm_split: null or misaligned output");
  SplitJob job;
  const ecgemm_status_t st = make_split_job(handle, op, rows, depth, src, ld, packed, 0, nullptr, &job);
  if (st != ECGEMM_OK) return st;
  return launch_split(handle, mode, job);
}

ecgemm_status_t ecgemm_set_scaling(ecgemm_handle_t handle, int log2_scale_a, int log2_scale_b) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (std::abs(log2_scale_a) > 126) return bad_arg(handle, 2, "ecgemm_set_scaling: exponent beyond +-126");
  if (std::abs(log2_scale_b) > 126 || std::abs(log2_scale_a + log2_scale_b) > 126)
    return bad_arg(handle, 3, "ecgemm_set_scaling: exponents (and their sum) must stay within +-126");
  handle->log2_scale_a = log2_scale_a;
  handle->log2_scale_b = log2_scale_b;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_exponent_range(ecgemm_handle_t handle, int64_t rows, int64_t cols, const float* src, int64_t ld,
                                      int* min_exponent, int* max_exponent) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (rows < 0) return bad_arg(handle, 2, "ecgemm_exponent_range: negative rows");
  if (cols < 0) return bad_arg(handle, 3, "ecgemm_exponent_range: negative cols");
  if (!min_exponent) return bad_arg(handle, 6, "ecgemm_exponent_range: null output");
  if (!max_exponent) return bad_arg(handle, 7, "ecgemm_exponent_range: null output");
  int host[2] = {INT_MAX, INT_MIN};
  if (rows > 0 && cols > 0) {
    if (!src) return bad_arg(handle, 4, "ecgemm_exponent_range: null source");
    if (ld < rows) return bad_arg(handle, 5, "ecgemm_exponent_range: ld < rows");
    if (!handle->range_buffer && hipMalloc(&handle->range_buffer, 2 * sizeof(int)) != hipSuccess) {
      handle->range_buffer = nullptr;
      (void)hipGetLastError();
      return fail(handle, ECGEMM_ERR_ALLOC, "ecgemm_exponent_range: hipMalloc failed");
    }
    ECGEMM_HIP(handle, hipMemcpyAsync(handle->range_buffer, host, sizeof(host), hipMemcpyHostToDevice, handle->stream));
    const int64_t row_blocks = (rows + 255) / 256;
    const dim3 grid((unsigned)(row_blocks < 1024 ? row_blocks : 1024), (unsigned)(cols < 4096 ? cols : 4096));
    hipLaunchKernelGGL(exponent_range_kernel, grid, dim3(256), 0, handle->stream, src, ld, rows, cols, handle->range_buffer);
    ECGEMM_HIP(handle, hipGetLastError());
    ECGEMM_HIP(handle, hipMemcpyAsync(host, handle->range_buffer, sizeof(host), hipMemcpyDeviceToHost, handle->stream));
    ECGEMM_HIP(handle, hipStreamSynchronize(handle->stream));
  }
  *min_exponent = host[0];
  *max_exponent = host[1];
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_row_scales(ecgemm_handle_t handle, ecgemm_op_t op, int64_t rows, int64_t depth, const float* src,
                                  int64_t ld, int target_exponent, int32_t* log2_scale) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_op(op)) return bad_arg(handle, 2, "ecgemm_row_scales: bad op");
  if (rows < 0) return bad_arg(handle, 3, "ecgemm_row_scales: negative rows");
  if (depth < 0) return bad_arg(handle, 4, "ecgemm_row_scales: negative depth");
  if (target_exponent < -126 || target_exponent > 126) return bad_arg(handle, 7, "ecgemm_row_scales: target exponent beyond +-126");
  if (rows == 0) return ECGEMM_OK;
  if (!log2_scale) return bad_arg(handle, 8, "ecgemm_row_scales: null output");
  if (depth > 0 && !src) return bad_arg(handle, 5, "ecgemm_row_scales: null source");
  if (depth > 0 && ld < (op == ECGEMM_OP_N ? rows : depth)) return bad_arg(handle, 6, "ecgemm_row_scales: leading dimension too small");
  RowScaleJob job;
  const ecgemm_status_t st = make_row_scale_job(handle, op, rows, depth, src, ld, target_exponent, log2_scale, &job);
  if (st != ECGEMM_OK) return st;
  return launch_row_scales(handle, job, RowScaleJob{}, nullptr, 0);
}

ecgemm_status_t ecgemm_choose_mode(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N,
                                   int64_t K, const float* A, int64_t lda, const float* B, int64_t ldb,
                                   ecgemm_mode_t* mode, int* log2_scale_a, int* log2_scale_b) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_op(transA)) return bad_arg(handle, 2, "ecgemm_choose_mode: bad transA");
  if (!valid_op(transB)) return bad_arg(handle, 3, "ecgemm_choose_mode: bad transB");
  if (M < 0) return bad_arg(handle, 4, "ecgemm_choose_mode: negative M");
  if (N < 0) return bad_arg(handle, 5, "ecgemm_choose_mode: negative N");
  if (K < 0) return bad_arg(handle, 6, "ecgemm_choose_mode: negative K");
  if (!mode) return bad_arg(handle, 11, "ecgemm_choose_mode: null output");
  if (!log2_scale_a) return bad_arg(handle, 12, "ecgemm_choose_mode: null output");
  if (!log2_scale_b) return bad_arg(handle, 13, "ecgemm_choose_mode: null output");
  int lo[2] = {0, 0}, hi[2] = {0, 0};
  ecgemm_status_t st = ecgemm_exponent_range(handle, transA == ECGEMM_OP_N ? M : K, transA == ECGEMM_OP_N ? K : M, A, lda,
                                             &lo[0], &hi[0]);
  if (st != ECGEMM_OK) {
    if (handle->last_error_argument) handle->last_error_argument += 3;  // src, ld of that call are A, lda (7, 8) here
    return st;
  }
  st = ecgemm_exponent_range(handle, transB == ECGEMM_OP_N ? K : N, transB == ECGEMM_OP_N ? N : K, B, ldb, &lo[1], &hi[1]);
  if (st != ECGEMM_OK) {
    if (handle->last_error_argument) handle->last_error_argument += 5;  // B, ldb (9, 10)
    return st;
  }
  // The FP16 pair is fully precise for magnitudes 2^-14 .. 2^15 (top binade kept one below the saturation point):
  // an operand fits if its non-zero elements span at most 29 binades; its top binade is then moved to 2^14.
  int scale[2] = {0, 0};
  bool fits = true;
  for (int i = 0; i < 2; ++i) {
    if (lo[i] > hi[i]) continue;  // no non-zero finite element
    if (hi[i] - lo[i] > 28) fits = false;
    scale[i] = 14 - hi[i];
  }
  if (fits && (std::abs(scale[0]) > 126 || std::abs(scale[1]) > 126 || std::abs(scale[0] + scale[1]) > 126)) fits = false;
  *mode = fits ? ECGEMM_MODE_FP16_SPLIT : ECGEMM_MODE_BF16_FULL;
  *log2_scale_a = fits ? scale[0] : 0;
  *log2_scale_b = fits ? scale[1] : 0;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_debug_mfma(ecgemm_handle_t handle, int bf16, int64_t count, const void* a, const void* b,
                                  const float* c, float* d) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (count < 0 || count > 0x7fffffff) return bad_arg(handle, 3, "ecgemm_debug_mfma: bad count");
  if (count == 0) return ECGEMM_OK;
  if (!a || ((uintptr_t)a % 16)) return bad_arg(handle, 4, "ecgemm_debug_mfma: null or misaligned pointer");
  if (!b || ((uintptr_t)b % 16)) return bad_arg(handle, 5, "ecgemm_debug_mfma: null or misaligned pointer");
  if (!c || ((uintptr_t)c % 64)) return bad_arg(handle, 6, "ecgemm_debug_mfma: null or misaligned pointer");
  if (!d || ((uintptr_t)d % 64)) return bad_arg(handle, 7, "ecgemm_debug_mfma: null or misaligned pointer");
  const unsigned short* ua = static_cast<const unsigned short*>(a);
  const unsigned short* ub = static_cast<const unsigned short*>(b);
  if (bf16) hipLaunchKernelGGL(single_mfma_kernel<true>, dim3((unsigned)count), dim3(64), 0, handle->stream, ua, ub, c, d);
  else hipLaunchKernelGGL(single_mfma_kernel<false>, dim3((unsigned)count), dim3(64), 0, handle->stream, ua, ub, c, d);
  ECGEMM_HIP(handle, hipGetLastError());
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_debug_mfma_rate(ecgemm_handle_t handle, int bf16, const void* operands, float* sink, int blocks,
                                       int iters, double* flops) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!operands || ((uintptr_t)operands % 16)) return bad_arg(handle, 3, "ecgemm_debug_mfma_rate: null or misaligned operands");
  if (!sink) return bad_arg(handle, 4, "ecgemm_debug_mfma_rate: null sink");
  if (blocks <= 0) return bad_arg(handle, 5, "ecgemm_debug_mfma_rate: blocks must be positive");
  if (iters <= 0) return bad_arg(handle, 6, "ecgemm_debug_mfma_rate: iters must be positive");
  if (!flops) return bad_arg(handle, 7, "ecgemm_debug_mfma_rate: null output");
  const unsigned short* ops = static_cast<const unsigned short*>(operands);
  if (bf16) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, handle->stream, ops, sink, iters);
  else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, handle->stream, ops, sink, iters);
  ECGEMM_HIP(handle, hipGetLastError());
  *flops = (double)blocks * 4.0 * iters * 24.0 * 2.0 * 32 * 32 * 16;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_set_timing(ecgemm_handle_t handle, int enabled) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  handle->timing = enabled != 0;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_get_timing(ecgemm_handle_t handle, int* calls, float* split_ms, float* product_ms) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!calls) return bad_arg(handle, 2, "ecgemm_get_timing: null output");
  if (!split_ms) return bad_arg(handle, 3, "ecgemm_get_timing: null output");
  if (!product_ms) return bad_arg(handle, 4, "ecgemm_get_timing: null output");
  *calls = 0;
  *split_ms = 0.0f;
  *product_ms = 0.0f;
  for (TimedCall& t : handle->timed) {
    ECGEMM_HIP(handle, hipEventSynchronize(t.product_done));
    float a = 0.0f, b = 0.0f;
    ECGEMM_HIP(handle, hipEventElapsedTime(&a, t.start, t.split_done));
    ECGEMM_HIP(handle, hipEventElapsedTime(&b, t.split_done, t.product_done));
    *split_ms += a;
    *product_ms += b;
    *calls += 1;
    handle->free_events.push_back(t.start);
    handle->free_events.push_back(t.split_done);
    handle->free_events.push_back(t.product_done);
  }
  handle->timed.clear();
  return ECGEMM_OK;
}

}  // extern "C"

namespace {

// Events for the optional timing go back to the handle's pool whenever the call does not complete.
struct EventLease {
  ecgemm_handle_t h;
  TimedCall tc{};
  bool keep = false;
  ~EventLease() {
    if (keep) return;
    for (hipEvent_t e : {tc.start, tc.split_done, tc.product_done})
      if (e) h->free_events.push_back(e);
  }
};

// ECGEMM_MODE_AUTO (arguments already checked).  Nothing here waits for the GPU: the kernels of every candidate are
// enqueued, each gated on the word `choice` in device memory, so the ones that are not wanted return at once.
//   1. the FP16 pair split of A and of B, which also leave per block the squared Frobenius norm of the operand and of
//      what the pair fails to represent of it, and per row the largest binary exponent (for step 3)
//   2. first choice: kChoiceFp16 if both operands are represented to within kAutoTolerance, relative; else undecided
//   3. if undecided: the per-row / per-column scaling exponents of both operands from step 1's exponents (largest
//      binade of every row of op(A) and column of op(B) to 2^14), the FP16 pair split of the scaled operands with the
//      same statistics, and the second choice: kChoiceFp16Scaled if that fits, else kChoiceBf16
//   4. the BF16 three-term split of both operands (if kChoiceBf16), over the FP16 parts, which are no longer needed then
//   5. the FP16 product, the FP16 product that undoes the scaling vectors, the BF16 product: one of them runs
enum AutoChoice { kChoiceFp16 = 0, kChoiceBf16 = 1, kChoiceFp16Scaled = 2, kChoiceUndecided = 3 };
constexpr int kAutoScaleTarget = 14;  // where the scaled candidate puts the largest binade of every row and column

ecgemm_status_t sgemm_auto(ecgemm_handle_t h, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N, int64_t K, float alpha,
                           const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc,
                           WorkspaceKind workspace_kind) {
  ecgemm_status_t st = check_sizes(h, M, N, K, ECGEMM_MODE_BF16_FULL, 4);
  if (st != ECGEMM_OK) return st;
  const AutoPlan ap = make_auto_plan(M, N, K, h->shape);
  if (!ap.exists) return fail(h, ECGEMM_ERR_UNSUPPORTED, "ecgemm_sgemm: ECGEMM_MODE_AUTO does not run with the fused kernel shape");
  if (ap.fp16.items() + 16 > 0x7fffffffLL || ap.bf16.items() + 16 > 0x7fffffffLL) return bad_arg(h, 4, "ecgemm_sgemm: too many tiles");
  // (the scaled candidate is left out for operands beyond what the kernels that find the exponents take: 2^29 rows)
  RowScaleJob rows_a{}, rows_b{};
  const ecgemm_op_t op_b = transB == ECGEMM_OP_N ? ECGEMM_OP_T : ECGEMM_OP_N;  // as in sgemm_common
  const bool try_scaled =
      make_row_scale_job(h, transA, M, K, A, lda, kAutoScaleTarget - h->log2_scale_a, nullptr, &rows_a) == ECGEMM_OK &&
      make_row_scale_job(h, op_b, N, K, B, ldb, kAutoScaleTarget - h->log2_scale_b, nullptr, &rows_b) == ECGEMM_OK &&
      (uint64_t)rows_a.blocks + rows_b.blocks <= 0x7fffffffu;
  char* ws = nullptr;
  st = acquire_workspace(h, ap.total_bytes, &ws, workspace_kind);
  if (st != ECGEMM_OK) return st;
  float* partials = ap.partial_bytes ? reinterpret_cast<float*>(ws + ap.packed_bytes) : nullptr;
  char* at = ws + ap.packed_bytes + ap.partial_bytes;
  double* stats_a = reinterpret_cast<double*>(at);
  double* stats_b = reinterpret_cast<double*>(at += ap.stats_a_bytes);
  int32_t* scales_a = reinterpret_cast<int32_t*>(at += ap.stats_b_bytes);
  int32_t* scales_b = reinterpret_cast<int32_t*>(at += ap.scales_a_bytes);
  int* choice = reinterpret_cast<int*>(at += ap.scales_b_bytes);
  rows_a.scale = scales_a;
  rows_b.scale = scales_b;
  SplitJob fp16_a, fp16_b, scaled_a, scaled_b, bf16_a, bf16_b;
  st = make_split_job(h, transA, M, K, A, lda, ws, h->log2_scale_a, nullptr, &fp16_a);
  if (st != ECGEMM_OK) return st;
  st = make_split_job(h, op_b, N, K, B, ldb, ws + ap.fp16.a_bytes, h->log2_scale_b, nullptr, &fp16_b);
  if (st != ECGEMM_OK) return st;
  st = make_split_job(h, transA, M, K, A, lda, ws, h->log2_scale_a, nullptr, &bf16_a);
  if (st != ECGEMM_OK) return st;
  st = make_split_job(h, op_b, N, K, B, ldb, ws + ap.bf16.a_bytes, h->log2_scale_b, nullptr, &bf16_b);
  if (st != ECGEMM_OK) return st;
  if (kStatsPerBlock * sizeof(double) * fp16_a.blocks > ap.stats_a_bytes ||
      kStatsPerBlock * sizeof(double) * fp16_b.blocks > ap.stats_b_bytes)
    return fail(h, ECGEMM_ERR_HIP, "ecgemm_sgemm: internal error, statistics array too small");
  fp16_a.stats = stats_a;
  fp16_b.stats = stats_b;
  scaled_a = fp16_a;
  scaled_b = fp16_b;
  scaled_a.row_log2_scale = scales_a;
  scaled_b.row_log2_scale = scales_b;
  scaled_a.gate = scaled_b.gate = choice;
  scaled_a.gate_value = scaled_b.gate_value = kChoiceUndecided;
  bf16_a.gate = bf16_b.gate = choice;
  bf16_a.gate_value = bf16_b.gate_value = kChoiceBf16;

  EventLease lease{h};
  TimedCall& tc = lease.tc;
  const bool timing = h->timing && workspace_kind != kWorkspaceBuiltIn;
  if (timing) {
    tc.start = take_event(h);
    tc.split_done = take_event(h);
    tc.product_done = take_event(h);
    if (!tc.start || !tc.split_done || !tc.product_done) return fail(h, ECGEMM_ERR_HIP, "ecgemm_sgemm: hipEventCreate failed");
    ECGEMM_HIP(h, hipEventRecord(tc.start, h->stream));
  }
  if (try_scaled) {
    // the first split also finds every row's largest exponent (on the operands as the caller passed them), so that
    // the scaled candidate needs no pass over A and B of its own for them
    st = launch_row_scales(h, rows_a, rows_b, nullptr, 0, kRowScaleClear);
    if (st != ECGEMM_OK) return st;
    fp16_a.row_max = scales_a;
    fp16_b.row_max = scales_b;
  }
  st = launch_split(h, ECGEMM_MODE_FP16_SPLIT, fp16_a, &fp16_b, true);
  if (st != ECGEMM_OK) return st;
  // (operands with few rows: the first choice also turns the rows' exponents into factors, which saves a launch)
  const bool finish_with_choice = try_scaled && M + N <= 4096;
  const RowScaleJob no_rows{};
  hipLaunchKernelGGL(choose_mode_kernel, dim3(1), dim3(1024), 0, h->stream, stats_a, fp16_a.blocks, (double)M, stats_b,
                     fp16_b.blocks, (double)N, kAutoTolerance, kAutoMinTerms, choice, (int)kChoiceFp16,
                     (int)(try_scaled ? kChoiceUndecided : kChoiceBf16), (const int*)nullptr, 0,
                     finish_with_choice ? rows_a : no_rows, finish_with_choice ? rows_b : no_rows);
  ECGEMM_HIP(h, hipGetLastError());
  h->auto_choice = choice;
  if (try_scaled) {
    // the exponents are found on the operands as the caller passed them; the handle's global pre-scaling, a common
    // factor of every row, comes on top in the split and is undone with the product's output scale
    if (!finish_with_choice) {
      st = launch_row_scales(h, rows_a, rows_b, choice, kChoiceUndecided, kRowScaleFinish);
      if (st != ECGEMM_OK) return st;
    }
    st = launch_split(h, ECGEMM_MODE_FP16_SPLIT, scaled_a, &scaled_b, true);
    if (st != ECGEMM_OK) return st;
    hipLaunchKernelGGL(choose_mode_kernel, dim3(1), dim3(1024), 0, h->stream, stats_a, scaled_a.blocks, (double)M, stats_b,
                       scaled_b.blocks, (double)N, kAutoTolerance, kAutoMinTerms, choice, (int)kChoiceFp16Scaled,
                       (int)kChoiceBf16, (const int*)choice, (int)kChoiceUndecided, no_rows, no_rows);
    ECGEMM_HIP(h, hipGetLastError());
  }
  // Every candidate runs the way ecgemm_sgemm would run it in that mode, so that the result is that call's bit for
  // bit: a small product as one launch on the FP32 operands (the measuring splits above still write their packed
  // parts, which nothing reads then), the others with the product kernels on the packed operands.
  const Plan one_fp16 = make_plan(M, N, K, ECGEMM_MODE_FP16_SPLIT, h->shape, kOneLaunchSliced);
  const Plan one_bf16 = make_plan(M, N, K, ECGEMM_MODE_BF16_FULL, h->shape, kOneLaunchSliced);
  const bool fp16_one_launch = one_fp16.shape && one_fp16.shape->fused, bf16_one_launch = one_bf16.shape && one_bf16.shape->fused;
  if (!bf16_one_launch) {
    st = launch_split(h, ECGEMM_MODE_BF16_FULL, bf16_a, &bf16_b);
    if (st != ECGEMM_OK) return st;
  }
  if (timing) ECGEMM_HIP(h, hipEventRecord(tc.split_done, h->stream));
  const int log2_out_scale = -(h->log2_scale_a + h->log2_scale_b);
  if (fp16_one_launch) {  // with and without the scaling vectors in one launch, which looks at the choice itself
    st = launch_fused(h, one_fp16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, try_scaled ? scales_a : nullptr,
                      try_scaled ? scales_b : nullptr, partials, choice, kChoiceFp16, try_scaled ? kChoiceFp16Scaled : kChoiceFp16);
    if (st != ECGEMM_OK) return st;
  } else {
    for (int scaled = 0; scaled <= (try_scaled ? 1 : 0); ++scaled) {
      st = launch_product(h, ap.fp16, M, N, alpha, ws, ws + ap.fp16.a_bytes, beta, C, ldc, ECGEMM_MODE_FP16_SPLIT, partials,
                          log2_out_scale, scaled ? scales_a : nullptr, scaled ? scales_b : nullptr, choice,
                          scaled ? kChoiceFp16Scaled : kChoiceFp16);
      if (st != ECGEMM_OK) return st;
    }
  }
  st = bf16_one_launch ? launch_fused(h, one_bf16, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, nullptr, nullptr, partials,
                                      choice, kChoiceBf16, kChoiceBf16)
                       : launch_product(h, ap.bf16, M, N, alpha, ws, ws + ap.bf16.a_bytes, beta, C, ldc, ECGEMM_MODE_BF16_FULL, partials,
                                        log2_out_scale, nullptr, nullptr, choice, kChoiceBf16);
  if (st != ECGEMM_OK) return st;
  if (timing) {
    ECGEMM_HIP(h, hipEventRecord(tc.product_done, h->stream));
    h->timed.push_back(tc);
    lease.keep = true;
  }
  return ECGEMM_OK;
}

// ecgemm_sgemm, ecgemm_sgemm_scaled and ecgemm_sgemm_noalloc: the same parameter list up to `mode` (the positions
// reported for bad arguments count it), then the scaling vectors and where the workspace comes from.  Everything that
// can be refused is checked before the first launch.
ecgemm_status_t sgemm_common(ecgemm_handle_t h, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N, int64_t K, float alpha,
                             const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc,
                             ecgemm_mode_t mode, const int32_t* row_log2_scale_a, const int32_t* col_log2_scale_b,
                             WorkspaceKind workspace_kind) {
  if (!h) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_op(transA)) return bad_arg(h, 2, "ecgemm_sgemm: bad transA");
  if (!valid_op(transB)) return bad_arg(h, 3, "ecgemm_sgemm: bad transB");
  if (M < 0) return bad_arg(h, 4, "ecgemm_sgemm: negative M");
  if (N < 0) return bad_arg(h, 5, "ecgemm_sgemm: negative N");
  if (K < 0) return bad_arg(h, 6, "ecgemm_sgemm: negative K");
  if (!valid_mode_or_auto(mode)) return bad_arg(h, 15, "ecgemm_sgemm: unknown mode");
  h->auto_choice = nullptr;
  if (M == 0 || N == 0) return ECGEMM_OK;
  if (!C) return bad_arg(h, 13, "ecgemm_sgemm: C is null");
  if (ldc < M) return bad_arg(h, 14, "ecgemm_sgemm: ldc < M");

  const dim3 block256(256);
  if (K == 0 || alpha == 0.0f) {
    const dim3 grid((unsigned)((M + 255) / 256), (unsigned)(N < 65535 ? N : 65535));
    hipLaunchKernelGGL(scale_c_kernel, grid, block256, 0, h->stream, M, N, beta, C, ldc);
    ECGEMM_HIP(h, hipGetLastError());
    return ECGEMM_OK;
  }
  if (!A) return bad_arg(h, 8, "ecgemm_sgemm: A is null");
  if (lda < (transA == ECGEMM_OP_N ? M : K)) return bad_arg(h, 9, "ecgemm_sgemm: lda too small");
  if (!B) return bad_arg(h, 10, "ecgemm_sgemm: B is null");
  if (ldb < (transB == ECGEMM_OP_N ? K : N)) return bad_arg(h, 11, "ecgemm_sgemm: ldb too small");

  if ((row_log2_scale_a == nullptr) != (col_log2_scale_b == nullptr))
    return bad_arg(h, row_log2_scale_a == nullptr ? 16 : 17, "ecgemm_sgemm_scaled: give both scaling vectors or neither");
  if (mode == ECGEMM_MODE_AUTO) {
    if (row_log2_scale_a) return fail(h, ECGEMM_ERR_UNSUPPORTED, "ecgemm_sgemm_scaled: ECGEMM_MODE_AUTO takes no scaling vectors");
    return sgemm_auto(h, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace_kind);
  }
  ecgemm_status_t st = check_sizes(h, M, N, K, mode, 4);
  if (st != ECGEMM_OK) return st;
  const Plan pl = make_plan(M, N, K, mode, h->shape, kOneLaunchSliced);
  if (!pl.shape) return no_plan(h, pl, "ecgemm_sgemm");
  if (pl.items() + 16 > 0x7fffffffLL) return bad_arg(h, 4, "ecgemm_sgemm: too many tiles");
  SplitJob job_a, job_b;
  char* ws = nullptr;
  st = acquire_workspace(h, pl.total_bytes, &ws, workspace_kind);
  if (st != ECGEMM_OK) return st;
  char* a_packed = ws;
  char* b_packed = ws + pl.a_bytes;
  float* partials = pl.tail_splits > 1 ? reinterpret_cast<float*>(ws + pl.a_bytes + pl.b_bytes) : nullptr;
  if (!pl.shape->fused) {
    // step 1: op(A) is M x K with rows m; op(B)^T is N x K with rows n.  For B the roles of N and T swap:
    // B stored K x N (transB == N) has k contiguous, i.e. it is the "T" case of the splitter.
    st = make_split_job(h, transA, M, K, A, lda, a_packed, h->log2_scale_a, row_log2_scale_a, &job_a);
    if (st != ECGEMM_OK) return st;
    st = make_split_job(h, transB == ECGEMM_OP_N ? ECGEMM_OP_T : ECGEMM_OP_N, N, K, B, ldb, b_packed, h->log2_scale_b,
                        col_log2_scale_b, &job_b);
    if (st != ECGEMM_OK) return st;
  }

  EventLease lease{h};
  TimedCall& tc = lease.tc;
  const bool timing = h->timing && workspace_kind != kWorkspaceBuiltIn;  // (creating an event allocates)
  if (timing) {
    tc.start = take_event(h);
    tc.split_done = take_event(h);
    tc.product_done = take_event(h);
    if (!tc.start || !tc.split_done || !tc.product_done) return fail(h, ECGEMM_ERR_HIP, "ecgemm_sgemm: hipEventCreate failed");
    ECGEMM_HIP(h, hipEventRecord(tc.start, h->stream));
  }

  if (pl.shape->fused) {
    if (timing) ECGEMM_HIP(h, hipEventRecord(tc.split_done, h->stream));  // no split pass: all the time is the product's
    st = launch_fused(h, pl, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, row_log2_scale_a, col_log2_scale_b, partials);
  } else {
    st = launch_split(h, mode, job_a, &job_b);
    if (st != ECGEMM_OK) return st;
    if (timing) ECGEMM_HIP(h, hipEventRecord(tc.split_done, h->stream));
    // steps 2 and 3
    st = launch_product(h, pl, M, N, alpha, a_packed, b_packed, beta, C, ldc, mode, partials,
                        -(h->log2_scale_a + h->log2_scale_b), row_log2_scale_a, col_log2_scale_b);
  }
  if (st != ECGEMM_OK) return st;
  if (timing) {
    ECGEMM_HIP(h, hipEventRecord(tc.product_done, h->stream));
    h->timed.push_back(tc);
    lease.keep = true;
  }
  return ECGEMM_OK;
}

}  // namespace

extern "C" {

ecgemm_status_t ecgemm_sgemm(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                             int64_t M, int64_t N, int64_t K, float alpha,
                             const float* A, int64_t lda, const float* B, int64_t ldb,
                             float beta, float* C, int64_t ldc, ecgemm_mode_t mode) {
  return sgemm_common(handle, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, mode, nullptr, nullptr,
                      kWorkspaceOfHandle);
}

ecgemm_status_t ecgemm_sgemm_scaled(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                                    int64_t M, int64_t N, int64_t K, float alpha,
                                    const float* A, int64_t lda, const float* B, int64_t ldb,
                                    float beta, float* C, int64_t ldc, ecgemm_mode_t mode,
                                    const int32_t* row_log2_scale_a, const int32_t* col_log2_scale_b) {
  return sgemm_common(handle, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, mode, row_log2_scale_a,
                      col_log2_scale_b, kWorkspaceOfHandle);
}

ecgemm_status_t ecgemm_sgemm_noalloc(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                                     int64_t M, int64_t N, int64_t K, float alpha,
                                     const float* A, int64_t lda, const float* B, int64_t ldb,
                                     float beta, float* C, int64_t ldc, ecgemm_mode_t mode) {
  return sgemm_common(handle, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, mode, nullptr, nullptr,
                      kWorkspaceBuiltIn);
}

ecgemm_status_t ecgemm_auto_choice(ecgemm_handle_t handle, ecgemm_mode_t* mode, int* scaling_vectors) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!mode) return bad_arg(handle, 2, "ecgemm_auto_choice: null output");
  if (!scaling_vectors) return bad_arg(handle, 3, "ecgemm_auto_choice: null output");
  if (!handle->auto_choice)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_auto_choice: the handle's last product call made no choice (not ECGEMM_MODE_AUTO, or empty)", 1);
  int choice = -1;
  ECGEMM_HIP(handle, hipMemcpyAsync(&choice, handle->auto_choice, sizeof(int), hipMemcpyDeviceToHost, handle->stream));
  ECGEMM_HIP(handle, hipStreamSynchronize(handle->stream));
  *mode = (choice == kChoiceFp16 || choice == kChoiceFp16Scaled) ? ECGEMM_MODE_FP16_SPLIT : ECGEMM_MODE_BF16_FULL;
  *scaling_vectors = choice == kChoiceFp16Scaled ? 1 : 0;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_product(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, float alpha,
                               const void* packedA, const void* packedB, float beta, float* C, int64_t ldc,
                               ecgemm_mode_t mode) {
  ecgemm_handle_t h = handle;
  if (!h) return ECGEMM_ERR_INVALID_ARG;
  if (M < 0) return bad_arg(h, 2, "ecgemm_product: negative M");
  if (N < 0) return bad_arg(h, 3, "ecgemm_product: negative N");
  if (K < 0) return bad_arg(h, 4, "ecgemm_product: negative K");
  if (!valid_mode(mode)) return bad_arg(h, 11, "ecgemm_product: unknown mode");
  h->auto_choice = nullptr;
  if (M == 0 || N == 0) return ECGEMM_OK;
  if (!C) return bad_arg(h, 9, "ecgemm_product: C is null");
  if (ldc < M) return bad_arg(h, 10, "ecgemm_product: ldc < M");
  if (K == 0 || alpha == 0.0f) {
    const dim3 grid((unsigned)((M + 255) / 256), (unsigned)(N < 65535 ? N : 65535));
    hipLaunchKernelGGL(scale_c_kernel, grid, dim3(256), 0, h->stream, M, N, beta, C, ldc);
    ECGEMM_HIP(h, hipGetLastError());
    return ECGEMM_OK;
  }
  if (!packedA || ((uintptr_t)packedA % 16) != 0) return bad_arg(h, 6, "ecgemm_product: packed operand is null or not 16-byte aligned");
  if (!packedB || ((uintptr_t)packedB % 16) != 0) return bad_arg(h, 7, "ecgemm_product: packed operand is null or not 16-byte aligned");
  ecgemm_status_t st = check_sizes(h, M, N, K, mode, 2);
  if (st != ECGEMM_OK) return st;
  const Plan pl = make_plan(M, N, K, mode, h->shape, kOneLaunchNever);
  if (!pl.shape || pl.shape->fused)
    return fail(h, ECGEMM_ERR_UNSUPPORTED, "ecgemm_product: the handle's kernel shape does not take packed operands in this mode");
  if (pl.items() + 16 > 0x7fffffffLL) return bad_arg(h, 2, "ecgemm_product: too many tiles");
  char* ws = nullptr;
  st = acquire_workspace(h, pl.partial_bytes, &ws);
  if (st != ECGEMM_OK) return st;
  return launch_product(h, pl, M, N, alpha, packedA, packedB, beta, C, ldc, mode, reinterpret_cast<float*>(ws));
}

}  // extern "C"
