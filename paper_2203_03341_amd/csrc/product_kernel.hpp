// Steps 2 and 3 of the error-corrected SGEMM: the MFMA main loop and the merge epilogue.
//
// FP16 mode (Eq. corr-5-1024-reduce):   C = A16 B16 + (dA16 B16 + A16 dB16) / 2^11
// BF16 mode (a = a0 + a1 + a2, b alike): C = a0 b0 + [a0 b1 + a1 b0 + a1 b1 + a0 b2 + a2 b0]
//
// The leading product has an FP32 accumulator of its own; every correction product goes to a
// second FP32 accumulator (the frag_dc of the paper's listing) and the two meet once, after
// the loop.  That matters on this hardware for the same reason it does in the paper: the
// matrix unit aligns all addends of one instruction to the largest exponent among them and
// drops what falls below about 2^-25 of it, so a correction term added into the big
// accumulator would lose its low bits, while among terms of its own size it loses nothing.
// The accumulate itself rounds to nearest even on gfx950 (measured), so the paper's
// zero-accumulator trick against round-toward-zero is not needed here.
//
// Data flow per workgroup (one per CU, 4 waves, one per SIMD, up to 512 registers each, for the
// 256 x 128 tile; two per CU for the 128 x 128 tile used when K is shallow):
//   packed operands (HBM/L2) --global_load_lds 16 B/lane--> LDS ring of 2 or 3 stages (no VGPR staging)
//   LDS --ds_read_b128--> operand fragments, double buffered in registers
//   v_mfma_f32_32x32x16_{f16,bf16} --> 2 x (TM x TN) accumulators of 16 floats per lane
// Operands are stored in fragment order (see split_kernels.hpp), so both hops are linear
// 1 KiB-per-wave copies: coalesced in global memory and bank-conflict free in LDS by construction.
//
// Besides the two modes of the method the kernel can run the paper's comparison methods (see ProductMethod):
// Markidis' four products into one accumulator, the three products with an unscaled residual, and plain
// one-product FP16 / BF16 GEMMs.  They share every line of the data path and differ only in the product list.
//
// The matrix instruction is used "transposed": the B-side fragment is its first operand and
// the A-side fragment its second, so a lane owns one row index m of C and a wave's store
// instruction covers 32 consecutive m: 128-byte runs of column-major C.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "split_kernels.hpp"

namespace ecgemm {

typedef float float16_t __attribute__((ext_vector_type(16)));


// 2^e as a float, e in [-126, 127]
__device__ __forceinline__ float exp2_int(int e) { return __builtin_bit_cast(float, (unsigned)(e + 127) << 23); }

// c * 2^-(row_exponent + col_exponent), exact whenever the result is a normal FP32 number.  The exponents are in
// [-126, 126] each, so their sum may be beyond what one factor expresses: it is applied in two halves, which keeps
// the intermediate between c and the result (taking the two exponents one after the other would not: 2^-row alone
// can overflow where the product of both is an ordinary number).
__device__ __forceinline__ float unscale(float c, int row_exponent, int col_exponent) {
  const int total = -(row_exponent + col_exponent), half = total / 2;
  return c * exp2_int(half) * exp2_int(total - half);
}

// An element of C is written once and not read again by this call: a non-temporal store keeps it from pushing the
// operand panels out of the L2 (measured: 19 % off the 256 x 128 kernel and 4 % off the 128 x 128 kernel at
// 16384 x 16384 x 256, where C is most of the traffic; nothing lost at 16384^3).
// (Through a pointer known to be global memory: a generic pointer makes these FLAT instructions, which also count
// against the LDS counter that the fragment reads of the main loop wait on.)
typedef __attribute__((address_space(1))) float global_float_t;
__device__ __forceinline__ void store_result(float* dst, float value) {
  __builtin_nontemporal_store(value, (global_float_t*)dst);
}
__device__ __forceinline__ float load_global(const float* src) { return *(const global_float_t*)src; }
__device__ __forceinline__ int load_global(const int* src) { return *(const __attribute__((address_space(1))) int*)src; }
// partial sums are read again soon by the kernel that adds the slices: an ordinary store
__device__ __forceinline__ void store_partial(float* dst, float value) { *(global_float_t*)dst = value; }

// alpha c + beta C_in with the roundings fixed (alpha c rounded, then one fused multiply-add), so that the compiler
// cannot pick a different contraction in each kernel and every kernel shape gives the same bits.
__device__ __forceinline__ float scaled_sum(float alpha, float c, float beta, float c_in) {
  return __builtin_fmaf(beta, c_in, alpha * c);
}

// Output tile number -> tile coordinates.  The tile grid is cut into column_bands bands of (nearly) equal width, taken
// one after the other; inside a band the tiles go in groups of group_m tile rows, each walked column by column, so
// that tiles with neighbouring numbers share A and B panels.  column_bands <= tiles_n.
__host__ __device__ __forceinline__ void tile_coordinates(int pid, int tiles_m, int tiles_n, int group_m, int column_bands,
                                                          int& tile_m, int& tile_n) {
  const int narrow = tiles_n / column_bands, wider = tiles_n % column_bands;  // the first `wider` bands have narrow + 1 columns
  const int tiles_wide = (narrow + 1) * tiles_m;
  int width, first_n;
  if (pid < wider * tiles_wide) {
    const int band = pid / tiles_wide;
    pid -= band * tiles_wide;
    width = narrow + 1;
    first_n = band * width;
  } else {
    pid -= wider * tiles_wide;
    const int band = pid / (narrow * tiles_m);
    pid -= band * (narrow * tiles_m);
    width = narrow;
    first_n = wider * (narrow + 1) + band * narrow;
  }
  const int group_size = group_m * width;
  const int group = pid / group_size;
  const int first_m = group * group_m;
  const int rows_here = tiles_m - first_m < group_m ? tiles_m - first_m : group_m;
  tile_m = first_m + (pid % group_size) % rows_here;
  tile_n = first_n + (pid % group_size) / rows_here;
}

// Division of 0 <= n < 2^31 by a divisor known to the host before the launch: one multiply-high and a shift instead of
// the forty-odd instructions of a 32-bit division (the tile arithmetic of an item sits on the critical path between
// two main loops, and a wave issues one instruction every four or five cycles).  With l = ceil(log2 d) and
// mul = ceil(2^(31 + l) / d), floor(n mul / 2^(31 + l)) = floor(n / d) for every n < 2^31.  mul == 0 stands for d == 1.
struct FastDivisor {
  unsigned mul, shift;
};
inline FastDivisor fast_divisor(int d) {  // d >= 1
  if (d <= 1) return FastDivisor{0u, 0u};
  unsigned l = 0;
  while ((1ull << l) < (unsigned long long)d) ++l;  // l = ceil(log2 d) >= 1
  const unsigned long long two = 1ull << (31 + l);
  return FastDivisor{(unsigned)((two + d - 1) / d), l - 1};
}
__host__ __device__ __forceinline__ int fast_div(int n, FastDivisor f) {
  return f.mul ? (int)((unsigned)(((unsigned long long)(unsigned)n * f.mul) >> 32) >> f.shift) : n;
}

// The tile order of tile_coordinates with everything that does not depend on the tile number worked out on the host.
struct TileOrder {
  int tiles_m, tiles_n, group_m, column_bands;
  int narrow, wider;             // tiles_n / column_bands and tiles_n % column_bands: the first `wider` bands have narrow + 1 columns
  int tiles_wide, tiles_narrow;  // tiles of a band of either width
  FastDivisor by_tiles_wide, by_tiles_narrow, by_group_wide, by_group_narrow, by_group_m, by_last_rows;
};
inline TileOrder make_tile_order(int tiles_m, int tiles_n, int group_m, int column_bands) {
  TileOrder o;
  o.tiles_m = tiles_m, o.tiles_n = tiles_n, o.group_m = group_m, o.column_bands = column_bands;
  o.narrow = tiles_n / column_bands, o.wider = tiles_n % column_bands;
  o.tiles_wide = (o.narrow + 1) * tiles_m, o.tiles_narrow = o.narrow * tiles_m;
  o.by_tiles_wide = fast_divisor(o.tiles_wide);
  o.by_tiles_narrow = fast_divisor(o.tiles_narrow);
  o.by_group_wide = fast_divisor(group_m * (o.narrow + 1));
  o.by_group_narrow = fast_divisor(group_m * o.narrow);
  o.by_group_m = fast_divisor(group_m);
  o.by_last_rows = fast_divisor(tiles_m % group_m);  // rows of the last, shorter group of tile rows (if there is one)
  return o;
}
// tile_coordinates(pid, o.tiles_m, o.tiles_n, o.group_m, o.column_bands, ...) without a division
__host__ __device__ __forceinline__ void tile_coordinates(int pid, const TileOrder& o, int& tile_m, int& tile_n) {
  int width, first_n;
  FastDivisor by_group;
  if (pid < o.wider * o.tiles_wide) {
    const int band = fast_div(pid, o.by_tiles_wide);
    pid -= band * o.tiles_wide;
    width = o.narrow + 1;
    first_n = band * width;
    by_group = o.by_group_wide;
  } else {
    pid -= o.wider * o.tiles_wide;
    const int band = fast_div(pid, o.by_tiles_narrow);
    pid -= band * o.tiles_narrow;
    width = o.narrow;
    first_n = o.wider * (o.narrow + 1) + band * o.narrow;
    by_group = o.by_group_narrow;
  }
  const int group = fast_div(pid, by_group);
  const int first_m = group * o.group_m;
  const int rest = pid - group * (o.group_m * width);
  const int rows_here = o.tiles_m - first_m < o.group_m ? o.tiles_m - first_m : o.group_m;
  const int column = fast_div(rest, rows_here == o.group_m ? o.by_group_m : o.by_last_rows);
  tile_m = first_m + (rest - column * rows_here);
  tile_n = first_n + column;
}

struct ProductParams {
  const char* a_packed;     // [Mp/32][k_steps][NP][64][8] 16-bit
  const char* b_packed;     // [Np/32][k_steps][NP][64][8] 16-bit
  int64_t row_block_bytes;  // k_steps * NP * 1024
  int k_tiles;              // depth_padded / (16 * K_STEPS): LDS stages along K
  // Work items: the first full_tiles output tiles (in the order of tile_coordinates) are one item each, over the whole
  // depth; each of the remaining tail_tiles is tail_splits items, one per slice of the depth, which leave raw sums in
  // `partials` for reduce_tail_kernel.  tail_splits == 1: those tiles are whole items too and nothing goes to partials.
  int full_tiles, tail_tiles, tail_splits;
  int kt_per_split;            // ceil(k_tiles / tail_splits)
  FastDivisor by_tail_tiles;
  // Tile order (tile_coordinates): group_m tile rows per group; with each XCD taking a contiguous run of the order,
  // column_bands bands of columns lay the 8 XCDs out (8 / column_bands) x column_bands over the tile grid
  TileOrder order;
  int xcd_remap;     // 1 (always, outside experiments): each XCD owns a contiguous run of the tile order; 0: workgroup b
                     // takes item b, b + gridDim.x, ... and the hardware's round-robin decides which XCD that is
  int64_t M, N, ldc;
  float alpha, beta;
  float out_scale;          // power of two that undoes the caller's pre-scaling of A and B (1 by default)
  // per-row / per-column pre-scaling (both null, or both set): element (m, n) of the product is multiplied by
  // 2^-(row_log2_scale[m] + col_log2_scale[n]) before alpha / beta (see unscale())
  const int* row_log2_scale;  // device, M entries
  const int* col_log2_scale;  // device, N entries
  float* C;
  float* partials;          // [tail_splits][tail_tiles][BN][BM] when tail_splits > 1
  // Automatic mode choice only, else null: the kernel does nothing unless *gate == gate_value
  const int* gate;
  int gate_value;
};

// The matrix instruction per element type of the packed operands.  `sub` picks one of the four 2-deep steps that an
// FP32 fragment (four floats per lane) holds; the 16-bit fragments are consumed whole.
enum ElementKind { kElemFp16 = 0, kElemBf16 = 1, kElemFp32 = 2 };
template <int ELEM>
struct Mfma;
template <>
struct Mfma<kElemFp16> {
  typedef half8_t frag_t;
  __device__ static __forceinline__ float16_t run(frag_t x, frag_t y, float16_t acc, int = 0) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, acc, 0, 0, 0);
  }
};
template <>
struct Mfma<kElemBf16> {
  typedef bf16x8_t frag_t;
  __device__ static __forceinline__ float16_t run(frag_t x, frag_t y, float16_t acc, int = 0) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc, 0, 0, 0);
  }
};
template <>
struct Mfma<kElemFp32> {
  typedef float frag_t __attribute__((ext_vector_type(4)));
  __device__ static __forceinline__ float16_t run(frag_t x, frag_t y, float16_t acc, int sub) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(x[sub], y[sub], acc, 0, 0, 0);
  }
};

// Which products are formed and where they are summed.
enum ProductMethod {
  kMethodFp16Split = 0,     // Eq. corr-5-1024-reduce: A16 B16 | dA16 B16 + A16 dB16 (scaled by 2^-11 at the end)
  kMethodBf16Full = 1,      // a0 b0 | a0 b1 + a1 b0 + a1 b1 + a0 b2 + a2 b0
  kMethodFp16Markidis = 2,  // Eq. corr-5 and listing "Markidis' error correction method": dA dB + dA B + A dB + A B, one accumulator
  kMethodFp16Unscaled = 3,  // the method's three products and two accumulators on Markidis' unscaled residual
  kMethodFp16Plain = 4,     // A16 B16 only (listing "A simple matrix-matrix multiplication ... on Tensor Cores")
  kMethodBf16Plain = 5,     // toBF16(A) toBF16(B) only
  kMethodFp16Outside = 6,   // kMethodFp16Split with A16 B16 added to its accumulator outside the matrix unit, every k
                            // step, through a zeroed temporary (frag_tmp of the paper's listing; its contribution 1)
  kMethodFp32 = 7,          // A B in FP32 on the matrix unit (v_mfma_f32_32x32x2_f32): what the method is measured against
  kMethodFp16Outside4 = 8,  // kMethodFp16Outside with A16 B16 left in the matrix unit's accumulator for 4 k steps (64 deep)
  kMethodFp16Outside16 = 9  // ... for 16 k steps (256 deep) before it is added to the running sum outside
};
constexpr int kMethods = 10;

// For the "outside" methods: the number of 16-deep k steps whose leading products the matrix unit sums by itself before
// that sum is added, by FP32 vector instructions, to the running sum kept outside it.  1 is the paper's listing
// (section "Avoiding RZ during Tensor Core accumulation"); 0: the running sum is the matrix unit's accumulator.
__host__ __device__ constexpr int flush_interval_of(int method) {
  return method == kMethodFp16Outside ? 1 : method == kMethodFp16Outside4 ? 4 : method == kMethodFp16Outside16 ? 16 : 0;
}

__host__ __device__ constexpr int split_kind_of(int method) {
  return (method == kMethodFp16Split || flush_interval_of(method) > 0) ? kSplitFp16Scaled
       : method == kMethodBf16Full ? kSplitBf16x3
       : (method == kMethodFp16Markidis || method == kMethodFp16Unscaled) ? kSplitFp16Unscaled
       : method == kMethodFp16Plain ? kSplitFp16Plain : method == kMethodFp32 ? kSplitFp32 : kSplitBf16Plain;
}
__host__ __device__ constexpr int element_kind_of(int method) {
  return method == kMethodFp32 ? kElemFp32 : split_is_bf16(split_kind_of(method)) ? kElemBf16 : kElemFp16;
}
__host__ __device__ constexpr int products_of(int method) {
  return method == kMethodFp16Split || method == kMethodFp16Unscaled || flush_interval_of(method) > 0 ? 3
       : method == kMethodBf16Full ? 6 : method == kMethodFp16Markidis ? 4 : method == kMethodFp32 ? 8 : 1;
}

// Term t of a method's product list: the parts of B and A it multiplies and the accumulator set it goes to.  One
// term at a time runs over all tiles of a wave, so consecutive matrix instructions never share an accumulator.
struct ProductTerm {
  int qb, qa;
  bool correction;
  int sub;  // FP32 only: which of the four 2-deep steps of the fragment pair
};
__host__ __device__ constexpr ProductTerm product_term(int method, int t) {
  if (method == kMethodFp16Markidis)  // everything into one accumulator, smallest first
    return t == 0 ? ProductTerm{1, 1, false, 0} : t == 1 ? ProductTerm{1, 0, false, 0} : t == 2 ? ProductTerm{0, 1, false, 0}
                                                                                                 : ProductTerm{0, 0, false, 0};
  if (method == kMethodBf16Full)
    return t == 0 ? ProductTerm{0, 0, false, 0} : t == 1 ? ProductTerm{2, 0, true, 0} : t == 2 ? ProductTerm{0, 2, true, 0}
         : t == 3 ? ProductTerm{1, 1, true, 0} : t == 4 ? ProductTerm{1, 0, true, 0} : ProductTerm{0, 1, true, 0};
  if (method == kMethodFp32)  // the two 8-deep halves of the k step, four 2-deep matrix instructions each, k ascending
    return ProductTerm{t / 4, t / 4, false, t % 4};
  // kMethodFp16Split, kMethodFp16Unscaled, the outside methods; the plain methods stop after the first term
  return t == 0 ? ProductTerm{0, 0, false, 0} : t == 1 ? ProductTerm{1, 0, true, 0} : ProductTerm{0, 1, true, 0};
}

template <class F, int... I>
__device__ __forceinline__ void static_for_each(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {  // f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>)
  static_for_each(f, std::make_integer_sequence<int, N>{});
}

template <int METHOD, int BM_, int BN_, int WM_, int WN_, int K_STEPS_, int STAGES_, int BLOCKS_PER_CU_ = 1>
struct ProductConfig {
  static constexpr int BLOCKS_PER_CU = BLOCKS_PER_CU_;            // resident workgroups per CU (registers and LDS permitting)
  static constexpr int kMethod = METHOD;
  static constexpr int kElem = element_kind_of(METHOD);
  static constexpr int NP = parts_of_split(split_kind_of(METHOD));  // parts per value
  static constexpr int PRODUCTS = products_of(METHOD);              // matrix products formed
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int K_STEPS = K_STEPS_, BK = 16 * K_STEPS;     // 16-deep MFMA steps per LDS stage
  static constexpr int STAGES = STAGES_;                          // LDS ring: tile t lives in buffer t % STAGES
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN, WAVES = WAVES_M * WAVES_N;
  static constexpr int THREADS = WAVES * 64;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int ROW_CHUNKS = K_STEPS * NP;                 // 1 KiB chunks per 32 rows per stage
  static constexpr int A_CHUNKS = (BM / 32) * ROW_CHUNKS, B_CHUNKS = (BN / 32) * ROW_CHUNKS;
  static constexpr int STAGE_BYTES = (A_CHUNKS + B_CHUNKS) * 1024;
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
  static constexpr int LOADS = (A_CHUNKS + B_CHUNKS) / WAVES;     // global_load_lds instructions per wave per stage
  static constexpr int FRAG_READS = (TM + TN) * NP;               // ds_read_b128 per wave per k step
  static constexpr int MFMAS = TM * TN * PRODUCTS;                // matrix instructions per wave per k step
  // Fragment reads of a k step in the order in which its matrix instructions first need them.
  struct ReadOrder {
    bool from_b[FRAG_READS];
    int tile[FRAG_READS], part[FRAG_READS];
  };
  static constexpr ReadOrder read_order() {
    ReadOrder r{};
    bool seen_a[TM][NP] = {}, seen_b[TN][NP] = {};
    int n = 0;
    for (int m = 0; m < MFMAS; ++m) {
      const ProductTerm t = product_term(METHOD, m / (TM * TN));
      const int i = (m % (TM * TN)) / TN, j = m % TN;
      if (!seen_b[j][t.qb]) {
        seen_b[j][t.qb] = true;
        r.from_b[n] = true, r.tile[n] = j, r.part[n] = t.qb, ++n;
      }
      if (!seen_a[i][t.qa]) {
        seen_a[i][t.qa] = true;
        r.from_b[n] = false, r.tile[n] = i, r.part[n] = t.qa, ++n;
      }
    }
    return r;
  }
  static_assert(K_STEPS == 1 || K_STEPS == 2, "one or two k steps per stage");
  static_assert(STAGES >= 2 && (STAGES - 1) * LOADS <= 63, "vmcnt is a 6-bit counter");
  static_assert(LDS_BYTES * BLOCKS_PER_CU <= 160 * 1024, "LDS budget");
  static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shapes");
  static_assert(kRowPad % BM == 0 && kRowPad % BN == 0, "padded operands must hold whole tiles");
  static_assert(A_CHUNKS % WAVES == 0 && B_CHUNKS % WAVES == 0, "chunks per wave");
};

template <int N>
__device__ __forceinline__ void wait_loads_and_lds() {  // at most N global loads of this wave still in flight
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(N) : "memory");
}

// Every instance undoes per-row / per-column scaling in its epilogue when p.row_log2_scale is set, element by element.
// FAST_SCALED instances, which exist for the method's two modes, do it with the factors and the elements of C fetched
// ahead, as the unscaled paths do; they are instances of their own because that epilogue, though it only runs in
// scaled calls, would weigh on the register allocation of the kernel every call uses.
template <class Cfg, bool FAST_SCALED = false>
__global__ void __launch_bounds__(Cfg::THREADS, Cfg::BLOCKS_PER_CU) product_kernel(const ProductParams p) {
  constexpr int NP = Cfg::NP, TM = Cfg::TM, TN = Cfg::TN, S = Cfg::STAGES;
  typedef typename Mfma<Cfg::kElem>::frag_t frag_t;
  // The ring of stages.  (It must stay the only LDS object of the kernel: with a second one the compiler starts to guard
  // every fragment read with a wait for all LDS-DMA loads in flight, which serialises the ring: 30 % slower.)
  __shared__ __attribute__((aligned(1024))) char lds[Cfg::LDS_BYTES];
  if (!gate_open(p.gate, p.gate_value)) return;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wave_m = wave % Cfg::WAVES_M, wave_n = wave / Cfg::WAVES_M;

  // ---- work items (an item = one output tile x one K slice).  The host launches either one block per item or
  // a persistent grid of one block per CU whose blocks each walk through several items.  Blocks are dealt
  // round-robin to the 8 XCDs, so block b lives on XCD b % 8; that XCD owns one contiguous run of the whole-tile
  // items, followed by one contiguous run of the sliced items, and its blocks stride through that list together, so
  // the ~32 tiles an XCD works on at any time are neighbours that share A and B panels in its L2.
  struct Work {
    int tile_m, tile_n, kt_begin, kt_count;
    int partial;  // index of the [BN][BM] partial tile this item writes, or -1 if it writes C
  };
  constexpr int kReadTail = 6;  // matrix-instruction slots at the end of a k step that carry no fragment read
  const int tail_items = p.tail_tiles * p.tail_splits;
  auto locate = [&](int item) {
    Work w;
    int pid = item;
    w.kt_begin = 0;
    w.kt_count = p.k_tiles;
    w.partial = -1;
    if (item >= p.full_tiles) {
      const int j = item - p.full_tiles, split = fast_div(j, p.by_tail_tiles);
      pid = p.full_tiles + (j - split * p.tail_tiles);
      if (p.tail_splits > 1) {
        w.kt_begin = split * p.kt_per_split;
        w.kt_count = max(0, min(p.k_tiles, w.kt_begin + p.kt_per_split) - w.kt_begin);
        w.partial = j;
      }
    }
    tile_coordinates(pid, p.order, w.tile_m, w.tile_n);
    return w;
  };
  // This block's list of items: position `slot`, slot + slot_stride, ... below slot_end.  (Handing the items of a
  // persistent grid out through atomic counters instead, so that workgroups that finish early take more, was built
  // and measured for the two-per-unit shape: 3 to 30 % slower than one workgroup per item, which the hardware
  // dispatches as slots free up.)
  int slot, slot_end, slot_stride, full_start = 0, full_count = p.full_tiles, tail_start = 0;
  if (p.xcd_remap) {
    constexpr int kXcds = 8;  // gridDim.x is a multiple of 8
    const int xcd = blockIdx.x % kXcds;
    auto share = [&](int n, int& start, int& count) {  // XCD x's part of n things dealt out in contiguous runs
      const int base = n / kXcds, rem = n % kXcds;
      start = xcd * base + min(xcd, rem);
      count = base + (xcd < rem ? 1 : 0);
    };
    int tail_count;
    share(p.full_tiles, full_start, full_count);
    share(tail_items, tail_start, tail_count);
    slot = blockIdx.x / kXcds;
    slot_end = full_count + tail_count;
    slot_stride = gridDim.x / kXcds;
  } else {
    slot = blockIdx.x;
    slot_end = p.full_tiles + tail_items;
    slot_stride = gridDim.x;
  }
  auto item_at = [&](int position) {
    return position < full_count ? full_start + position : p.full_tiles + tail_start + (position - full_count);
  };
  if (slot >= slot_end) return;
  Work work = locate(item_at(slot));

  // ---- global -> LDS: wave w moves the 1 KiB chunks w, w + WAVES, ... of a stage; A_CHUNKS is a
  // multiple of WAVES, so whether load i fetches from A or from B is known at compile time.  Source
  // addresses are wave-uniform (scalar registers) plus 16 bytes per lane.
  constexpr int kLoads = Cfg::LOADS, kALoads = Cfg::A_CHUNKS / Cfg::WAVES;
  const unsigned lane_bytes = lane * 16;
  // What changes from item to item are two addresses, those of the item's first tile in A and in B; this wave's load i
  // starts a fixed distance behind one of them.
  struct Source {
    const char* a;
    const char* b;
  };
  auto source_of = [&](const Work& w) {
    const int64_t first_tile = (int64_t)w.kt_begin * (Cfg::ROW_CHUNKS * 1024);
    return Source{p.a_packed + (int64_t)w.tile_m * (Cfg::BM / 32) * p.row_block_bytes + first_tile,
                  p.b_packed + (int64_t)w.tile_n * (Cfg::BN / 32) * p.row_block_bytes + first_tile};
  };
  const char* src[kLoads];  // of the item whose tiles are being requested
  unsigned k_off = 0;       // bytes from the first tile of that item to the next tile to request
  auto point_sources = [&](const Source& from) {
    k_off = 0;
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      const int c = (i < kALoads ? i : i - kALoads) * Cfg::WAVES + wave;
      src[i] = (i < kALoads ? from.a : from.b) + (int64_t)(c / Cfg::ROW_CHUNKS) * p.row_block_bytes + (c % Cfg::ROW_CHUNKS) * 1024;
    }
  };
  // (returned as a plain pointer: a lambda whose return type carries an address space silently invalidates the host
  // side's instantiation of the kernel, and with it the launch stub)
  auto load_address = [&](int i, unsigned voff) { return src[i] + voff; };
  auto issue_stage = [&](int buf) {  // requests the next tile not yet requested, then moves on by one tile
    char* stage = lds + buf * Cfg::STAGE_BYTES + wave * 1024;
    // one 32-bit vector offset per tile; kept opaque inside this block so that every address folds to
    // "scalar base + vector offset"
    unsigned voff = lane_bytes + k_off;
    asm volatile("" : "+v"(voff));
#pragma unroll
    for (int i = 0; i < kLoads; ++i)
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)load_address(i, voff), (void __attribute__((address_space(3)))*)(stage + i * Cfg::WAVES * 1024),
                                       16, 0, 0);
    k_off += Cfg::ROW_CHUNKS * 1024;
  };

  // ---- LDS -> registers
  frag_t fa[2][TM][NP], fb[2][TN][NP];
  const int a_frag_off = wave_m * TM * Cfg::ROW_CHUNKS * 1024 + lane * 16;
  const int b_frag_off = Cfg::A_CHUNKS * 1024 + wave_n * TN * Cfg::ROW_CHUNKS * 1024 + lane * 16;
  auto read_frags = [&](int set, int buf, int ks) {
    const char* stage = lds + buf * Cfg::STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int q = 0; q < NP; ++q)
        fa[set][i][q] = *reinterpret_cast<const frag_t*>(stage + a_frag_off + ((i * Cfg::K_STEPS + ks) * NP + q) * 1024);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < NP; ++q)
        fb[set][j][q] = *reinterpret_cast<const frag_t*>(stage + b_frag_off + ((j * Cfg::K_STEPS + ks) * NP + q) * 1024);
  };

  float16_t acc_main[TM][TN], acc_corr[TM][TN];
  // "Outside" methods only: the sum that the matrix unit keeps for FLUSH k steps, added to acc_main (which the matrix
  // unit then never touches) by vector instructions, after which it starts from zero again.
  constexpr int FLUSH = flush_interval_of(Cfg::kMethod);
  float16_t acc_inside[FLUSH > 0 ? TM : 1][FLUSH > 0 ? TN : 1];
  int steps_inside = 0;
  auto flush_inside = [&]() {
    if constexpr (FLUSH > 0) {
      float16_t zero;
#pragma unroll
      for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
          for (int v = 0; v < 16; ++v) acc_main[i][j][v] += acc_inside[i][j][v];
          acc_inside[i][j] = zero;
        }
      steps_inside = 0;
    }
  };
  // Zeroing through the matrix unit: 0 x 0 + 0 written by one instruction per 32 x 32 tile instead of sixteen register
  // writes (256 instructions for the 256 x 128 shape: a microsecond per item at one instruction every four or five
  // cycles, while the matrix pipes have nothing to do).  The zero fragment is opaque so that nothing is folded away.
  auto clear_accumulators = [&]() {
    if constexpr (Cfg::BLOCKS_PER_CU > 1) {
      frag_t zero_fragment;
#pragma unroll
      for (int e = 0; e < (int)(sizeof(frag_t) / sizeof(zero_fragment[0])); ++e) zero_fragment[e] = 0;
      asm volatile("" : "+v"(zero_fragment));
      float16_t zero;
#pragma unroll
      for (int v = 0; v < 16; ++v) zero[v] = 0.0f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc_main[i][j] = Mfma<Cfg::kElem>::run(zero_fragment, zero_fragment, zero, 0);
          acc_corr[i][j] = Mfma<Cfg::kElem>::run(zero_fragment, zero_fragment, zero, 0);
        }
    } else {
      // (the 256 x 128 shape, with every register in use, is spilled by the compiler when its accumulators are set by
      // matrix instructions here; it keeps the plain writes)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            acc_main[i][j][v] = 0.0f;
            acc_corr[i][j][v] = 0.0f;
            if constexpr (FLUSH > 0) acc_inside[i][j][v] = 0.0f;
          }
    }
    steps_inside = 0;
  };

  // One k step, in a fixed order.  Matrix instruction m of the step (term by term over all TM x TN tiles) is followed
  // by its share of the step's other work: at most one LDS-DMA load of the tile being requested (LOAD != 0) and at
  // most one fragment read for a later k step (READ_SET >= 0), each spread evenly over the step.  A matrix instruction
  // occupies the pipe for 8 passes, so whatever is issued behind it is free.  The fence after every slot keeps the
  // compiler's scheduler from regrouping them: left to itself it issued the loads in one burst and put dependent
  // matrix instructions next to each other.
  auto fused_step = [&](auto set_c, auto load_c, auto read_set_c, int load_buf, int read_buf, auto read_ks_c, bool load_now = true) {
    constexpr int SET = decltype(set_c)::value, READ_SET = decltype(read_set_c)::value, READ_KS = decltype(read_ks_c)::value;
    // load_c: 0 no loads, 1 loads, 2 loads if load_now (each load under a scalar branch of its own, so that the matrix
    // instructions stay one straight line whichever way it goes)
    constexpr bool kLoadsDecidedHere = decltype(load_c)::value == 2;
    constexpr int LOADS = decltype(load_c)::value != 0 ? kLoads : 0, READS = READ_SET >= 0 ? Cfg::FRAG_READS : 0;
    constexpr int M = Cfg::MFMAS;
    char* load_stage = lds + load_buf * Cfg::STAGE_BYTES + wave * 1024;
    const char* read_stage = lds + read_buf * Cfg::STAGE_BYTES;
    // one 32-bit vector offset per requested tile; kept opaque so that every address folds to "scalar base + vector
    // offset" and the scalar bases never change
    unsigned voff = lane_bytes + k_off;
    if constexpr (LOADS > 0) {
      asm volatile("" : "+v"(voff));
      if (!kLoadsDecidedHere || load_now) k_off += Cfg::ROW_CHUNKS * 1024;
    }
    static_for<M>([&](auto m_c) {
      constexpr int m = decltype(m_c)::value;
      constexpr ProductTerm term = product_term(Cfg::kMethod, m / (TM * TN));
      constexpr int i = (m % (TM * TN)) / TN, j = m % TN;
      if constexpr (FLUSH > 0 && !term.correction) {
        acc_inside[i][j] = Mfma<Cfg::kElem>::run(fb[SET][j][term.qb], fa[SET][i][term.qa], acc_inside[i][j], term.sub);
      } else if constexpr (term.correction) {
        acc_corr[i][j] = Mfma<Cfg::kElem>::run(fb[SET][j][term.qb], fa[SET][i][term.qa], acc_corr[i][j], term.sub);
      } else {
        acc_main[i][j] = Mfma<Cfg::kElem>::run(fb[SET][j][term.qb], fa[SET][i][term.qa], acc_main[i][j], term.sub);
      }
      static_for<(m + 1) * LOADS / M - m * LOADS / M>([&](auto d_c) {
        constexpr int l = m * LOADS / M + decltype(d_c)::value;
        if (!kLoadsDecidedHere || load_now)
          __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)load_address(l, voff), (void __attribute__((address_space(3)))*)(load_stage + l * Cfg::WAVES * 1024),
                                           16, 0, 0);
      });
      // (the reads stop kReadTail slots before the end of the step, so that the last of them has arrived
      // when the wave gets to the wait in front of the barrier or of the next step)
      // (two slots in a step of twelve instructions or fewer, the 128 x 128 FP16 shape: 1 to 2 %)
      constexpr int SPAN = M > 2 * kReadTail ? M - kReadTail : M > 4 ? M - 2 : M;
      constexpr int r_begin = m < SPAN ? m * READS / SPAN : READS, r_end = m + 1 < SPAN ? (m + 1) * READS / SPAN : READS;
      static_for<r_end - r_begin>([&](auto d_c) {
        constexpr int r = r_begin + decltype(d_c)::value;
        constexpr typename Cfg::ReadOrder order = Cfg::read_order();
        constexpr int tile = order.tile[r], part = order.part[r];
        constexpr bool from_b = order.from_b[r];
        if constexpr (from_b)
          fb[READ_SET < 0 ? 0 : READ_SET][tile][part] =
              *reinterpret_cast<const frag_t*>(read_stage + b_frag_off + ((tile * Cfg::K_STEPS + READ_KS) * NP + part) * 1024);
        else
          fa[READ_SET < 0 ? 0 : READ_SET][tile][part] =
              *reinterpret_cast<const frag_t*>(read_stage + a_frag_off + ((tile * Cfg::K_STEPS + READ_KS) * NP + part) * 1024);
      });
      __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (FLUSH > 0) {
      if (++steps_inside == FLUSH) flush_inside();
    }
  };
  typedef std::integral_constant<int, 0> none_t;
  typedef std::integral_constant<int, 1> loads_t;
  typedef std::integral_constant<int, 2> loads_if_t;
  typedef std::integral_constant<int, -1> no_reads_t;
  typedef std::integral_constant<int, 0> set0_t;
  typedef std::integral_constant<int, 1> set1_t;
  typedef std::integral_constant<int, 0> ks0_t;
  typedef std::integral_constant<int, 1> ks1_t;

  // Matrix instructions have no memory side effects, so the compiler would move the barrier across them;
  // the fences pin it.  The wait lets the newest STAGES - 2 tiles stay in flight (or none, near the end).
  auto stage_barrier = [&](auto pending_c) {
    __builtin_amdgcn_sched_barrier(0);
    wait_loads_and_lds<decltype(pending_c)::value>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- the stream of tiles.  The tiles (LDS stages) of this block's items form one sequence: all tiles of its first
  // item, then all tiles of its second item, and so on.  Tile g of the sequence lives in ring buffer g % STAGES, and
  // requests run up to STAGES tiles ahead of the multiplications - across the boundary to the next item, so that its
  // first tiles travel while the last tiles of this one are multiplied and while its results are written out.  (Asking
  // for them after the loop instead leaves the matrix pipes idle for as long as the vector memory path needs to take
  // STAGES stages in: 1.7 us for 144 KiB at 64 bytes per cycle.)
  //   multiply side:  work = item being multiplied, buf = buffer of the tile being multiplied
  //   request side:   req_src / k_off = where the next tile to request starts, req_left = tiles still to request of the
  //                   item that requests are in (the one being multiplied, or the one after it once req_ahead is set;
  //                   requests never look further ahead), fill_buf = the buffer the next request goes to,
  //                   pending = tiles requested whose arrival has not been waited for yet
  int req_left = 0, fill_buf = 0, pending = 0;
  bool req_ahead = false, have_next = false;
  Source next_src{nullptr, nullptr};
  int next_tiles = 0;
  auto look_ahead = [&](int next_slot) {  // the item after the one being multiplied, if there is one
    have_next = next_slot < slot_end;
    if (have_next) {
      const Work w = locate(item_at(next_slot));
      next_src = source_of(w);
      next_tiles = w.kt_count;
    }
  };
  auto tile_requested = [&]() {  // after the loads of one tile have been issued into fill_buf
    fill_buf = (fill_buf + 1 == S) ? 0 : fill_buf + 1;
    ++pending;
    if (--req_left == 0 && !req_ahead && have_next) {  // on to the first tile of the next item
      req_ahead = true;
      point_sources(next_src);
      req_left = next_tiles;
    }
  };
  auto top_up = [&]() {  // as many requests as there are free buffers (start of the kernel; after items of few tiles)
    while (pending < S && req_left > 0) {
      issue_stage(fill_buf);
      tile_requested();
    }
  };
  // waits until at most `tiles` of the tiles requested by this wave are still in flight (and for its LDS reads)
  auto wait_for_tiles = [&](int tiles) {
    static_assert(S <= 4, "wait_for_tiles knows up to three tiles in flight");
    if (tiles <= 0) wait_loads_and_lds<0>();
    else if (tiles == 1) wait_loads_and_lds<Cfg::LOADS>();
    else if (tiles == 2) wait_loads_and_lds<(S > 2 ? 2 : 0) * Cfg::LOADS>();
    else wait_loads_and_lds<(S > 3 ? 3 : 0) * Cfg::LOADS>();
  };
  // The next tile to multiply has been requested (it always has: it is at most one item ahead); when this returns it
  // has landed for every wave.  Matrix instructions have no memory side effects: the fences pin the barrier.
  auto tile_barrier = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    wait_for_tiles(pending - 1);
    --pending;
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  // barrier that only protects a buffer about to be refilled (no tile is waited for)
  auto refill_barrier = [&]() { stage_barrier(std::integral_constant<int, 63>{}); };

  point_sources(source_of(work));
  req_left = work.kt_count;
  look_ahead(slot + slot_stride);
  if (req_left == 0 && have_next) {
    req_ahead = true;
    point_sources(next_src);
    req_left = next_tiles;
  }
  top_up();

  int buf = 0;
  while (true) {
  const int kt_count = work.kt_count;
  clear_accumulators();
  if (kt_count > 0) {
    // The first tile of the item must have landed.  (Stores of the previous item's epilogue may still be in flight
    // behind the loads: waiting for "all but the newest n operations" then waits for more than needed, never for less.)
    tile_barrier();
    read_frags(0, buf, 0);
    int next = (buf + 1 == S) ? 0 : buf + 1;
    auto advance = [&]() {
      buf = next;
      next = (next + 1 == S) ? 0 : next + 1;
    };
    // The loops below keep the matrix instructions of an iteration in one straight line (a branch with matrix
    // instructions on both sides makes the register allocator shuffle the accumulators where the sides join).
    // Steady state - the ring is full (STAGES - 1 tiles requested beyond the one being multiplied) and the next
    // request stays within the same item - runs in a loop of its own with fixed waits and no bookkeeping; the iterations
    // after it (the last few of an item, or all of a short one) count tiles and take their loads under scalar branches.
    typedef std::integral_constant<int, (S - 2) * Cfg::LOADS> steady_t;
    if constexpr (Cfg::K_STEPS == 2) {
      // Iteration t multiplies tile t: its first k step from fragment set 0 while set 1 is read, then, once every wave
      // holds the tile's last fragments (barrier), its second k step while the buffer is refilled and the first
      // fragments of tile t + 1 are read.
      const int steady = (pending == S - 1 && req_left >= 2) ? min(kt_count - 1, req_left - 1) : 0;
      for (int i = 0; i < steady; ++i) {
        fused_step(set0_t{}, none_t{}, set1_t{}, 0, buf, ks1_t{});
        stage_barrier(steady_t{});
        fused_step(set1_t{}, loads_t{}, set0_t{}, buf, next, ks0_t{});
        advance();
      }
      req_left -= steady;
      if (steady > 0) fill_buf = buf;  // (with the ring full, the buffer to fill is the one being multiplied from)
      for (int t = steady; t < kt_count - 1; ++t) {
        fused_step(set0_t{}, none_t{}, set1_t{}, 0, buf, ks1_t{});
        tile_barrier();
        const bool request = req_left > 0;
        fused_step(set1_t{}, loads_if_t{}, set0_t{}, fill_buf, next, ks0_t{}, request);
        if (request) tile_requested();
        advance();
      }
      // the last tile of the item: nothing of this item is left to read
      fused_step(set0_t{}, none_t{}, set1_t{}, 0, buf, ks1_t{});
      const bool request = req_left > 0;
      if (request) refill_barrier();
      fused_step(set1_t{}, loads_if_t{}, no_reads_t{}, fill_buf, 0, ks0_t{}, request);
      if (request) tile_requested();
      advance();
    } else {
      // One k step per stage: tile t is multiplied from one fragment set while the other is filled with the fragments
      // of tile t + 1.  The barrier in front of a step comes when every wave holds the fragments of tile t, whose
      // buffer is then refilled.  Register arrays must be indexed statically, so the steady loop advances two tiles at
      // a time; a single step is followed by a register copy that puts the live fragments back into set 0.
      auto fragments_back_to_set0 = [&]() {
#pragma unroll
        for (int q = 0; q < NP; ++q) {
#pragma unroll
          for (int i = 0; i < TM; ++i) fa[0][i][q] = fa[1][i][q];
#pragma unroll
          for (int j = 0; j < TN; ++j) fb[0][j][q] = fb[1][j][q];
        }
      };
      auto steady_step = [&](auto set_c) {
        constexpr int set = decltype(set_c)::value;
        stage_barrier(steady_t{});
        fused_step(set_c, loads_t{}, std::integral_constant<int, set ^ 1>{}, buf, next, ks0_t{});
        advance();
      };
      const int steady = (pending == S - 1 && req_left >= 2) ? min(kt_count - 1, req_left - 1) : 0;
      if (steady & 1) {
        steady_step(set0_t{});
        fragments_back_to_set0();
      }
      for (int i = steady & 1; i < steady; i += 2) {
        steady_step(set0_t{});
        steady_step(set1_t{});
      }
      req_left -= steady;
      if (steady > 0) fill_buf = buf;
      for (int t = steady; t < kt_count - 1; ++t) {
        tile_barrier();
        const bool request = req_left > 0;
        fused_step(set0_t{}, loads_if_t{}, set1_t{}, fill_buf, next, ks0_t{}, request);
        if (request) tile_requested();
        advance();
        fragments_back_to_set0();
      }
      // the last tile of the item
      const bool request = req_left > 0;
      if (request) refill_barrier();
      fused_step(set0_t{}, loads_if_t{}, no_reads_t{}, fill_buf, 0, ks0_t{}, request);
      if (request) tile_requested();
      advance();
    }
  }
  // ---- next item (its first tiles have been on their way since the last iterations above)
  const Work done = work;
  slot += slot_stride;
  const bool more = slot < slot_end;
  if (more) {
    work = locate(item_at(slot));
    const bool stalled = req_left == 0;  // every tile of the new item has been requested already
    req_ahead = false;
    look_ahead(slot + slot_stride);
    if (stalled && have_next) {
      req_ahead = true;
      point_sources(next_src);
      req_left = next_tiles;
    }
    top_up();
  }

  // ---- epilogue: merge the two accumulators, then alpha / beta (or raw partial sums for a slice of a tile).
  // Lane l holds row m = m_base + 32 i and, in register v of tile (i, j), column n_base + 32 j + 8 (v / 4) + v % 4.
  const int tile_m = done.tile_m, tile_n = done.tile_n;
  const float corr_scale = (Cfg::kMethod == kMethodFp16Split || FLUSH > 0) ? 0x1p-11f : 1.0f;  // unused accumulators stay zero
  if constexpr (FLUSH > 0) flush_inside();  // what the matrix unit still holds of the leading product
  auto merged = [&](int i, int j, int v) { return acc_main[i][j][v] + acc_corr[i][j][v] * corr_scale; };
  // The compiler must not carry this item's 128 store addresses (or their lane-dependent parts) through the main
  // loop of the next item, where it would have to spill them: what they are computed from is made opaque here, so
  // they are recomputed per item.  The lane number itself is counted afresh (two instructions) rather than kept: with
  // all 512 registers of the 256 x 128 shape in use, keeping it alive through the loop cost a trip to scratch memory
  // per item, whose wait also drained the next item's first loads.
  int lane_here;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_here));
  int64_t ldc = p.ldc;
  float* c_base = p.C;
  asm volatile("" : "+s"(ldc), "+s"(c_base));
  const int64_t m_base = (int64_t)tile_m * Cfg::BM + wave_m * Cfg::WM + (lane_here & 31);
  const int64_t n_base = (int64_t)tile_n * Cfg::BN + wave_n * Cfg::WN + 4 * (lane_here >> 5);
  auto for_each_output = [&](auto&& store) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          store(m_base + i * 32, n_base + j * 32 + 8 * (v / 4) + (v % 4),
                merged(i, j, v) * p.out_scale);
  };
  const bool interior = (int64_t)(tile_m + 1) * Cfg::BM <= p.M && (int64_t)(tile_n + 1) * Cfg::BN <= p.N;
  if (p.row_log2_scale != nullptr) {
    // rows of op(A) and columns of op(B) were scaled one by one before the split: undo that per element
    const int* row_scale = p.row_log2_scale;
    const int* col_scale = p.col_log2_scale;
    asm volatile("" : "+s"(row_scale), "+s"(col_scale));
    float* out = done.partial >= 0 ? p.partials + (int64_t)done.partial * (Cfg::BM * Cfg::BN) : nullptr;
    const int64_t m0 = (int64_t)tile_m * Cfg::BM, n0 = (int64_t)tile_n * Cfg::BN;
    bool written = false;
    if constexpr (FAST_SCALED) {
      if (interior && out == nullptr) {
        written = true;
        // a lane needs the exponents of its TM rows and, per 32 x 32 block, of 16 columns
        int row_exponent[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) row_exponent[i] = load_global(row_scale + m_base + i * 32);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          int col_exponent[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) col_exponent[v] = load_global(col_scale + n_base + j * 32 + 8 * (v / 4) + (v % 4));
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            float* dst = c_base + (m_base + i * 32) + (n_base + j * 32) * ldc;
            if (p.beta != 0.0f) {
              float c_in[16];
#pragma unroll
              for (int v = 0; v < 16; ++v) c_in[v] = load_global(dst + (8 * (v / 4) + (v % 4)) * ldc);
#pragma unroll
              for (int v = 0; v < 16; ++v)
                store_result(dst + (8 * (v / 4) + (v % 4)) * ldc,
                             scaled_sum(p.alpha, unscale(merged(i, j, v) * p.out_scale, row_exponent[i], col_exponent[v]), p.beta, c_in[v]));
            } else {
#pragma unroll
              for (int v = 0; v < 16; ++v)
                store_result(dst + (8 * (v / 4) + (v % 4)) * ldc,
                             p.alpha * unscale(merged(i, j, v) * p.out_scale, row_exponent[i], col_exponent[v]));
            }
          }
        }
      }
    }
    if (!written) for_each_output([&](int64_t m, int64_t n, float c) {
      if (m < p.M && n < p.N) {
        c = unscale(c, load_global(row_scale + m), load_global(col_scale + n));
        if (out) {
          store_partial(out + (n - n0) * Cfg::BM + (m - m0), c);
        } else {
          float* dst = c_base + m + n * ldc;
          store_result(dst, (p.beta == 0.0f) ? p.alpha * c : scaled_sum(p.alpha, c, p.beta, load_global(dst)));
        }
      } else if (out) {
        store_partial(out + (n - n0) * Cfg::BM + (m - m0), 0.0f);
      }
    });
  } else if (done.partial >= 0) {
    float* out = p.partials + (int64_t)done.partial * (Cfg::BM * Cfg::BN);
    const int64_t m0 = (int64_t)tile_m * Cfg::BM, n0 = (int64_t)tile_n * Cfg::BN;
    for_each_output([&](int64_t m, int64_t n, float c) { store_partial(out + (n - n0) * Cfg::BM + (m - m0), c); });
  } else if (interior && p.beta == 0.0f) {
    // (multiplying by an out_scale or an alpha of exactly 1 changes no bit, so the common case may skip both)
    if (p.alpha == 1.0f && p.out_scale == 1.0f) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            store_result(c_base + (m_base + i * 32) + (n_base + j * 32 + 8 * (v / 4) + (v % 4)) * ldc,
                         merged(i, j, v));
    } else {
      for_each_output([&](int64_t m, int64_t n, float c) { store_result(c_base + m + n * ldc, p.alpha * c); });
    }
  } else if (interior) {
    // beta != 0: the elements of C that a 32 x 32 tile updates are requested together, then merged and written, so that
    // their latencies overlap (taken one by one, every load would be waited for before the store in front of the next)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float* dst[16];
        float c_in[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          dst[v] = c_base + (m_base + i * 32) + (n_base + j * 32 + 8 * (v / 4) + (v % 4)) * ldc;
          c_in[v] = load_global(dst[v]);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v)
          store_result(dst[v], scaled_sum(p.alpha, merged(i, j, v) * p.out_scale, p.beta, c_in[v]));
      }
  } else {
    for_each_output([&](int64_t m, int64_t n, float c) {
      if (m < p.M && n < p.N) {
        float* dst = c_base + m + n * ldc;
        store_result(dst, (p.beta == 0.0f) ? p.alpha * c : scaled_sum(p.alpha, c, p.beta, load_global(dst)));
      }
    });
  }
  if (!more) break;
  }  // items
}

// Sums the slices of the sliced tiles in a fixed order (bitwise reproducible, no atomics), then alpha / beta.
// partials is [tail_splits][tail_tiles][BN][BM]; block (t, q) handles elements 1024 q .. 1024 q + 1023 of tail tile t,
// four consecutive rows of one column per thread, so that every load is 16 bytes per lane and the loads of different
// slices are independent of each other.
template <int BM, int BN>
__global__ void __launch_bounds__(256) reduce_tail_kernel(const float* __restrict__ partials, int tail_splits, int tail_tiles,
                                                          int full_tiles, int tiles_m, int tiles_n, int group_m,
                                                          int column_bands, int64_t M, int64_t N, float alpha, float beta, float* __restrict__ C,
                                                          int64_t ldc, const int* gate, int gate_value, int gate_value_too) {
  static_assert(BM % 4 == 0 && (BM * BN) % 1024 == 0, "tile shape");
  // (two values: the one-launch kernel serves the FP16 candidate of the automatic choice with and without scaling
  // vectors; everyone else passes the same value twice)
  if (!gate_open(gate, gate_value) && !gate_open(gate, gate_value_too)) return;
  int tile_m, tile_n;
  tile_coordinates(full_tiles + blockIdx.x, tiles_m, tiles_n, group_m, column_bands, tile_m, tile_n);
  const int e = (blockIdx.y * 256 + threadIdx.x) * 4;  // element of the tile, stored [n_local][m_local]
  const int64_t m = (int64_t)tile_m * BM + e % BM, n = (int64_t)tile_n * BN + e / BM;
  if (m >= M || n >= N) return;
  const float* src = partials + (int64_t)blockIdx.x * (BM * BN) + e;
  const int64_t slice_stride = (int64_t)tail_tiles * (BM * BN);
  float4 sum = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll 4
  for (int s = 0; s < tail_splits; ++s) {
    const float4 v = *reinterpret_cast<const float4*>(src + s * slice_stride);
    sum.x += v.x, sum.y += v.y, sum.z += v.z, sum.w += v.w;
  }
  const float part[4] = {sum.x, sum.y, sum.z, sum.w};
  float* dst = C + m + n * ldc;
  if (m + 3 < M && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
    typedef float vec4_t __attribute__((ext_vector_type(4)));
    vec4_t out;
    if (beta == 0.0f) {
#pragma unroll
      for (int i = 0; i < 4; ++i) out[i] = alpha * part[i];
    } else {
      const vec4_t c_in = *reinterpret_cast<const vec4_t*>(dst);
#pragma unroll
      for (int i = 0; i < 4; ++i) out[i] = scaled_sum(alpha, part[i], beta, c_in[i]);
    }
    __builtin_nontemporal_store(out, reinterpret_cast<vec4_t*>(dst));
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (m + i < M) store_result(dst + i, (beta == 0.0f) ? alpha * part[i] : scaled_sum(alpha, part[i], beta, dst[i]));
  }
}

}  // namespace ecgemm
