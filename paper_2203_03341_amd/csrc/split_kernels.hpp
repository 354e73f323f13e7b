// Step 1 of the error-corrected SGEMM: element split + repack, HBM-bandwidth bound.
//
// FP16 mode (Eqs. corr-1-1024 .. corr-4-1024):  v16 = toFP16(v),  dv16 = toFP16((v - toFP32(v16)) * 2^11)
// BF16 mode (three exact terms, stands in for the paper's TF32 pair on hardware without a TF32
// matrix instruction):  b0 = toBF16(v), b1 = toBF16(v - b0), b2 = toBF16(v - b0 - b1)
// Conversions round to nearest even (the hardware converts) and saturate: a finite input never
// yields an infinite part.  An infinite input keeps only its high part.  SplitKind lists the other
// splits the kernels can produce for the paper's comparison methods.
//
// Output layout ("fragment order"), 16-bit elements:
//     packed[row_block][k_step][part][lane][8],  row_block = r / 32, k_step = k / 16,
//     lane = ((k % 16) / 8) * 32 + r % 32, element = k % 8
// so that one 1 KiB chunk is exactly what the 64 lanes of a wave feed to one
// v_mfma_f32_32x32x16 operand, and a block tile is a run of whole chunks.  Rows are padded to
// kRowPad and depth to kDepthPad with zeros, which makes every tile of the product kernel full.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ecgemm {

constexpr int kRowPad = 256;
constexpr int kDepthPad = 32;
constexpr int kChunkElems = 512;  // 64 lanes x 8 elements

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short ushort8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float saturate_finite(float v, float limit) {
  // leaves Inf and NaN alone, clamps everything finite into [-limit, limit]
  return (__builtin_fabsf(v) <= 3.402823466e+38f) ? __builtin_fminf(__builtin_fmaxf(v, -limit), limit) : v;
}

// What a value is split into.  The first two are the method; the others exist to reproduce the paper's
// comparisons (Markidis' unscaled residual, and plain conversion with no residual at all).
enum SplitKind {
  kSplitFp16Scaled = 0,    // v16, (v - v16) * 2^11      Eqs. corr-elm-1, corr-elm-2-1024 ("halfhalf")
  kSplitBf16x3 = 1,        // three exact BF16 terms
  kSplitFp16Unscaled = 2,  // v16, v - v16               Eqs. corr-elm-1, corr-elm-2 ("Markidis' halfhalf")
  kSplitFp16Plain = 3,     // v16 only
  kSplitBf16Plain = 4,     // toBF16(v) only
  kSplitFp32 = 5           // v itself, repacked for the FP32 matrix instruction (the baseline the method is set against)
};

// 1 KiB chunks per (32 rows x 16 k).  kSplitFp32 has two as well, but they are the two 8-deep halves of the k step,
// 32 rows x 8 k of 32-bit elements each, not two parts of every element.
__host__ __device__ constexpr int parts_of_split(int kind) {
  return kind == kSplitBf16x3 ? 3 : (kind == kSplitFp16Plain || kind == kSplitBf16Plain) ? 1 : 2;
}
__host__ __device__ constexpr bool split_is_bf16(int kind) { return kind == kSplitBf16x3 || kind == kSplitBf16Plain; }

constexpr float kBf16Max = 3.3895313892515355e+38f;  // largest finite BF16

// 2^e for a per-row scaling exponent e in [-126, 127]
__device__ __forceinline__ float row_scale_factor(int e) { return __builtin_bit_cast(float, (unsigned)(e + 127) << 23); }

template <int KIND>
struct Splitter {
  static constexpr int kParts = parts_of_split(KIND);
  __device__ static __forceinline__ void split(float v, unsigned short (&out)[kParts]) {
    if constexpr (!split_is_bf16(KIND)) {
      const _Float16 hi = (_Float16)saturate_finite(v, 65504.0f);
      out[0] = __builtin_bit_cast(unsigned short, hi);
      if constexpr (kParts == 2) {
        float residual = v - (float)hi;                                  // exact
        // exact; a residual beyond +-32 saturates the low part anyway, and cutting it there first keeps the
        // multiplication from overflowing FP32 for inputs of magnitude 2^117 and more
        if constexpr (KIND == kSplitFp16Scaled) residual = saturate_finite(residual, 32.0f) * 2048.0f;
        const _Float16 lo = (_Float16)saturate_finite(residual, 65504.0f);
        // an infinite input keeps only its high part (selected on the bits: no branch around the conversion)
        const unsigned short keep = (__builtin_bit_cast(unsigned short, hi) & 0x7fffu) == 0x7c00u ? 0u : 0xffffu;
        out[1] = __builtin_bit_cast(unsigned short, lo) & keep;
      }
    } else {
      const __bf16 b0 = (__bf16)saturate_finite(v, kBf16Max);
      out[0] = __builtin_bit_cast(unsigned short, b0);
      if constexpr (kParts == 3) {
        const float r1 = v - (float)b0;
        const __bf16 b1 = (__bf16)saturate_finite(r1, kBf16Max);
        const float r2 = r1 - (float)b1;
        const __bf16 b2 = (__bf16)saturate_finite(r2, kBf16Max);
        const unsigned short keep = (out[0] & 0x7fffu) == 0x7f80u ? 0u : 0xffffu;  // infinite input: high part only
        out[1] = __builtin_bit_cast(unsigned short, b1) & keep;
        out[2] = __builtin_bit_cast(unsigned short, b2) & keep;
      }
    }
  }
};

// What the automatic mode choice needs to know about an operand: how much of it the FP16 pair loses, and how many
// elements of a row carry its weight.  Per thread, then per block: the sums of (x - (v16 + dv16 2^-11))^2, of x^2 and
// of |x| over the elements handled, in FP64.
struct SplitStats {
  double err2 = 0.0, norm2 = 0.0, abs1 = 0.0;
};
constexpr int kStatsPerBlock = 3;  // doubles a block leaves: err2, norm2, abs1

// Binary exponent of a non-zero finite value, FP32 subnormals counted as -127; INT_MIN for zero, infinities and NaN
// (the elements that the per-row scaling exponents ignore).
__device__ __forceinline__ int finite_exponent(float v) {
  const unsigned bits = __builtin_bit_cast(unsigned, v) & 0x7fffffffu;
  return (bits != 0 && bits < 0x7f800000u) ? (int)(bits >> 23) - 127 : -0x7fffffff - 1;
}
// max of finite_exponent over eight values (before any pre-scaling)
__device__ __forceinline__ int finite_exponent8(const float (&v)[8]) {
  int hi = -0x7fffffff - 1;
#pragma unroll
  for (int e = 0; e < 8; ++e) hi = max(hi, finite_exponent(v[e]));
  return hi;
}
// Four neighbouring lanes hold values of one row: the row's maximum goes to row_max[r] from the first of them.
__device__ __forceinline__ void publish_row_exponent_of_4_lanes(int* __restrict__ row_max, int64_t r, bool row_exists, int hi) {
  hi = max(hi, __shfl_xor(hi, 1, 64));
  hi = max(hi, __shfl_xor(hi, 2, 64));
  if ((threadIdx.x & 3) == 0 && row_exists && hi != -0x7fffffff - 1) atomicMax(&row_max[r], hi);
}

// Writes the eight consecutive-k values `v` of row r (global indices) to their place in `packed`.
template <int KIND, bool STATS = false>
__device__ __forceinline__ void store_fragment_row(unsigned short* __restrict__ packed, int64_t k_steps_total,
                                                   int64_t r, int64_t k, const float (&v)[8], SplitStats* stats = nullptr) {
  if constexpr (KIND == kSplitFp32) {
    // v_mfma_f32_32x32x2_f32 takes one float per lane: lane l supplies row l % 32 and k = l / 32 of a 2-deep step.
    // A 1 KiB chunk holds four such steps, 16 bytes per lane: element k % 8 of the row goes to lane
    // (k % 2) * 32 + r % 32, float (k % 8) / 2.
    typedef float native4 __attribute__((ext_vector_type(4)));
    const int64_t chunk_index = ((r >> 5) * k_steps_total + (k >> 4)) * 2 + ((k >> 3) & 1);
    float* chunk = reinterpret_cast<float*>(packed) + chunk_index * (kChunkElems / 2) + (int)(r & 31) * 4;
    native4 even = {v[0], v[2], v[4], v[6]}, odd = {v[1], v[3], v[5], v[7]};
    *reinterpret_cast<native4*>(chunk) = even;
    *reinterpret_cast<native4*>(chunk + 32 * 4) = odd;
    return;
  }
  constexpr int NP = Splitter<KIND>::kParts;
  ushort8_t parts[NP];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    unsigned short s[NP];
    Splitter<KIND>::split(v[e], s);
#pragma unroll
    for (int p = 0; p < NP; ++p) parts[p][e] = s[p];
    if constexpr (STATS && KIND == kSplitFp16Scaled) {
      const float kept = (float)__builtin_bit_cast(_Float16, s[0]) + (float)__builtin_bit_cast(_Float16, s[1]) * 0x1p-11f;
      const double lost = (double)v[e] - (double)kept, x = (double)v[e];
      stats->err2 += lost * lost;
      stats->norm2 += x * x;
      stats->abs1 += __builtin_fabs(x);
    }
  }
  const int64_t row_block = r >> 5, k_step = k >> 4;
  const int lane = (int)((k >> 3) & 1) * 32 + (int)(r & 31);
  unsigned short* chunk = packed + ((row_block * k_steps_total + k_step) * NP) * kChunkElems + lane * 8;
#pragma unroll
  for (int p = 0; p < NP; ++p) *reinterpret_cast<ushort8_t*>(chunk + p * kChunkElems) = parts[p];
}

// One operand to split: X = op(src), rows x depth, into `packed`.
struct SplitJob {
  const float* src;
  int64_t ld, rows, depth;
  int64_t k_steps_total;      // padded depth / 16
  float prescale;             // a power of two chosen by the caller (1 by default): exact
  const int* row_log2_scale;  // optional per-row exponents, applied on top of prescale
  unsigned short* packed;
  unsigned fast_tiles;        // tiles along the direction in which the blocks are numbered first
  unsigned blocks;
  int variant;                // SplitVariant
  // Automatic mode choice only, else null: block b leaves its SplitStats at stats[kStatsPerBlock b ...]
  double* stats;
  // Automatic mode choice only, else null: the kernel does nothing unless *gate == gate_value
  const int* gate;
  int gate_value;
  // Automatic mode choice only, else null (STATS kernels): row_max[r] is raised to the largest finite_exponent of row
  // r's elements as they are in `src` (the caller has set every entry to INT_MIN), so that the scaling exponents of
  // ecgemm_row_scales need no pass of their own
  int* row_max;
};

// Sums the threads' statistics over the block in a fixed order and stores them (all 256 threads call this).
__device__ __forceinline__ void store_block_stats(const SplitStats& mine, double* __restrict__ out, double* scratch12) {
  double e = mine.err2, n = mine.norm2, a = mine.abs1;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    e += __shfl_xor(e, d, 64);
    n += __shfl_xor(n, d, 64);
    a += __shfl_xor(a, d, 64);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) scratch12[3 * wave] = e, scratch12[3 * wave + 1] = n, scratch12[3 * wave + 2] = a;
  __syncthreads();
  if (threadIdx.x < kStatsPerBlock)
    out[threadIdx.x] = (scratch12[threadIdx.x] + scratch12[3 + threadIdx.x]) + (scratch12[6 + threadIdx.x] + scratch12[9 + threadIdx.x]);
}
enum SplitVariant { kSplitKContiguousVec = 0, kSplitKContiguous = 1, kSplitRContiguous = 2, kSplitRContiguousWide = 3 };

// Source with k contiguous, X(r, k) = src[k + r * ld], base and leading dimension multiples of 16 bytes.  One block:
// 64 rows x 32 k, 256 threads, thread t handles row t / 4 and the 8 values starting at k = 8 * (t % 4), two 16-byte
// loads.  Blocks are numbered with the k tile fastest.
template <int KIND, bool STATS = false>
__device__ __forceinline__ void split_block_k_contiguous_vec(const SplitJob& job, unsigned block, SplitStats* stats = nullptr) {
  const int t = threadIdx.x;
  const int64_t r = (int64_t)(block / job.fast_tiles) * 64 + (t >> 2);
  const int64_t k = (int64_t)(block % job.fast_tiles) * 32 + (t & 3) * 8;
  float prescale = job.prescale;
  if (job.row_log2_scale != nullptr && r < job.rows) prescale *= row_scale_factor(job.row_log2_scale[r]);
  const float* src = job.src;
  float v[8];
  if (r < job.rows && k + 8 <= job.depth) {
    const float4 lo = *reinterpret_cast<const float4*>(src + r * job.ld + k);
    const float4 hi = *reinterpret_cast<const float4*>(src + r * job.ld + k + 4);
    v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
    v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (r < job.rows && k + e < job.depth) ? src[r * job.ld + k + e] : 0.0f;
  }
  if constexpr (STATS)
    if (job.row_max != nullptr) publish_row_exponent_of_4_lanes(job.row_max, r, r < job.rows, finite_exponent8(v));
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] *= prescale;
  store_fragment_row<KIND, STATS>(job.packed, job.k_steps_total, r, k, v, stats);
}

// Source with k contiguous, any alignment (rows that do not start on 16 bytes: lda = 5003).  One block: 64 rows x
// 64 k, read with lanes along k, so that a wave instruction fetches one 256-byte run instead of 4 bytes from each of
// 16 rows, and handed to the row's thread through LDS (`tile`, 64 x 65 floats; the odd stride keeps both the writes
// and the reads free of bank conflicts).  Blocks are numbered with the k tile fastest.
template <int KIND, bool STATS = false>
__device__ __forceinline__ void split_block_k_contiguous_staged(const SplitJob& job, unsigned block, float* tile, SplitStats* stats = nullptr) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t r0 = (int64_t)(block / job.fast_tiles) * 64, k0 = (int64_t)(block % job.fast_tiles) * 64;
  const float* src = job.src;
  const int64_t k_in = k0 + lane;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int row = 4 * j + wave;
    const int64_t r = r0 + row;
    tile[row * 65 + lane] = (r < job.rows && k_in < job.depth) ? src[r * job.ld + k_in] : 0.0f;
  }
  __syncthreads();
  const int64_t r = r0 + (t >> 2);
  float prescale = job.prescale;
  if (job.row_log2_scale != nullptr && r < job.rows) prescale *= row_scale_factor(job.row_log2_scale[r]);
  int row_hi = -0x7fffffff - 1;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int k_local = half * 32 + (t & 3) * 8;
    if (k0 + k_local >= job.k_steps_total * 16) break;  // the padded depth is a multiple of 32, not of 64
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[(t >> 2) * 65 + k_local + e];
    if constexpr (STATS) row_hi = max(row_hi, finite_exponent8(v));
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= prescale;
    store_fragment_row<KIND, STATS>(job.packed, job.k_steps_total, r, k0 + k_local, v, stats);
  }
  if constexpr (STATS)
    if (job.row_max != nullptr) publish_row_exponent_of_4_lanes(job.row_max, r, r < job.rows, row_hi);
}

// Source with r contiguous: X(r, k) = src[r + k * ld], any alignment.  One block: 64 rows x 32 k.  Lanes run along r,
// so a thread reads the 8 consecutive-k values of its row directly and each read instruction of a wave is a 256-byte
// run.  Blocks are numbered with the row tile fastest: neighbours in the launch order read neighbouring runs.
template <int KIND, bool STATS = false>
__device__ __forceinline__ void split_block_r_contiguous(const SplitJob& job, unsigned block, SplitStats* stats = nullptr) {
  const int t = threadIdx.x;
  const int64_t r = (int64_t)(block % job.fast_tiles) * 64 + (t & 63);
  const int64_t k = (int64_t)(block / job.fast_tiles) * 32 + (t >> 6) * 8;
  float prescale = job.prescale;
  if (job.row_log2_scale != nullptr && r < job.rows) prescale *= row_scale_factor(job.row_log2_scale[r]);
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (r < job.rows && k + e < job.depth) ? job.src[r + (k + e) * job.ld] : 0.0f;
  if constexpr (STATS) {
    const int hi = finite_exponent8(v);
    if (job.row_max != nullptr && r < job.rows && hi != -0x7fffffff - 1) atomicMax(&job.row_max[r], hi);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] *= prescale;
  store_fragment_row<KIND, STATS>(job.packed, job.k_steps_total, r, k, v, stats);
}

// Source with r contiguous, base and leading dimension multiples of 16 bytes.  One block: 256 rows x 32 k through
// 32 KiB of LDS (`tile`).  A wave reads one k line of 256 rows per instruction (1 KiB runs, 16 bytes per lane); after
// the barrier thread t owns row t and picks its 8-value groups out of LDS along k (lanes on consecutive words: no bank
// conflicts).  5.4 TB/s at 16384^2 against 3.9 TB/s for the 64-row kernel above.
template <int KIND, bool STATS = false>
__device__ __forceinline__ void split_block_r_contiguous_wide(const SplitJob& job, unsigned block, float* tile, SplitStats* stats = nullptr) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t r0 = (int64_t)(block % job.fast_tiles) * 256, k0 = (int64_t)(block / job.fast_tiles) * 32;
  const float* src = job.src;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int kk = wave + 4 * j;
    const int64_t k = k0 + kk, r = r0 + 4 * lane;
    float4 x = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (k < job.depth) {
      if (r + 4 <= job.rows) {
        x = *reinterpret_cast<const float4*>(src + r + k * job.ld);
      } else {
        if (r + 0 < job.rows) x.x = src[r + 0 + k * job.ld];
        if (r + 1 < job.rows) x.y = src[r + 1 + k * job.ld];
        if (r + 2 < job.rows) x.z = src[r + 2 + k * job.ld];
      }
    }
    *reinterpret_cast<float4*>(&tile[kk * 256 + 4 * lane]) = x;
  }
  __syncthreads();
  float prescale = job.prescale;
  if (job.row_log2_scale != nullptr && r0 + t < job.rows) prescale *= row_scale_factor(job.row_log2_scale[r0 + t]);
  int row_hi = -0x7fffffff - 1;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[(8 * g + e) * 256 + t];
    if constexpr (STATS) row_hi = max(row_hi, finite_exponent8(v));
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= prescale;
    store_fragment_row<KIND, STATS>(job.packed, job.k_steps_total, r0 + t, k0 + 8 * g, v, stats);
  }
  if constexpr (STATS)
    if (job.row_max != nullptr && r0 + t < job.rows && row_hi != -0x7fffffff - 1) atomicMax(&job.row_max[r0 + t], row_hi);
}

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  For a source whose rows are not aligned to
// cache lines, block b of n takes the tile at this position, so that every XCD works through one contiguous run of the
// tile list: neighbouring tiles, whose rows share a cache line at their common edge, then meet in one L2 instead of
// being fetched by two (FETCH_SIZE was 45 % above the source's size at lda = 5003; the split of that operand is 10 %
// faster).  The aligned kernels keep the plain order: for them the runs cost up to 7 % (fewer neighbouring DRAM pages
// open at a time).
__device__ __forceinline__ unsigned xcd_run_position(unsigned b, unsigned n) {
  const unsigned per = n / 8, rem = n % 8, x = b % 8;
  return x * per + (x < rem ? x : rem) + b / 8;
}

// Whether a gated kernel is to run (automatic mode choice: both candidates' kernels are enqueued, and the ones of the
// mode not chosen return at once).
__device__ __forceinline__ bool gate_open(const int* gate, int gate_value) {
  return gate == nullptr || *gate == gate_value;
}

// One operand per launch; VARIANT is fixed at compile time so that only the kernels that stage through LDS hold any.
// STATS (automatic mode choice): block b also leaves its SplitStats at job.stats[2 b], [2 b + 1].
template <int KIND, int VARIANT, bool STATS = false>
__global__ void __launch_bounds__(256) split_kernel(const SplitJob job) {
  if (!gate_open(job.gate, job.gate_value)) return;
  SplitStats stats;
  if constexpr (VARIANT == kSplitRContiguousWide) {
    __shared__ float tile[32 * 256];
    split_block_r_contiguous_wide<KIND, STATS>(job, blockIdx.x, tile, &stats);
  } else if constexpr (VARIANT == kSplitRContiguous) {
    split_block_r_contiguous<KIND, STATS>(job, blockIdx.x, &stats);
  } else if constexpr (VARIANT == kSplitKContiguousVec) {
    split_block_k_contiguous_vec<KIND, STATS>(job, blockIdx.x, &stats);
  } else {
    __shared__ float tile[64 * 65];
    split_block_k_contiguous_staged<KIND, STATS>(job, xcd_run_position(blockIdx.x, job.blocks), tile, &stats);
  }
  if constexpr (STATS) {
    __shared__ double sums[12];
    // (indexed by the launch's block number: the choice adds all blocks of an operand, in that order)
    store_block_stats(stats, job.stats + kStatsPerBlock * (size_t)blockIdx.x, sums);
  }
}

// Both operands of a product in one launch, for small operands where a launch costs more than the work: blocks
// 0 .. a.blocks - 1 split A, the rest split B.
template <int KIND, bool STATS = false>
__global__ void __launch_bounds__(256) split_pair_kernel(const SplitJob a, const SplitJob b) {
  if (!gate_open(a.gate, a.gate_value)) return;
  __shared__ float tile[32 * 256];
  const bool second = blockIdx.x >= a.blocks;  // block-uniform
  const SplitJob& job = second ? b : a;
  const unsigned block = second ? blockIdx.x - a.blocks : blockIdx.x;
  SplitStats stats;
  switch (job.variant) {
    case kSplitRContiguousWide: split_block_r_contiguous_wide<KIND, STATS>(job, block, tile, &stats); break;
    case kSplitRContiguous: split_block_r_contiguous<KIND, STATS>(job, block, &stats); break;
    case kSplitKContiguousVec: split_block_k_contiguous_vec<KIND, STATS>(job, block, &stats); break;
    default: split_block_k_contiguous_staged<KIND, STATS>(job, xcd_run_position(block, job.blocks), tile, &stats); break;
  }
  if constexpr (STATS) {
    __shared__ double sums[12];
    store_block_stats(stats, job.stats + kStatsPerBlock * (size_t)block, sums);
  }
}

}  // namespace ecgemm
