// The paper's own arrangement of the method for one block (section "Incorporating our method into CUTLASS", last
// paragraph): the block reads FP32 tiles of A and B, forms the low-precision parts in registers (Eqs. corr-1-1024 ..
// corr-4-1024, or the three BF16 terms) and multiplies them right away; no split pass over the operands, no packed
// copies in HBM: one launch (two where a deep product of few tiles is cut into slices of the depth, a block each,
// whose partial sums reduce_tail_kernel adds up).  Every block that touches a tile of A splits it again (N / 64 times per
// element), so this pays where launches and latencies, not arithmetic, decide the time: small products.
//
// One block: TILE x TILE of C over the whole depth of the product, TILE = 64 or 32, made by eight waves that fetch and
// split and, next to them on the same SIMDs, one wave per 32 x 32 of the tile that multiplies (one v_mfma_f32_32x32x16
// accumulator pair): 12 or 9 waves.  A chain of dependent matrix instructions leaves its wave waiting most of the
// time; with the two roles in different waves the hardware fills that time with the other waves' split, and with two
// splitting waves per SIMD one of them can issue while the other waits.  Same term order and same accumulator
// discipline as product_kernel.hpp, so an element is summed in the same order as in an unsliced tile there; the
// fragments lie in LDS as they do there except for a rotation of the rows (fused_lds_slot).  Small tiles are what
// make a small product many blocks, and what bounds a block is its split work, (TILE + TILE) x K elements: 512^3 is
// 64 blocks of 64 x 64 or 256 of 32 x 32 with half the work each, one per compute unit.  The host picks 32 while that
// still leaves compute units idle.
//
// Depth is walked in chunks of 64.  The 512 splitting threads fetch the chunk's TILE x 64 values of op(A) and of
// op(B), TILE / 8 of each per thread, with the lanes of a wave along whichever index is contiguous in memory
// (FusedLayout); the values of the next kFusedRing chunks are in flight in registers while the current one is split
// and written to LDS in fragment order (two buffers, one barrier per chunk), where the multiplying waves pick it up.
// The split takes a short form (FastSplit, 3.5 to 7.5 vector instructions per element) whenever every value a wave
// holds is ordinary, and Splitter, which saturates and handles infinities and NaN, otherwise; both give the same
// bits on the values the short form accepts.  Measured on single blocks, what bounded a chunk in turn was: the
// instruction stream of one splitting wave per SIMD (hence eight waves, a loop for the bulk of the depth without
// conditions that are the same for the whole block, loads whose addresses are a scalar base plus a constant lane
// offset), bank conflicts of the LDS writes of k-contiguous operands (hence the rotation), and the trip of the
// fragments from LDS in front of each chunk's first matrix instruction (hence the two half-chunk register sets of
// the multiplying waves).
#pragma once
#include "product_kernel.hpp"

namespace ecgemm {

// How the V = TILE / 8 values per thread and chunk are laid over one operand's TILE rows x 64 k (X(r, k): op(A)(m, k)
// or op(B)(k, n) with r = n), wave w, lane l:
//   kFusedRows      r contiguous, X(r, k) = src[r + k ld]: row l % TILE, the V consecutive k from 8 w + V (l / TILE)
//   kFusedDepth     k contiguous, X(r, k) = src[k + r ld]: k = l, rows V w .. V w + V - 1
//   kFusedDepthVec  k contiguous, base and ld multiples of 16 bytes, K a multiple of 4: the four values k = 4 (l % 16) ..
//                   + 3 of rows w + 8 (l / 16) + 32 j, j = 0 .. V / 4 - 1, one 16-byte load each (rows 8 apart: with
//                   the rotation of fused_lds_slot the 64 lanes of a write then go to 64 different places of a bank period)
enum FusedLayout { kFusedRows = 0, kFusedDepth = 1, kFusedDepthVec = 2 };
// Chunks in flight in registers (the loop is unrolled by this: a register ring is indexed statically).  Four and six
// instead of two measured slower at every size (1024^3: 18.9 and 29.6 against 18.1 us).
constexpr int kFusedRing = 2;
constexpr int kFusedSplitWaves = 8;  // two per SIMD: one wave alone cannot issue the split's instructions fast enough

struct FusedParams {
  const float* A;  // device, column-major, as passed to ecgemm_sgemm
  const float* B;
  int64_t lda, ldb;
  float prescale_a, prescale_b;  // powers of two applied before the split (1 by default)
  int64_t M, N, K, ldc;
  int tiles_m, tiles_n;
  float alpha, beta, out_scale;
  // per-row / per-column pre-scaling as in ProductParams (both null, or both set)
  const int* row_log2_scale;  // device, M entries
  const int* col_log2_scale;  // device, N entries
  float* C;
  // k_slices > 1 (deep products of small matrices, where whole tiles would leave most compute units idle): block b
  // takes tile b % tiles over chunks_per_slice 64-deep chunks from chunk (b / tiles) chunks_per_slice on and leaves
  // its sums, before alpha / beta, in partials[b / tiles][b % tiles][n][m] for reduce_tail_kernel, as the product
  // kernels do for their sliced tiles.  k_slices == 1: every block the whole depth, nothing written but C.
  int k_slices, chunks_per_slice;
  float* partials;
  // Automatic mode choice only, else null: the kernel runs without the scaling vectors if *gate == gate_value, with
  // them if *gate == gate_value_scaled, and does nothing otherwise
  const int* gate;
  int gate_value, gate_value_scaled;
};

// The split for values that need no care, two at a time (the two 16-bit results of a part share a register: out[q]
// holds part q of v0 in its low half and of v1 in its high half).  It has none of Splitter's clamps and masks; on a
// value whose high part comes out finite both give the same bits: the high part is then at most the largest finite
// number of the format whether or not the value was clamped to it first, the residuals are at most half a unit of
// its last place, far inside the range of the low parts, and nothing is masked.  A value that Splitter treats
// differently (beyond the format's range, where it saturates; infinite; NaN) shows as a high part that is infinite or
// NaN, which high_parts_finite() finds on the packed registers.
typedef float fused_float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 fused_half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 fused_bf16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned short fused_ushort2_t __attribute__((ext_vector_type(2)));
template <int KIND>
struct FastSplit {
  static constexpr int kParts = parts_of_split(KIND);
  // `scaled0`, `scaled1`: the same two values times 2^11 (used by kSplitFp16Scaled only), so that the scaled residual
  // is one fused multiply-add on the packed high part: hi * -2^11 + v * 2^11 = (v - hi) * 2^11, exact like the
  // two-step form (v * 2^11 overflows only for values whose high part is not finite, which do not end up here).
  __device__ static __forceinline__ void split2(float v0, float v1, float scaled0, float scaled1, unsigned (&out)[kParts]) {
    if constexpr (!split_is_bf16(KIND)) {
      const fused_half2_t hi = __builtin_convertvector(fused_float2_t{v0, v1}, fused_half2_t);
      out[0] = __builtin_bit_cast(unsigned, hi);
      if constexpr (KIND == kSplitFp16Scaled) {
        // (each rounded to FP16 by itself: the multiply-add then delivers its result as one half of the register)
        const fused_half2_t lo = {(_Float16)__builtin_fmaf((float)hi[0], -2048.0f, scaled0), (_Float16)__builtin_fmaf((float)hi[1], -2048.0f, scaled1)};
        out[1] = __builtin_bit_cast(unsigned, lo);
      } else if constexpr (kParts == 2) {
        const fused_float2_t residual = {v0 - (float)hi[0], v1 - (float)hi[1]};  // exact
        out[1] = __builtin_bit_cast(unsigned, __builtin_convertvector(residual, fused_half2_t));
      }
    } else {
      const fused_bf16x2_t b0 = __builtin_convertvector(fused_float2_t{v0, v1}, fused_bf16x2_t);
      out[0] = __builtin_bit_cast(unsigned, b0);
      if constexpr (kParts == 3) {
        const fused_float2_t r1 = {v0 - (float)b0[0], v1 - (float)b0[1]};
        const fused_bf16x2_t b1 = __builtin_convertvector(r1, fused_bf16x2_t);
        const fused_float2_t r2 = {r1[0] - (float)b1[0], r1[1] - (float)b1[1]};
        out[1] = __builtin_bit_cast(unsigned, b1);
        out[2] = __builtin_bit_cast(unsigned, __builtin_convertvector(r2, fused_bf16x2_t));
      }
    }
  }
  // true if none of the 2 W high parts in `words[..][0]` is infinite or NaN
  template <int W>
  __device__ static __forceinline__ bool high_parts_finite(const unsigned (&words)[W][kParts]) {
    const unsigned magnitude = 0x7fff7fffu;
    fused_ushort2_t most = {0, 0};
#pragma unroll
    for (int e = 0; e < W; ++e)
      most = __builtin_elementwise_max(most, __builtin_bit_cast(fused_ushort2_t, words[e][0] & magnitude));
    const unsigned short exponent_all_ones = split_is_bf16(KIND) ? 0x7f80 : 0x7c00;
    return most[0] < exponent_all_ones && most[1] < exponent_all_ones;
  }
};

// Where element (row, k) of a chunk lies in an operand's region of LDS, part 0 (bytes): fragment order, [row / 32]
// [k step][part] blocks of 1 KiB, each two halves (k % 16 / 8) of 32 rows x 16 bytes, except that the rows of a half
// are rotated by 2 (k step) + half places.  A fragment read takes a whole half either way.  The rotation is for
// the writes of the k-contiguous layouts, where the lanes of one instruction hold few rows and many k: without it
// their addresses differ by multiples of 512 bytes and meet in the same banks, eight at a time.
__device__ __forceinline__ int fused_lds_rotation(int k) { return (k >> 3) & 7; }
template <int NP>
__device__ __forceinline__ int fused_lds_slot(int row, int k) {
  return ((row >> 5) * 4 + (k >> 4)) * NP * 1024 + ((k >> 3) & 1) * 512 + (((row & 31) + fused_lds_rotation(k)) & 31) * 16 + (k & 7) * 2;
}

// One operand of the block: where this thread's V values per chunk come from and where their parts go.
template <int KIND, int LAYOUT, int TILE>
struct FusedOperand {
  static_assert(TILE == 64 || TILE == 32, "tile sizes");
  static constexpr int NP = parts_of_split(KIND);
  static constexpr int V = TILE / kFusedSplitWaves;                                      // values per thread and chunk
  static constexpr int ROWS = LAYOUT == kFusedRows ? 1 : LAYOUT == kFusedDepth ? V : V / 4;  // rows this thread holds values of
  static constexpr int PER_ROW = V / ROWS;                                               // consecutive k per row
  static constexpr int REGION_BYTES = (TILE / 32) * 4 * NP * 1024;  // a chunk of one operand in LDS: [row block][k step][part] x 1 KiB
  static constexpr int LOADS = LAYOUT == kFusedDepthVec ? ROWS : V;  // load instructions per thread and chunk
  static constexpr int64_t kLargestShortLd = (int64_t)1 << 23;       // up to here every value of a chunk lies within 2^32 bytes of its first

  // Addresses are a part that is the same for the whole wave plus a small per-lane offset wherever the layout allows
  // it, which leaves the address arithmetic to the scalar unit.  A row beyond the matrix reads the last row instead
  // (its values end up in rows or columns of the tile that are never stored).
  const float* tile;           // &X(first row of the tile, 0)
  const float* row_ptr[ROWS];  // &X(row, 0) for each of the thread's rows
  unsigned lane_offset;        // kFusedRows: the lane's row within the tile; kFusedDepth: the lane's k within the chunk
  float factor[ROWS];          // the handle's pre-scaling times the row's own
  bool unscaled;               // every factor is 1 (the same for the whole block)
  int64_t ld, K;
  int k_here;                  // k within the chunk of the thread's first value
  // byte offset within the operand's region, part 0, of the thread's first value (kFusedRows), of the first value of
  // each of its rows (kFusedDepthVec); kFusedDepth: of row 0 at the thread's k, before the rotation
  int lds_offset[LAYOUT == kFusedDepthVec ? ROWS : 1];
  int first_row;               // within the tile
  // A whole chunk, when ld <= kLargestShortLd: load i reads at &X(first row of the tile, 64 c) + offset[i] bytes, an
  // address that is the same for the wave plus 32 bits per lane that never change, so a chunk's loads need no
  // address arithmetic at all.  (kFusedDepth: a wave's rows are the same for all its lanes, row_ptr is not a vector
  // and serves as it is.)
  unsigned offset[LAYOUT == kFusedDepth ? 1 : LOADS];
  int64_t chunk_bytes;         // from one chunk's first value to the next one's

  __device__ __forceinline__ void init(const float* src, int64_t ld_, int64_t rows, int64_t K_, int64_t tile_row0, float prescale,
                                       const int* log2_scale, int lane, int wave) {
    ld = ld_, K = K_;
    unscaled = prescale == 1.0f && log2_scale == nullptr;
    const int rows_here = (int)(rows - tile_row0 < TILE ? rows - tile_row0 : TILE);  // >= 1
    tile = LAYOUT == kFusedRows ? src + tile_row0 : src + tile_row0 * ld;
    if constexpr (LAYOUT == kFusedRows) {
      first_row = lane % TILE, k_here = (64 / kFusedSplitWaves) * wave + V * (lane / TILE);
      lane_offset = (unsigned)(first_row < rows_here ? first_row : rows_here - 1);
    } else if constexpr (LAYOUT == kFusedDepth) {
      first_row = V * wave, k_here = lane;
      lane_offset = (unsigned)lane;
    } else {
      first_row = wave + 8 * (lane >> 4), k_here = 4 * (lane & 15);
      lane_offset = 0;
    }
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const int row = first_row + (LAYOUT == kFusedDepthVec ? 32 * j : j);
      const int row_clamped = row < rows_here ? row : rows_here - 1;
      row_ptr[j] = tile + (LAYOUT == kFusedRows ? (int64_t)row_clamped : row_clamped * ld);
      factor[j] = prescale;
      if (log2_scale != nullptr) factor[j] *= row_scale_factor(log2_scale[tile_row0 + row_clamped]);
    }
    const bool short_ld = ld <= kLargestShortLd;  // else `offset` is not used
    chunk_bytes = LAYOUT == kFusedRows ? 256 * ld : 256;
    offset[0] = 0;
    if constexpr (LAYOUT != kFusedDepth) {
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        if constexpr (LAYOUT == kFusedRows) {
          offset[i] = short_ld ? (unsigned)(((k_here + i) * ld + lane_offset) * 4) : 0u;
        } else {
          const int row = first_row + 32 * i;
          const int row_clamped = row < rows_here ? row : rows_here - 1;
          offset[i] = short_ld ? (unsigned)((row_clamped * ld + k_here) * 4) : 0u;
        }
      }
    }
    if constexpr (LAYOUT == kFusedRows) {
      static_assert(V <= 8, "a thread's values lie in one half of a k step");
      lds_offset[0] = fused_lds_slot<NP>(first_row, k_here);
    } else if constexpr (LAYOUT == kFusedDepthVec) {
#pragma unroll
      for (int j = 0; j < ROWS; ++j) lds_offset[j] = fused_lds_slot<NP>(first_row + 32 * j, k_here);
    } else {
      static_assert(V <= 32, "a thread's rows lie in one block of 32");
      lds_offset[0] = (k_here >> 4) * NP * 1024 + ((k_here >> 3) & 1) * 512 + (k_here & 7) * 2;
    }
  }

  // Requests the values of chunk c (which exists).  Every address is valid: in the last chunk, k beyond the depth is
  // clamped to the last k (and replaced by zero in deposit()).  No load sits under a condition and both branches
  // issue the same number of loads, so the number in flight is the same on every path: the waits that the compiler
  // places count them.
  __device__ __forceinline__ void fetch(float (&x)[V], int c) const {
    const int64_t chunk_k = (int64_t)c * 64;
    if (chunk_k + 64 <= K) {  // block-uniform
      if constexpr (LAYOUT == kFusedRows) {
        const float* first = tile + chunk_k * ld;
#pragma unroll
        for (int i = 0; i < V; ++i) x[i] = first[(k_here + i) * ld + lane_offset];
      } else if constexpr (LAYOUT == kFusedDepth) {
#pragma unroll
        for (int j = 0; j < V; ++j) x[j] = (row_ptr[j] + chunk_k)[lane_offset];
      } else {
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
          const float4 v = *reinterpret_cast<const float4*>(row_ptr[j] + chunk_k + k_here);
          x[4 * j] = v.x, x[4 * j + 1] = v.y, x[4 * j + 2] = v.z, x[4 * j + 3] = v.w;
        }
      }
    } else {
      const int64_t k0 = chunk_k + k_here;
      if constexpr (LAYOUT == kFusedDepthVec) {
        // K is a multiple of 4 here (the host's condition for this layout): four values that start below K end below it
        const int64_t k = k0 < K ? k0 : K - 4;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
          const float4 v = *reinterpret_cast<const float4*>(row_ptr[j] + k);
          x[4 * j] = v.x, x[4 * j + 1] = v.y, x[4 * j + 2] = v.z, x[4 * j + 3] = v.w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const int64_t k = k0 + e % PER_ROW < K ? k0 + e % PER_ROW : K - 1;
          x[e] = LAYOUT == kFusedRows ? row_ptr[0][k * ld] : row_ptr[e][k];
        }
      }
    }
  }

  // The same for a chunk that lies inside the depth, ld <= kLargestShortLd.
  __device__ __forceinline__ void fetch_whole(float (&x)[V], int c) {
    const char* first = reinterpret_cast<const char*>(tile) + c * chunk_bytes;  // the same for the whole wave
    // (Both halves of every address are kept from the optimizer's view.  It would otherwise carry one 64-bit address
    // per load through the loop in vector registers and advance each of them every chunk, or widen the offsets to 64
    // bits outside the loop and add the base to each with a vector instruction.)
    asm volatile("" : "+s"(first));
    if constexpr (LAYOUT != kFusedDepth) {
#pragma unroll
      for (int i = 0; i < LOADS; ++i) asm volatile("" : "+v"(offset[i]));
    }
    typedef __attribute__((address_space(1))) char global_char_t;  // (what passed through the line above is no longer known to be global memory)
    typedef float plain_float4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(1))) plain_float4_t global_float4_t;
    const global_char_t* chunk = (const global_char_t*)first;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      if constexpr (LAYOUT == kFusedDepth) {
        x[i] = (row_ptr[i] + (int64_t)c * 64)[lane_offset];
      } else if constexpr (LAYOUT == kFusedDepthVec) {
        const plain_float4_t v = *reinterpret_cast<const global_float4_t*>(chunk + offset[i]);
        x[4 * i] = v[0], x[4 * i + 1] = v[1], x[4 * i + 2] = v[2], x[4 * i + 3] = v[3];
      } else {
        x[i] = *reinterpret_cast<const global_float_t*>(chunk + offset[i]);
      }
    }
  }

  // The short split of all V values, with (general == true) or without the multiplication by the scaling factors.
  template <bool GENERAL>
  __device__ __forceinline__ void split_ordinary(const float (&x)[V], unsigned (&words)[V / 2][NP]) const {
#pragma unroll
    for (int e = 0; e < V / 2; ++e) {
      const float v0 = GENERAL ? x[2 * e] * factor[(2 * e) / PER_ROW] : x[2 * e];
      const float v1 = GENERAL ? x[2 * e + 1] * factor[(2 * e + 1) / PER_ROW] : x[2 * e + 1];
      // (times 2^11 after the factor, not with it: a factor of 2^126 is legitimate, 2^137 is not a number)
      FastSplit<KIND>::split2(v0, v1, v0 * 2048.0f, v1 * 2048.0f, words[e]);
    }
  }

  // Splitter on all V values; k beyond the depth (last chunk) counts as zero.
  __device__ __forceinline__ void split_with_care(const float (&x)[V], int c, unsigned (&words)[V / 2][NP]) const {
    const int64_t k0 = (int64_t)c * 64 + k_here;
#pragma unroll
    for (int e = 0; e < V / 2; ++e) {
      unsigned short even[NP], odd[NP];
      Splitter<KIND>::split(k0 + (2 * e) % PER_ROW < K ? x[2 * e] * factor[(2 * e) / PER_ROW] : 0.0f, even);
      Splitter<KIND>::split(k0 + (2 * e + 1) % PER_ROW < K ? x[2 * e + 1] * factor[(2 * e + 1) / PER_ROW] : 0.0f, odd);
#pragma unroll
      for (int q = 0; q < NP; ++q) words[e][q] = (unsigned)even[q] | ((unsigned)odd[q] << 16);
    }
  }

  // Splits the values of chunk c and writes the parts to `region` where the fragment reads expect them.
  __device__ __forceinline__ void deposit(const float (&x)[V], int c, char* region) const {
    unsigned words[V / 2][NP];  // part q of values 2 e and 2 e + 1
    const bool whole = (int64_t)c * 64 + 64 <= K;  // block-uniform
    bool done = false;
    if (whole) {
      if (unscaled)  // block-uniform: no pre-scaling, no scaling vectors: every factor is 1
        split_ordinary<false>(x, words);
      else
        split_ordinary<true>(x, words);
      done = __builtin_amdgcn_ballot_w64(!FastSplit<KIND>::high_parts_finite(words)) == 0;  // wave-uniform
    }
    if (!done) split_with_care(x, c, words);
    write(words, region);
  }

  // The same for a chunk that lies inside the depth, with what is the same for the whole block decided by the caller:
  // GENERAL == false if every factor is 1.
  template <bool GENERAL>
  __device__ __forceinline__ void deposit_whole(const float (&x)[V], int c, char* region) const {
    unsigned words[V / 2][NP];
    split_ordinary<GENERAL>(x, words);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(!FastSplit<KIND>::high_parts_finite(words)) != 0, 0)) {
      // (with a write of its own: joining the two paths in front of one write costs a register copy per word)
      unsigned careful[V / 2][NP];
      split_with_care(x, c, careful);
      write(careful, region);
    } else {
      write(words, region);
    }
  }

  __device__ __forceinline__ void write(const unsigned (&words)[V / 2][NP], char* region) const {
    char* base = region + lds_offset[0];
    typedef unsigned uint4_t __attribute__((ext_vector_type(4)));
    typedef unsigned uint2_t __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int q = 0; q < NP; ++q) {
      if constexpr (LAYOUT == kFusedRows) {  // consecutive k of one row: one or both 8-deep halves of a k step
        if constexpr (V >= 8) {
#pragma unroll
          for (int h = 0; h < V / 8; ++h)
            *reinterpret_cast<uint4_t*>(base + q * 1024 + h * 512) =
                uint4_t{words[4 * h][q], words[4 * h + 1][q], words[4 * h + 2][q], words[4 * h + 3][q]};
        } else {
          static_assert(V == 4, "half of an 8-deep run");
          *reinterpret_cast<uint2_t*>(base + q * 1024) = uint2_t{words[0][q], words[1][q]};
        }
      } else if constexpr (LAYOUT == kFusedDepth) {  // one k of consecutive rows
#pragma unroll
        for (int e = 0; e < V / 2; ++e) {
          const int row = first_row + 2 * e, rotation = fused_lds_rotation(k_here);
          char* block = base + (row >> 5) * 4 * NP * 1024 + q * 1024;
          *reinterpret_cast<unsigned short*>(block + ((row + rotation) & 31) * 16) = (unsigned short)words[e][q];
          *reinterpret_cast<unsigned short*>(block + ((row + 1 + rotation) & 31) * 16) = (unsigned short)(words[e][q] >> 16);
        }
      } else {  // four consecutive k of each of the thread's rows
#pragma unroll
        for (int j = 0; j < ROWS; ++j)
          *reinterpret_cast<uint2_t*>(region + lds_offset[j] + q * 1024) = uint2_t{words[2 * j][q], words[2 * j + 1][q]};
      }
    }
  }
};

constexpr int kFusedSliceChunks = 8;  // chunks of 64 per slice of the depth (see the multiplying waves)
__host__ __device__ constexpr int fused_threads(int tile) { return 64 * (kFusedSplitWaves + (tile / 32) * (tile / 32)); }

template <int METHOD, int LAYOUT_A, int LAYOUT_B, int TILE>
__global__ void __launch_bounds__(fused_threads(TILE), 1) fused_kernel(const FusedParams params) {
  FusedParams p = params;
  if (p.gate != nullptr) {  // the same for every thread of the grid, and before any barrier
    const int choice = *p.gate;
    if (choice == p.gate_value)
      p.row_log2_scale = p.col_log2_scale = nullptr;
    else if (choice != p.gate_value_scaled)
      return;
  }
  constexpr int KIND = split_kind_of(METHOD);
  constexpr bool BF16 = split_is_bf16(KIND);
  constexpr int NP = parts_of_split(KIND), PRODUCTS = products_of(METHOD);
  constexpr int BM = TILE, BN = TILE, K_STEPS = 4;
  typedef FusedOperand<KIND, LAYOUT_A, TILE> OperandA;
  typedef FusedOperand<KIND, LAYOUT_B, TILE> OperandB;
  constexpr int V = OperandA::V;
  constexpr int REGION_BYTES = OperandA::REGION_BYTES, STAGE_BYTES = 2 * REGION_BYTES;
  typedef typename Mfma<BF16 ? kElemBf16 : kElemFp16>::frag_t frag_t;
  __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE_BYTES];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  int tile_index = (int)blockIdx.x, slice = 0;
  if (p.k_slices > 1) {  // the block's slice of the depth is a product of its own from here on
    const int tiles = p.tiles_m * p.tiles_n;
    slice = tile_index / tiles, tile_index -= slice * tiles;
    const int64_t k_begin = (int64_t)slice * p.chunks_per_slice * 64;  // < K: the host makes no empty slices
    const int64_t k_end = k_begin + (int64_t)p.chunks_per_slice * 64;
    p.A += LAYOUT_A == kFusedRows ? k_begin * p.lda : k_begin;
    p.B += LAYOUT_B == kFusedRows ? k_begin * p.ldb : k_begin;
    p.K = (k_end < p.K ? k_end : p.K) - k_begin;
  }
  int tile_m, tile_n;
  tile_coordinates(tile_index, p.tiles_m, p.tiles_n, 4, 1, tile_m, tile_n);
  const int chunks = (int)((p.K + 63) / 64);  // >= 1

  // Every wave of the block passes exactly `chunks` barriers, whichever of the two roles it has: a splitting wave one
  // after each chunk it has written, a multiplying wave one before each chunk it reads.  Chunk c lives in LDS buffer
  // c % 2; a splitting wave writes chunk c + 2 there only after barrier c + 1, which the multiplying waves reach when
  // their reads of chunk c have returned.
  if (wave < kFusedSplitWaves) {
    // ---- splitting waves: chunk c is split into LDS while chunks c + 1 .. c + kFusedRing travel
    OperandA a;
    OperandB b;
    a.init(p.A, p.lda, p.M, p.K, (int64_t)tile_m * BM, p.prescale_a, p.row_log2_scale, lane, wave);
    b.init(p.B, p.ldb, p.N, p.K, (int64_t)tile_n * BN, p.prescale_b, p.col_log2_scale, lane, wave);
    static_assert(kFusedRing % 2 == 0, "a ring slot always meets the same LDS buffer");
    float xa[kFusedRing][V], xb[kFusedRing][V];
    // (a chunk beyond the last is requested again as the last one and never used: in the loop every fetch is
    // unconditional; the scheduling barriers keep the requests of one ring slot together and the slots in order, which
    // is what lets the wait in front of a slot's first use leave the younger slots' loads in flight)
    const int last = chunks - 1;
    static_for<kFusedRing>([&](auto r_c) {
      constexpr int r = decltype(r_c)::value;
      a.fetch(xa[r], r < last ? r : last), b.fetch(xb[r], r < last ? r : last);
      __builtin_amdgcn_sched_barrier(0);
    });
    int c0 = 0;
    // The bulk of the depth: chunks that lie inside it and whose successors in the ring do too, so that nothing in
    // the loop depends on where the depth ends, and what is the same for the whole block (are there scaling factors?)
    // is decided outside it.  Ring slot r holds chunk c0 + r at the top of every loop here.  The loops further down,
    // which decide everything chunk by chunk, are for the calls that cannot take this one.
    auto bulk = [&](auto general_c) {
      constexpr bool GENERAL = decltype(general_c)::value;
      const int whole_chunks = (int)(p.K / 64);
      for (; c0 + 2 * kFusedRing <= whole_chunks; c0 += kFusedRing) {
        static_for<kFusedRing>([&](auto r_c) {
          constexpr int r = decltype(r_c)::value;
          char* stage = lds + (r & 1) * STAGE_BYTES;
          a.template deposit_whole<GENERAL>(xa[r], c0 + r, stage);
          b.template deposit_whole<GENERAL>(xb[r], c0 + r, stage + REGION_BYTES);
          __builtin_amdgcn_sched_barrier(0);
          a.fetch_whole(xa[r], c0 + r + kFusedRing), b.fetch_whole(xb[r], c0 + r + kFusedRing);
          __syncthreads();
        });
      }
      // The last chunks, whose successors in the ring do not exist or are not whole: the same split for those that
      // lie inside the depth, the general one for the last if it does not, and the general fetch for what is left to
      // request.  (Every condition here is the same for the whole block, and every chunk still has its one barrier.)
      while (c0 < chunks) {
        static_for<kFusedRing>([&](auto r_c) {
          constexpr int r = decltype(r_c)::value;
          const int c = c0 + r;
          if (c < chunks) {
            char* stage = lds + (r & 1) * STAGE_BYTES;
            if (c < whole_chunks) {
              a.template deposit_whole<GENERAL>(xa[r], c, stage);
              b.template deposit_whole<GENERAL>(xb[r], c, stage + REGION_BYTES);
            } else {
              a.deposit(xa[r], c, stage);
              b.deposit(xb[r], c, stage + REGION_BYTES);
            }
            if (c + kFusedRing < chunks) a.fetch(xa[r], c + kFusedRing), b.fetch(xb[r], c + kFusedRing);
            __syncthreads();
          }
        });
        c0 += kFusedRing;
      }
    };
    // (kFusedDepth, the layout of last resort, only next to kFusedRows: with one row pointer and one factor per
    // value it leaves no registers for a second copy of the loop next to another depth-contiguous operand)
    if constexpr ((LAYOUT_A != kFusedDepth && LAYOUT_B != kFusedDepth) || LAYOUT_A == kFusedRows || LAYOUT_B == kFusedRows) {
      if (p.lda <= OperandA::kLargestShortLd && p.ldb <= OperandB::kLargestShortLd) {  // block-uniform
        if (a.unscaled && b.unscaled)
          bulk(std::false_type{});
        else
          bulk(std::true_type{});  // (a factor of 1 changes no bit)
      }
    }
    for (; c0 + kFusedRing <= chunks; c0 += kFusedRing) {
      static_for<kFusedRing>([&](auto r_c) {
        constexpr int r = decltype(r_c)::value;
        const int c = c0 + r, ahead = c + kFusedRing < last ? c + kFusedRing : last;
        char* stage = lds + (r & 1) * STAGE_BYTES;
        a.deposit(xa[r], c, stage);
        b.deposit(xb[r], c, stage + REGION_BYTES);
        __builtin_amdgcn_sched_barrier(0);
        a.fetch(xa[r], ahead), b.fetch(xb[r], ahead);
        __syncthreads();
      });
    }
    static_for<kFusedRing - 1>([&](auto r_c) {  // the chunks left over: their values are on their way or here
      constexpr int r = decltype(r_c)::value;
      if (c0 + r < chunks) {  // block-uniform
        char* stage = lds + (r & 1) * STAGE_BYTES;
        a.deposit(xa[r], c0 + r, stage);
        b.deposit(xb[r], c0 + r, stage + REGION_BYTES);
        __syncthreads();
      }
    });
    return;
  }

  // ---- multiplying waves: one 32 x 32 block of the tile each.  They share their SIMDs with the splitting waves, whose
  // vector instructions fill the time that a chain of dependent matrix instructions leaves.
  const int block = wave - kFusedSplitWaves;
  const int wave_m = block % (TILE / 32), wave_n = block / (TILE / 32);
  float16_t acc_main, acc_corr;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_main[v] = 0.0f, acc_corr[v] = 0.0f;
  // The depth is added up in slices of kFusedSliceChunks chunks (512 deep, as shallow as the split-first plans ever
  // slice a tile): the sum of a slice, main + correction, joins `sliced` in ascending order and the accumulators start
  // again from zero.  The error of the matrix unit's accumulation grows with the length of the sum (the paper's
  // section "Avoiding RZ during Tensor Core accumulation"); at K = 1024 one accumulator over the whole depth gave a
  // relative residual of 2.15e-07 where two slices give 1.65e-07.  Up to 512 deep there is one slice and the bits are
  // those of an unsliced tile of the product kernels.
  const float corr_scale = (METHOD == kMethodFp16Split) ? 0x1p-11f : 1.0f;
  float sliced[16];
  bool earlier_slices = false;  // block-uniform
  const int a_frag_off = wave_m * K_STEPS * NP * 1024;
  const int b_frag_off = REGION_BYTES + wave_n * K_STEPS * NP * 1024;
  int lane_off[K_STEPS];  // of this lane's 16 bytes within a 1 KiB block of k step ks (see fused_lds_slot)
#pragma unroll
  for (int ks = 0; ks < K_STEPS; ++ks) lane_off[ks] = fused_lds_slot<NP>(lane & 31, 16 * ks + 8 * (lane >> 5)) - ks * NP * 1024;
  // A chunk is taken in two halves of two k steps, each with a register set of its own, and the next half is requested
  // before the matrix instructions of the one before it are issued: a half's way from LDS is covered by the other
  // half's arithmetic, also across the barrier between two chunks.  Within a chunk the k steps are multiplied in
  // ascending order.
  frag_t fa[2][K_STEPS / 2][NP], fb[2][K_STEPS / 2][NP];
  auto request = [&](auto half_c, int c) {  // the fragments of half HALF of chunk c -> register set HALF
    constexpr int HALF = decltype(half_c)::value;
    const char* stage = lds + (c & 1) * STAGE_BYTES;
#pragma unroll
    for (int s = 0; s < K_STEPS / 2; ++s) {
      const int ks = HALF * (K_STEPS / 2) + s;
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        fa[HALF][s][q] = *reinterpret_cast<const frag_t*>(stage + a_frag_off + (ks * NP + q) * 1024 + lane_off[ks]);
        fb[HALF][s][q] = *reinterpret_cast<const frag_t*>(stage + b_frag_off + (ks * NP + q) * 1024 + lane_off[ks]);
      }
    }
  };
  auto multiply = [&](auto half_c) {
    constexpr int HALF = decltype(half_c)::value;
#pragma unroll
    for (int s = 0; s < K_STEPS / 2; ++s) {
      static_for<PRODUCTS>([&](auto m_c) {
        constexpr ProductTerm term = product_term(METHOD, decltype(m_c)::value);
        if constexpr (term.correction)
          acc_corr = Mfma<BF16 ? kElemBf16 : kElemFp16>::run(fb[HALF][s][term.qb], fa[HALF][s][term.qa], acc_corr);
        else
          acc_main = Mfma<BF16 ? kElemBf16 : kElemFp16>::run(fb[HALF][s][term.qb], fa[HALF][s][term.qa], acc_main);
      });
    }
  };
  __syncthreads();  // chunk 0 is there
  request(std::integral_constant<int, 0>{}, 0);
  for (int c = 0; c < chunks; ++c) {
    request(std::integral_constant<int, 1>{}, c);
    multiply(std::integral_constant<int, 0>{});
    if (c + 1 < chunks) {  // block-uniform
      // (this wave's reads of chunk c have returned when it passes the barrier: __syncthreads() waits for them; only
      // then may the splitting waves overwrite the buffer)
      __syncthreads();  // chunk c + 1 is there
      request(std::integral_constant<int, 0>{}, c + 1);
    }
    multiply(std::integral_constant<int, 1>{});
    if (c % kFusedSliceChunks == kFusedSliceChunks - 1 && c + 1 < chunks) {  // a slice is complete and another follows
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float slice = acc_main[v] + acc_corr[v] * corr_scale;
        sliced[v] = earlier_slices ? sliced[v] + slice : slice;
        acc_main[v] = 0.0f, acc_corr[v] = 0.0f;
      }
      earlier_slices = true;
    }
  }

  // ---- epilogue, as in product_kernel: lane l holds row m and columns n_base + 8 (v / 4) + v % 4
  const int64_t m = (int64_t)tile_m * BM + wave_m * 32 + (lane & 31);
  const int64_t n_base = (int64_t)tile_n * BN + wave_n * 32 + 4 * (lane >> 5);
  if (p.k_slices > 1) {
    // the slice's sums, scaling undone, before alpha / beta; zero where the tile reaches beyond C
    float* out = p.partials + ((int64_t)slice * (p.tiles_m * p.tiles_n) + tile_index) * (BM * BN) +
                 (wave_n * 32 + 4 * (lane >> 5)) * BM + wave_m * 32 + (lane & 31);
    const int row_exponent = (p.row_log2_scale != nullptr && m < p.M) ? p.row_log2_scale[m] : 0;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t n = n_base + 8 * (v / 4) + (v % 4);
      const float last_slice = acc_main[v] + acc_corr[v] * corr_scale;
      float c = (earlier_slices ? sliced[v] + last_slice : last_slice) * p.out_scale;
      const bool inside = m < p.M && n < p.N;
      if (p.row_log2_scale != nullptr && inside) c = unscale(c, row_exponent, p.col_log2_scale[n]);
      store_partial(out + (8 * (v / 4) + (v % 4)) * BM, inside ? c : 0.0f);
    }
    return;
  }
  if (m >= p.M) return;
  const int row_exponent = p.row_log2_scale != nullptr ? p.row_log2_scale[m] : 0;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int64_t n = n_base + 8 * (v / 4) + (v % 4);
    if (n < p.N) {
      const float last_slice = acc_main[v] + acc_corr[v] * corr_scale;
      float c = (earlier_slices ? sliced[v] + last_slice : last_slice) * p.out_scale;
      // rows of op(A) and columns of op(B) were scaled one by one before the split: undo that per element
      if (p.row_log2_scale != nullptr) c = unscale(c, row_exponent, p.col_log2_scale[n]);
      float* dst = p.C + m + n * p.ldc;
      store_result(dst, (p.beta == 0.0f) ? p.alpha * c : scaled_sum(p.alpha, c, p.beta, *dst));
    }
  }
}

}  // namespace ecgemm
