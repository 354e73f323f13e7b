// The small kernels around the hot path: C <- beta C, exponent statistics for the pre-scaling helpers, and the two
// diagnostic kernels that run bare matrix instructions.  Compiled with the host code (ecgemm.hip) only.
#pragma once
#include "product_kernel.hpp"

namespace ecgemm {

// K == 0 or alpha == 0: C <- beta * C, and C <- 0 without reading it when beta == 0.
__global__ void __launch_bounds__(256) scale_c_kernel(int64_t M, int64_t N, float beta, float* __restrict__ C, int64_t ldc) {
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= M) return;
  for (int64_t n = blockIdx.y; n < N; n += gridDim.y) {
    float* dst = C + m + n * ldc;
    *dst = (beta == 0.0f) ? 0.0f : beta * *dst;
  }
}

// Smallest and largest binary exponent among the non-zero finite elements of a column-major rows x cols matrix
// (subnormals count as exponent -127).  range[0] must start at INT_MAX and range[1] at INT_MIN.
__global__ void __launch_bounds__(256) exponent_range_kernel(const float* __restrict__ src, int64_t ld, int64_t rows,
                                                             int64_t cols, int* __restrict__ range) {
  int lo = 0x7fffffff, hi = -0x7fffffff - 1;
  for (int64_t c = blockIdx.y; c < cols; c += gridDim.y)
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < rows; r += (int64_t)gridDim.x * 256) {
      const unsigned bits = __builtin_bit_cast(unsigned, src[r + c * ld]) & 0x7fffffffu;
      if (bits != 0 && bits < 0x7f800000u) {
        const int e = (int)(bits >> 23) - 127;
        lo = e < lo ? e : lo;
        hi = e > hi ? e : hi;
      }
    }
  if (lo <= hi) {
    atomicMin(&range[0], lo);
    atomicMax(&range[1], hi);
  }
}

// Per-row scaling exponents of one operand, or of both operands of a product, in three small kernels on one stream.
// Each takes a gate like the split and product kernels (null: always runs).
struct RowScaleJob {
  const float* src;  // X(r, k) = src[r + k * ld] or src[k + r * ld]
  int64_t ld, rows, depth;
  int slab;          // k per workgroup in step 2
  int k_contiguous;
  int target;        // where step 3 puts the row's largest binade
  unsigned grid_x;   // step 2: workgroups along the rows (256 rows each, or 4 when k is contiguous: one wave per row) ...
  unsigned blocks;   // ... times slabs
  int* scale;        // device, `rows` entries: the largest exponent after step 2, the scaling exponent after step 3
};

// (1) scale[r] <- INT_MIN, both jobs (b.rows may be 0)
__global__ void __launch_bounds__(256) row_scales_clear_kernel(const RowScaleJob a, const RowScaleJob b, const int* gate,
                                                               int gate_value) {
  if (!gate_open(gate, gate_value)) return;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < a.rows) a.scale[i] = -0x7fffffff - 1;
  else if (i - a.rows < b.rows) b.scale[i - a.rows] = -0x7fffffff - 1;
}

// (2) scale[r] <- largest binary exponent among the non-zero finite elements of row r of X (subnormals count as
// -127).  A workgroup takes a slab of `slab` k of its rows; lanes run along the contiguous direction.  (r contiguous:
// a thread walks its row's slab eight independent loads at a time; the host keeps those slabs short, 128 k, so that
// a matrix makes thousands of workgroups and not a hundred.)  Workgroups 0 .. a.blocks - 1 work on a, the rest on b.
__global__ void __launch_bounds__(256) row_max_exponent_kernel(const RowScaleJob a, const RowScaleJob b, const int* gate,
                                                               int gate_value) {
  if (!gate_open(gate, gate_value)) return;
  const bool second = blockIdx.x >= a.blocks;  // block-uniform
  const RowScaleJob& job = second ? b : a;
  const unsigned block = second ? blockIdx.x - a.blocks : blockIdx.x;
  const unsigned bx = block % job.grid_x, by = block / job.grid_x;
  const float* src = job.src;
  const int64_t ld = job.ld, rows = job.rows;
  const int64_t k_begin = (int64_t)by * job.slab, k_end = k_begin + job.slab < job.depth ? k_begin + job.slab : job.depth;
  auto exponent_of = [](float v) { return finite_exponent(v); };
  int hi = -0x7fffffff - 1;
  if (!job.k_contiguous) {
    const int64_t r = (int64_t)bx * 256 + threadIdx.x;
    if (r >= rows) return;
    const float* at = src + r + k_begin * ld;
    int64_t k = k_begin;
    for (; k + 8 <= k_end; k += 8, at += 8 * ld) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = at[u * ld];
#pragma unroll
      for (int u = 0; u < 8; ++u) hi = max(hi, exponent_of(v[u]));
    }
    for (; k < k_end; ++k, at += ld) hi = max(hi, exponent_of(*at));
    if (hi != -0x7fffffff - 1) atomicMax(&job.scale[r], hi);
  } else {
    const int64_t r = (int64_t)bx * 4 + (threadIdx.x >> 6);  // one wave per row
    if (r >= rows) return;
    for (int64_t k = k_begin + (threadIdx.x & 63); k < k_end; k += 64) hi = max(hi, exponent_of(src[k + r * ld]));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) hi = max(hi, __shfl_xor(hi, d, 64));
    if ((threadIdx.x & 63) == 0 && hi != -0x7fffffff - 1) atomicMax(&job.scale[r], hi);
  }
}

// Step (3) for entry i of the two jobs' rows taken together (a's first).
__device__ __forceinline__ void finish_row_scale(const RowScaleJob& a, const RowScaleJob& b, int64_t i) {
  const bool second = i >= a.rows;
  const RowScaleJob& job = second ? b : a;
  const int64_t r = second ? i - a.rows : i;
  if (r >= job.rows) return;
  const int hi = job.scale[r];
  int e = hi == -0x7fffffff - 1 ? 0 : job.target - hi;
  e = e < -126 ? -126 : e > 126 ? 126 : e;
  job.scale[r] = e;
}

// (3) in place: the exponent that moves the row's largest binade to 2^target (0 for a row without non-zero finite
// elements), kept inside what one power-of-two factor can express.
__global__ void __launch_bounds__(256) row_scales_finish_kernel(const RowScaleJob a, const RowScaleJob b, const int* gate,
                                                                int gate_value) {
  if (!gate_open(gate, gate_value)) return;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  finish_row_scale(a, b, i);
}

// One v_mfma_f32_32x32x16 per wave on caller-supplied registers, for tests that pin down what the matrix unit does
// (lane map, rounding, subnormals): lane l of problem p reads a[(p * 64 + l) * 8 .. +8], b likewise, c[(p * 64 + l) * 16
// .. +16] and writes d at the same place.
template <bool BF16>
__global__ void __launch_bounds__(64) single_mfma_kernel(const unsigned short* __restrict__ a, const unsigned short* __restrict__ b,
                                                         const float* __restrict__ c, float* __restrict__ d) {
  typedef typename Mfma<BF16 ? kElemBf16 : kElemFp16>::frag_t frag_t;
  const int64_t slot = (int64_t)blockIdx.x * 64 + threadIdx.x;
  const frag_t fa = *reinterpret_cast<const frag_t*>(a + slot * 8);
  const frag_t fb = *reinterpret_cast<const frag_t*>(b + slot * 8);
  float16_t acc = *reinterpret_cast<const float16_t*>(c + slot * 16);
  acc = Mfma<BF16 ? kElemBf16 : kElemFp16>::run(fa, fb, acc);
  *reinterpret_cast<float16_t*>(d + slot * 16) = acc;
}

// Matrix instructions only, no memory traffic in the loop: every wave of the grid issues `iters` x 24
// v_mfma_f32_32x32x16 on operands it read once (12 fragments per lane from `operands`, 256 lanes x 16 bytes each).
// Timed by the caller, this gives the rate the matrix pipes sustain for a given operand content; with random
// operands it is well below the nominal peak because the clock drops under load.
template <bool BF16>
__global__ void __launch_bounds__(256, 1) mfma_rate_kernel(const unsigned short* __restrict__ operands, float* __restrict__ sink,
                                                           int iters) {
  typedef typename Mfma<BF16 ? kElemBf16 : kElemFp16>::frag_t frag_t;
  frag_t fa[6], fb[6];
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    fa[i] = *reinterpret_cast<const frag_t*>(operands + (i * 256 + threadIdx.x) * 8);
    fb[i] = *reinterpret_cast<const frag_t*>(operands + ((6 + i) * 256 + threadIdx.x) * 8);
  }
  float16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = Mfma<BF16 ? kElemBf16 : kElemFp16>::run(fa[(i + 2 * r) % 6], fb[(i * 5 + r) % 6], acc[i]);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Automatic mode choice: from the blocks' statistics of both operands, *choice = if_fits or if_not.  It fits if
//   * the FP16 pair represents both operands as they were split to within `tolerance`, relative, in the Frobenius
//     norm, and
//   * at least one operand spreads the weight of a row over `min_terms` elements or more, measured by the
//     participation ratio (sum |x|)^2 / (rows sum x^2): the pair holds 22.75 of FP32's 24 bits, which is as good as
//     an FP32 product only where that product's own summation error outweighs the missing bit; a dot product carried
//     by a handful of terms is rounded a handful of times by FP32 and is better served by the exact three-term split.
// One block of 1024 threads; every sum in a fixed order, so that equal inputs give an equal choice.  A NaN anywhere
// gives if_not.  Gated like the other kernels, on the word it writes: the second round runs only if the first failed.
// If it does not fit and `finish_a` / `finish_b` have rows, the block goes on to turn their rows' largest exponents
// into scaling exponents (step 3 of the row scales: for operands with few rows, where that saves a launch).
__global__ void __launch_bounds__(1024) choose_mode_kernel(const double* __restrict__ stats_a, unsigned blocks_a, double rows_a,
                                                           const double* __restrict__ stats_b, unsigned blocks_b, double rows_b,
                                                           double tolerance, double min_terms, int* __restrict__ choice,
                                                           int if_fits, int if_not, const int* gate, int gate_value,
                                                           const RowScaleJob finish_a, const RowScaleJob finish_b) {
  if (!gate_open(gate, gate_value)) return;
  __shared__ int chosen;
  constexpr int kThreads = 1024, kS = kStatsPerBlock;
  __shared__ double partial[kThreads][2 * kS];
  // Thread t adds entries t, t + 1024, ... of an operand in that order; eight of them are fetched at a time (a large
  // operand leaves 100000 entries, and one workgroup taking them one by one would be bound by the latency of each).
  auto sum_of = [&](const double* stats, unsigned blocks, double* sums) {
#pragma unroll
    for (int q = 0; q < kS; ++q) sums[q] = 0.0;
    unsigned i = threadIdx.x;
    for (; (uint64_t)i + 7 * kThreads < blocks; i += 8 * kThreads) {
      double v[8][kS];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int q = 0; q < kS; ++q) v[u][q] = stats[kS * (size_t)(i + u * kThreads) + q];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int q = 0; q < kS; ++q) sums[q] += v[u][q];
    }
    for (; i < blocks; i += kThreads)
#pragma unroll
      for (int q = 0; q < kS; ++q) sums[q] += stats[kS * (size_t)i + q];
  };
  double sums[2 * kS];
  sum_of(stats_a, blocks_a, sums);
  sum_of(stats_b, blocks_b, sums + kS);
#pragma unroll
  for (int q = 0; q < 2 * kS; ++q) partial[threadIdx.x][q] = sums[q];
  __syncthreads();
  for (int half = kThreads / 2; half >= 1; half >>= 1) {
    if ((int)threadIdx.x < half)
#pragma unroll
      for (int q = 0; q < 2 * kS; ++q) partial[threadIdx.x][q] += partial[threadIdx.x + half][q];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double* a = partial[0];      // err2, norm2, abs1 of A
    const double* b = partial[0] + kS;  // ... of B
    const double t2 = tolerance * tolerance;
    const bool represented = a[0] <= t2 * a[1] && b[0] <= t2 * b[1];
    // (sum |x|)^2 >= min_terms rows sum x^2, for either operand; an all-zero operand has nothing to lose
    const bool spread = a[2] * a[2] >= min_terms * rows_a * a[1] || b[2] * b[2] >= min_terms * rows_b * b[1] ||
                        a[1] == 0.0 || b[1] == 0.0;
    chosen = (represented && spread) ? if_fits : if_not;
    *choice = chosen;
  }
  __syncthreads();
  if (chosen == if_not)
    for (int64_t i = threadIdx.x; i < finish_a.rows + finish_b.rows; i += kThreads) finish_row_scale(finish_a, finish_b, i);
}

}  // namespace ecgemm
