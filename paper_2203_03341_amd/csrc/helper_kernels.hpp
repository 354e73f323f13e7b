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

// Per-row scaling exponents, in three small kernels on one stream.  (1) row_max[r] <- INT_MIN.
__global__ void __launch_bounds__(256) fill_int_kernel(int* __restrict__ dst, int64_t count, int value) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) dst[i] = value;
}

// (2) row_max[r] <- largest binary exponent among the non-zero finite elements of row r of X (subnormals count as
// -127), X(r, k) = src[r + k * ld] or src[k + r * ld].  blockIdx.y takes a slab of 2048 k; lanes run along the
// contiguous direction.
__global__ void __launch_bounds__(256) row_max_exponent_kernel(const float* __restrict__ src, int64_t ld, int64_t rows,
                                                               int64_t depth, int k_contiguous, int* __restrict__ row_max) {
  const int64_t k_begin = (int64_t)blockIdx.y * 2048, k_end = k_begin + 2048 < depth ? k_begin + 2048 : depth;
  auto exponent_of = [](float v) {
    const unsigned bits = __builtin_bit_cast(unsigned, v) & 0x7fffffffu;
    return (bits != 0 && bits < 0x7f800000u) ? (int)(bits >> 23) - 127 : -0x7fffffff - 1;
  };
  int hi = -0x7fffffff - 1;
  if (!k_contiguous) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    for (int64_t k = k_begin; k < k_end; ++k) hi = max(hi, exponent_of(src[r + k * ld]));
    if (hi != -0x7fffffff - 1) atomicMax(&row_max[r], hi);
  } else {
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // one wave per row
    if (r >= rows) return;
    for (int64_t k = k_begin + (threadIdx.x & 63); k < k_end; k += 64) hi = max(hi, exponent_of(src[k + r * ld]));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) hi = max(hi, __shfl_xor(hi, d, 64));
    if ((threadIdx.x & 63) == 0 && hi != -0x7fffffff - 1) atomicMax(&row_max[r], hi);
  }
}

// (3) in place: the exponent that moves the row's largest binade to 2^target (0 for a row without non-zero finite
// elements), kept inside what one power-of-two factor can express.
__global__ void __launch_bounds__(256) finish_row_scales_kernel(int* __restrict__ row_scale, int64_t rows, int target) {
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  const int hi = row_scale[r];
  int e = hi == -0x7fffffff - 1 ? 0 : target - hi;
  e = e < -126 ? -126 : e > 126 ? 126 : e;
  row_scale[r] = e;
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

// Automatic mode choice: from the blocks' statistics of both operands, *choice = 0 (the FP16 pair represents both
// operands to within `tolerance`, relative, in the Frobenius norm) or 1 (it does not: three BF16 terms).  One block of
// 256 threads; every sum in a fixed order, so that equal inputs give an equal choice.  A NaN anywhere gives 1.
__global__ void __launch_bounds__(256) choose_mode_kernel(const double* __restrict__ stats_a, unsigned blocks_a,
                                                          const double* __restrict__ stats_b, unsigned blocks_b,
                                                          double tolerance, int* __restrict__ choice) {
  __shared__ double partial[256][4];
  double sums[4] = {0.0, 0.0, 0.0, 0.0};
  for (unsigned i = threadIdx.x; i < blocks_a; i += 256) sums[0] += stats_a[2 * (size_t)i], sums[1] += stats_a[2 * (size_t)i + 1];
  for (unsigned i = threadIdx.x; i < blocks_b; i += 256) sums[2] += stats_b[2 * (size_t)i], sums[3] += stats_b[2 * (size_t)i + 1];
#pragma unroll
  for (int q = 0; q < 4; ++q) partial[threadIdx.x][q] = sums[q];
  __syncthreads();
  for (int half = 128; half >= 1; half >>= 1) {
    if ((int)threadIdx.x < half)
#pragma unroll
      for (int q = 0; q < 4; ++q) partial[threadIdx.x][q] += partial[threadIdx.x + half][q];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double t2 = tolerance * tolerance;
    const bool fits = partial[0][0] <= t2 * partial[0][1] && partial[0][2] <= t2 * partial[0][3];
    *choice = fits ? 0 : 1;
  }
}

}  // namespace ecgemm
