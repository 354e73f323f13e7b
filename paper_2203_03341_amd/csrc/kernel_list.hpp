// The kernel instantiations of the library, and which translation unit compiles which of them.
//
// Each kernels_*.hip file defines ECGEMM_INSTANTIATE_<group> before including this header and so compiles that group;
// everywhere else (the host code in ecgemm.hip) the same lines are `extern template` declarations, so that the host
// code can take the kernels' addresses without compiling them again.  The groups only exist to let the build compile
// them side by side.
#pragma once
#include "fused_kernel.hpp"
#include "product_kernel.hpp"
#include "split_kernels.hpp"

namespace ecgemm {

// Kernel shapes: block tile, waves per block, k steps per LDS stage, stages, resident blocks per CU.
//   W4: 256 x 128, 4 waves (one per SIMD) of 128 x 64.  Least LDS and L2 traffic per flop.
//   X2: 128 x 128, 4 waves of 64 x 64, two blocks per CU.  A third more LDS reads and L2 traffic per flop; one block's
//       epilogue and pipeline fill hide behind the other's main loop, and a problem makes twice as many tiles.
// (A 256 x 128 shape with 8 waves of 64 x 64, two per SIMD, was also built and timed on 60 sizes: never more than
// 2 % ahead of W4, usually 1 % behind.)
typedef ProductConfig<kMethodFp16Split, 256, 128, 128, 64, 2, 3, 1> Fp16W4;     // 3 x 48 KiB of LDS
typedef ProductConfig<kMethodFp16Split, 128, 128, 64, 64, 1, 4, 2> Fp16X2;      // 4 x 16 KiB of LDS per block
typedef ProductConfig<kMethodBf16Full, 256, 128, 128, 64, 2, 2, 1> Bf16W4;      // 2 x 72 KiB (4 x 36 and 3 x 36 KiB: within 0.5 %)
typedef ProductConfig<kMethodBf16Full, 128, 128, 64, 64, 1, 3, 2> Bf16X2;       // 3 x 24 KiB per block
// comparison methods: the W4 shape only
typedef ProductConfig<kMethodFp16Markidis, 256, 128, 128, 64, 2, 3, 1> MarkidisConfig;
typedef ProductConfig<kMethodFp16Unscaled, 256, 128, 128, 64, 2, 3, 1> UnscaledConfig;
typedef ProductConfig<kMethodFp16Plain, 256, 128, 128, 64, 2, 3, 1> PlainFp16Config;
typedef ProductConfig<kMethodBf16Plain, 256, 128, 128, 64, 2, 3, 1> PlainBf16Config;
// (the "outside" methods keep a third accumulator set: 128 x 128 tiles of 64 x 64 per wave, one workgroup per unit)
typedef ProductConfig<kMethodFp16Outside, 128, 128, 64, 64, 1, 4, 1> OutsideConfig;
typedef ProductConfig<kMethodFp16Outside4, 128, 128, 64, 64, 1, 4, 1> Outside4Config;
typedef ProductConfig<kMethodFp16Outside16, 128, 128, 64, 64, 1, 4, 1> Outside16Config;
typedef ProductConfig<kMethodFp32, 256, 128, 128, 64, 2, 3, 1> Fp32Config;

#ifdef ECGEMM_INSTANTIATE_FP16
#define ECGEMM_FP16_GROUP
#else
#define ECGEMM_FP16_GROUP extern
#endif
#ifdef ECGEMM_INSTANTIATE_BF16
#define ECGEMM_BF16_GROUP
#else
#define ECGEMM_BF16_GROUP extern
#endif
#ifdef ECGEMM_INSTANTIATE_COMPARE_A
#define ECGEMM_COMPARE_A_GROUP
#else
#define ECGEMM_COMPARE_A_GROUP extern
#endif
#ifdef ECGEMM_INSTANTIATE_COMPARE_B
#define ECGEMM_COMPARE_B_GROUP
#else
#define ECGEMM_COMPARE_B_GROUP extern
#endif
#ifdef ECGEMM_INSTANTIATE_FUSED
#define ECGEMM_FUSED_GROUP
#else
#define ECGEMM_FUSED_GROUP extern
#endif
#ifdef ECGEMM_INSTANTIATE_SPLIT
#define ECGEMM_SPLIT_GROUP
#else
#define ECGEMM_SPLIT_GROUP extern
#endif

ECGEMM_FP16_GROUP template __global__ void product_kernel<Fp16W4, false>(const ProductParams);
ECGEMM_FP16_GROUP template __global__ void product_kernel<Fp16X2, false>(const ProductParams);
ECGEMM_FP16_GROUP template __global__ void product_kernel<Fp16W4, true>(const ProductParams);  // for calls with scaling vectors
ECGEMM_FP16_GROUP template __global__ void product_kernel<Fp16X2, true>(const ProductParams);
#define ECGEMM_REDUCE_KERNEL(BM, BN)                                                                                        \
  ECGEMM_FP16_GROUP template __global__ void reduce_tail_kernel<BM, BN>(const float*, int, int, int, int, int, int, int, int64_t, \
                                                                        int64_t, float, float, float*, int64_t, const int*, int, int);
ECGEMM_REDUCE_KERNEL(256, 128)
ECGEMM_REDUCE_KERNEL(128, 128)
ECGEMM_REDUCE_KERNEL(64, 64)  // (the one-launch shapes, when they slice the depth)
ECGEMM_REDUCE_KERNEL(32, 32)
ECGEMM_BF16_GROUP template __global__ void product_kernel<Bf16W4, false>(const ProductParams);
ECGEMM_BF16_GROUP template __global__ void product_kernel<Bf16X2, false>(const ProductParams);
ECGEMM_BF16_GROUP template __global__ void product_kernel<Bf16W4, true>(const ProductParams);
ECGEMM_BF16_GROUP template __global__ void product_kernel<Bf16X2, true>(const ProductParams);
ECGEMM_COMPARE_A_GROUP template __global__ void product_kernel<MarkidisConfig, false>(const ProductParams);
ECGEMM_COMPARE_A_GROUP template __global__ void product_kernel<UnscaledConfig, false>(const ProductParams);
ECGEMM_COMPARE_A_GROUP template __global__ void product_kernel<OutsideConfig, false>(const ProductParams);
ECGEMM_COMPARE_A_GROUP template __global__ void product_kernel<Outside4Config, false>(const ProductParams);
ECGEMM_COMPARE_A_GROUP template __global__ void product_kernel<Outside16Config, false>(const ProductParams);
ECGEMM_COMPARE_B_GROUP template __global__ void product_kernel<PlainFp16Config, false>(const ProductParams);
ECGEMM_COMPARE_B_GROUP template __global__ void product_kernel<PlainBf16Config, false>(const ProductParams);
ECGEMM_COMPARE_B_GROUP template __global__ void product_kernel<Fp32Config, false>(const ProductParams);
#define ECGEMM_FUSED_KERNELS_OF(METHOD, LAYOUT_A, TILE)                                                            \
  ECGEMM_FUSED_GROUP template __global__ void fused_kernel<METHOD, LAYOUT_A, kFusedRows, TILE>(const FusedParams);   \
  ECGEMM_FUSED_GROUP template __global__ void fused_kernel<METHOD, LAYOUT_A, kFusedDepth, TILE>(const FusedParams);  \
  ECGEMM_FUSED_GROUP template __global__ void fused_kernel<METHOD, LAYOUT_A, kFusedDepthVec, TILE>(const FusedParams);
#define ECGEMM_FUSED_KERNELS_OF_METHOD(METHOD)           \
  ECGEMM_FUSED_KERNELS_OF(METHOD, kFusedRows, 64)        \
  ECGEMM_FUSED_KERNELS_OF(METHOD, kFusedDepth, 64)       \
  ECGEMM_FUSED_KERNELS_OF(METHOD, kFusedDepthVec, 64)    \
  ECGEMM_FUSED_KERNELS_OF(METHOD, kFusedRows, 32)        \
  ECGEMM_FUSED_KERNELS_OF(METHOD, kFusedDepth, 32)       \
  ECGEMM_FUSED_KERNELS_OF(METHOD, kFusedDepthVec, 32)
ECGEMM_FUSED_KERNELS_OF_METHOD(kMethodFp16Split)
ECGEMM_FUSED_KERNELS_OF_METHOD(kMethodBf16Full)

#define ECGEMM_SPLIT_KERNELS_OF(KIND)                                                                     \
  ECGEMM_SPLIT_GROUP template __global__ void split_kernel<KIND, kSplitKContiguousVec, false>(const SplitJob);   \
  ECGEMM_SPLIT_GROUP template __global__ void split_kernel<KIND, kSplitKContiguous, false>(const SplitJob);      \
  ECGEMM_SPLIT_GROUP template __global__ void split_kernel<KIND, kSplitRContiguous, false>(const SplitJob);      \
  ECGEMM_SPLIT_GROUP template __global__ void split_kernel<KIND, kSplitRContiguousWide, false>(const SplitJob);  \
  ECGEMM_SPLIT_GROUP template __global__ void split_pair_kernel<KIND, false>(const SplitJob, const SplitJob);
ECGEMM_SPLIT_KERNELS_OF(kSplitFp16Scaled)
ECGEMM_SPLIT_KERNELS_OF(kSplitBf16x3)
ECGEMM_SPLIT_KERNELS_OF(kSplitFp16Unscaled)
ECGEMM_SPLIT_KERNELS_OF(kSplitFp16Plain)
ECGEMM_SPLIT_KERNELS_OF(kSplitBf16Plain)
ECGEMM_SPLIT_KERNELS_OF(kSplitFp32)
#undef ECGEMM_SPLIT_KERNELS_OF
// (the FP16 pair split that also measures what the pair loses: automatic mode choice)
ECGEMM_SPLIT_GROUP template __global__ void split_kernel<kSplitFp16Scaled, kSplitKContiguousVec, true>(const SplitJob);
ECGEMM_SPLIT_GROUP template __global__ void split_kernel<kSplitFp16Scaled, kSplitKContiguous, true>(const SplitJob);
ECGEMM_SPLIT_GROUP template __global__ void split_kernel<kSplitFp16Scaled, kSplitRContiguous, true>(const SplitJob);
ECGEMM_SPLIT_GROUP template __global__ void split_kernel<kSplitFp16Scaled, kSplitRContiguousWide, true>(const SplitJob);
ECGEMM_SPLIT_GROUP template __global__ void split_pair_kernel<kSplitFp16Scaled, true>(const SplitJob, const SplitJob);

}  // namespace ecgemm
