// The paper's own arrangement of the method for one block (section "Incorporating our method into CUTLASS", last
// paragraph): the block reads FP32 tiles of A and B, forms the low-precision parts in registers (Eqs. corr-1-1024 ..
// corr-4-1024, or the three BF16 terms) and multiplies them right away; no split pass over the operands, no packed
// copies in HBM, one launch instead of three.  Every block that touches a tile of A splits it again (N / 128 times
// per element), so this only pays where launches, not arithmetic, decide the time: small products.
//
// One block: 128 x 128 of C, 4 waves of 64 x 64 (the X2 geometry of product_kernel.hpp, same fragment layout in
// LDS, same term order, same accumulator discipline, so an element is summed in the same order as there).
// Per 32-deep stage: waves 0 and 1 fetch and split the A tile, waves 2 and 3 the B tile; thread u of a pair of
// waves owns row u of its tile, holds the row's 32 FP32 values of the next stage in registers while the current
// stage is multiplied, then writes their parts to the other LDS buffer in fragment order.
#pragma once
#include "product_kernel.hpp"

namespace ecgemm {

struct FusedParams {
  const float* A;  // device, column-major, as passed to ecgemm_sgemm
  const float* B;
  int64_t lda, ldb;
  int a_k_contiguous, b_k_contiguous;  // op(A)(m, k) = A[k + m lda] (transA == T);  op(B)(k, n) = B[k + n ldb] (transB == N)
  int a_vec, b_vec;                    // k contiguous and 16-byte aligned rows: float4 loads
  float prescale_a, prescale_b;        // powers of two applied before the split (1 by default)
  int64_t M, N, K, ldc;
  int stages;                          // ceil(K / 32)
  int tiles_m, tiles_n, splits;        // splits > 1: every tile is cut into slices along K, raw sums go to partials
  float alpha, beta, out_scale;
  // per-row / per-column pre-scaling as in ProductParams (both null, or both set)
  const int* row_log2_scale;           // device, M entries
  const int* col_log2_scale;           // device, N entries
  float* C;
  float* partials;                     // [splits][tiles][128][128]
};

template <int METHOD>
__global__ void __launch_bounds__(256, 1) fused_kernel(const FusedParams p) {
  constexpr int KIND = split_kind_of(METHOD);
  constexpr bool BF16 = split_is_bf16(KIND);
  constexpr int NP = parts_of_split(KIND), PRODUCTS = products_of(METHOD);
  constexpr int BM = 128, BN = 128, TM = 2, TN = 2, K_STEPS = 2;
  constexpr int ROW_CHUNKS = K_STEPS * NP;                 // 1 KiB chunks per 32 rows per stage
  constexpr int A_CHUNKS = (BM / 32) * ROW_CHUNKS;
  constexpr int STAGE_BYTES = (A_CHUNKS + (BN / 32) * ROW_CHUNKS) * 1024;
  typedef typename Mfma<BF16 ? kElemBf16 : kElemFp16>::frag_t frag_t;
  __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE_BYTES];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wave_m = wave % 2, wave_n = wave / 2;

  const int tiles = p.tiles_m * p.tiles_n;
  const int split = blockIdx.x / tiles, pid = blockIdx.x % tiles;
  int tile_m, tile_n;
  tile_coordinates(pid, p.tiles_m, p.tiles_n, 4, 1, tile_m, tile_n);
  const int stages_per_split = (p.stages + p.splits - 1) / p.splits;
  const int stage_begin = split * stages_per_split;
  const int stage_count = max(0, min(p.stages, stage_begin + stages_per_split) - stage_begin);

  // ---- this thread's row of its operand tile
  const bool for_b = wave >= 2;  // wave-uniform
  const int u = t & 127;
  const float* src = for_b ? p.B : p.A;
  const int64_t ld = for_b ? p.ldb : p.lda;
  const bool k_contiguous = for_b ? p.b_k_contiguous : p.a_k_contiguous;
  const bool vec = for_b ? p.b_vec : p.a_vec;
  const int64_t row = (for_b ? (int64_t)tile_n * BN : (int64_t)tile_m * BM) + u;
  const bool row_ok = row < (for_b ? p.N : p.M);
  float prescale = for_b ? p.prescale_b : p.prescale_a;
  if (p.row_log2_scale != nullptr && row_ok) prescale *= row_scale_factor((for_b ? p.col_log2_scale : p.row_log2_scale)[row]);
  // Requests the 32 values X(row, k0 .. k0 + 31) of a stage.  Every load is unconditional on a clamped, valid address
  // (a load under a per-lane condition would make the compiler wait for it at the end of its branch, one load at a
  // time); what lies beyond the matrix is replaced by zeros in deposit(), after the multiplications that the loads
  // are meant to overlap.
  const int64_t row_clamped = row_ok ? row : (for_b ? p.N : p.M) - 1;
  auto fetch = [&](float (&x)[32], int stage) {
    const int64_t k0 = (int64_t)stage * 32;
    if (k_contiguous) {
      const float* base = src + row_clamped * ld;
      if (vec && k0 + 32 <= p.K) {  // block-uniform
#pragma unroll
        for (int g = 0; g < 8; ++g) {
          const float4 v = *reinterpret_cast<const float4*>(base + k0 + 4 * g);
          x[4 * g] = v.x, x[4 * g + 1] = v.y, x[4 * g + 2] = v.z, x[4 * g + 3] = v.w;
        }
      } else {
#pragma unroll
        for (int k = 0; k < 32; ++k) x[k] = base[min(k0 + k, p.K - 1)];
      }
    } else {
      const float* base = src + row_clamped;
#pragma unroll
      for (int k = 0; k < 32; ++k) x[k] = base[min(k0 + k, p.K - 1) * ld];
    }
  };
  // Splits the held values and writes the parts where the fragment reads below expect them: chunk
  // (row_block, k_step, part), lane (k % 16 / 8) * 32 + row % 32, 16 bytes per lane.
  char* my_chunks = lds + (for_b ? A_CHUNKS * 1024 : 0) + (u >> 5) * ROW_CHUNKS * 1024 + (u & 31) * 16;
  auto deposit = [&](const float (&x)[32], int stage, int buf) {
    char* base = my_chunks + buf * STAGE_BYTES;
    const int64_t k0 = (int64_t)stage * 32;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      ushort8_t parts[NP];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        unsigned short s[NP];
        Splitter<KIND>::split((row_ok && k0 + 8 * g + e < p.K) ? x[8 * g + e] * prescale : 0.0f, s);
#pragma unroll
        for (int q = 0; q < NP; ++q) parts[q][e] = s[q];
      }
#pragma unroll
      for (int q = 0; q < NP; ++q)
        *reinterpret_cast<ushort8_t*>(base + ((g >> 1) * NP + q) * 1024 + (g & 1) * 512) = parts[q];
    }
  };

  // ---- fragments and accumulators
  float16_t acc_main[TM][TN], acc_corr[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        acc_main[i][j][v] = 0.0f;
        acc_corr[i][j][v] = 0.0f;
      }
  const int a_frag_off = wave_m * TM * ROW_CHUNKS * 1024 + lane * 16;
  const int b_frag_off = A_CHUNKS * 1024 + wave_n * TN * ROW_CHUNKS * 1024 + lane * 16;
  auto multiply_stage = [&](int buf) {
    const char* stage = lds + buf * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < K_STEPS; ++ks) {
      frag_t fa[TM][NP], fb[TN][NP];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int q = 0; q < NP; ++q)
          fa[i][q] = *reinterpret_cast<const frag_t*>(stage + a_frag_off + ((i * K_STEPS + ks) * NP + q) * 1024);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < NP; ++q)
          fb[j][q] = *reinterpret_cast<const frag_t*>(stage + b_frag_off + ((j * K_STEPS + ks) * NP + q) * 1024);
      static_for<PRODUCTS * TM * TN>([&](auto m_c) {
        constexpr int m = decltype(m_c)::value;
        constexpr ProductTerm term = product_term(METHOD, m / (TM * TN));
        constexpr int i = (m % (TM * TN)) / TN, j = m % TN;
        if constexpr (term.correction)
          acc_corr[i][j] = Mfma<BF16 ? kElemBf16 : kElemFp16>::run(fb[j][term.qb], fa[i][term.qa], acc_corr[i][j]);
        else
          acc_main[i][j] = Mfma<BF16 ? kElemBf16 : kElemFp16>::run(fb[j][term.qb], fa[i][term.qa], acc_main[i][j]);
      });
    }
  };

  // ---- main loop: stage s is multiplied out of LDS buffer s % 2 while the values of stage s + 1 travel to registers
  float x[32];
  if (stage_count > 0) {
    fetch(x, stage_begin);
    deposit(x, stage_begin, 0);
    __syncthreads();
    for (int s = 0; s < stage_count; ++s) {
      const bool more = s + 1 < stage_count;
      if (more) fetch(x, stage_begin + s + 1);
      multiply_stage(s & 1);
      if (more) deposit(x, stage_begin + s + 1, (s + 1) & 1);
      __syncthreads();
    }
  }

  // ---- epilogue, as in product_kernel: lane l holds row m_base + 32 i and columns n_base + 32 j + 8 (v / 4) + v % 4
  const float corr_scale = (METHOD == kMethodFp16Split) ? 0x1p-11f : 1.0f;
  const int64_t m_base = (int64_t)tile_m * BM + wave_m * 64 + (lane & 31);
  const int64_t n_base = (int64_t)tile_n * BN + wave_n * 64 + 4 * (lane >> 5);
  auto for_each_output = [&](auto&& store) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          store(m_base + i * 32, n_base + j * 32 + 8 * (v / 4) + (v % 4),
                (acc_main[i][j][v] + acc_corr[i][j][v] * corr_scale) * p.out_scale);
  };
  if (p.row_log2_scale != nullptr) {
    // rows of op(A) and columns of op(B) were scaled one by one before the split: undo that per element
    float* out = p.splits > 1 ? p.partials + ((int64_t)split * tiles + pid) * (BM * BN) : nullptr;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    for_each_output([&](int64_t m, int64_t n, float c) {
      if (m < p.M && n < p.N) {
        c = unscale(c, p.row_log2_scale[m], p.col_log2_scale[n]);
        if (out) {
          out[(n - n0) * BM + (m - m0)] = c;
        } else {
          float* dst = p.C + m + n * p.ldc;
          store_result(dst, (p.beta == 0.0f) ? p.alpha * c : scaled_sum(p.alpha, c, p.beta, *dst));
        }
      } else if (out) {
        out[(n - n0) * BM + (m - m0)] = 0.0f;
      }
    });
  } else if (p.splits > 1) {
    float* out = p.partials + ((int64_t)split * tiles + pid) * (BM * BN);
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    for_each_output([&](int64_t m, int64_t n, float c) { out[(n - n0) * BM + (m - m0)] = c; });
  } else {
    for_each_output([&](int64_t m, int64_t n, float c) {
      if (m < p.M && n < p.N) {
        float* dst = p.C + m + n * p.ldc;
        store_result(dst, (p.beta == 0.0f) ? p.alpha * c : scaled_sum(p.alpha, c, p.beta, *dst));
      }
    });
  }
}

}  // namespace ecgemm
