// Host side of the ecgemm C-ABI (see include/ecgemm.h): argument checks, workspace, kernel launches.
#include "../../include/ecgemm.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "product_kernel.hpp"
#include "split_kernels.hpp"

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
  int* range_buffer = nullptr;  // two ints of device memory for ecgemm_exponent_range
  std::vector<TimedCall> timed;
  std::vector<hipEvent_t> free_events;
  std::string last_error;
};

namespace {

// Tile shapes.  The macros exist so that other shapes can be built and timed side by side; the defaults are
// the ones every figure in this repository was measured with.
#ifndef ECGEMM_FP16_KSTEPS
#define ECGEMM_FP16_KSTEPS 2
#endif
#ifndef ECGEMM_FP16_STAGES
#define ECGEMM_FP16_STAGES 3
#endif
#ifndef ECGEMM_BF16_KSTEPS
#define ECGEMM_BF16_KSTEPS 1
#endif
#ifndef ECGEMM_BF16_STAGES
#define ECGEMM_BF16_STAGES 4
#endif
typedef ProductConfig<kMethodFp16Split, 256, 128, 128, 64, ECGEMM_FP16_KSTEPS, ECGEMM_FP16_STAGES> Fp16Config;  // 3 x 48 KiB of LDS
typedef ProductConfig<kMethodBf16Full, 256, 128, 128, 64, ECGEMM_BF16_KSTEPS, ECGEMM_BF16_STAGES> Bf16Config;   // 4 x 36 KiB of LDS
// comparison methods: same tile, same pipeline
typedef ProductConfig<kMethodFp16Markidis, 256, 128, 128, 64, ECGEMM_FP16_KSTEPS, ECGEMM_FP16_STAGES> MarkidisConfig;
typedef ProductConfig<kMethodFp16Unscaled, 256, 128, 128, 64, ECGEMM_FP16_KSTEPS, ECGEMM_FP16_STAGES> UnscaledConfig;
typedef ProductConfig<kMethodFp16Plain, 256, 128, 128, 64, 2, 3> PlainFp16Config;
typedef ProductConfig<kMethodBf16Plain, 256, 128, 128, 64, 2, 3> PlainBf16Config;
typedef ProductConfig<kMethodFp16Outside, 256, 128, 128, 64, ECGEMM_FP16_KSTEPS, ECGEMM_FP16_STAGES> OutsideConfig;
// 128 x 128 tiles, two workgroups per CU: twice the LDS and L2 traffic per flop, but one workgroup's epilogue and
// pipeline fill hide behind the other's main loop.  Used for shallow K, where those fixed costs dominate.
typedef ProductConfig<kMethodFp16Split, 128, 128, 64, 64, 2, 2, 2> SmallFp16Config;   // 2 x 32 KiB of LDS per workgroup
typedef ProductConfig<kMethodBf16Full, 128, 128, 64, 64, 1, 3, 2> SmallBf16Config;    // 3 x 24 KiB of LDS per workgroup
#ifndef ECGEMM_SMALL_TILE_MAX_K
#define ECGEMM_SMALL_TILE_MAX_K 512
#endif
// Deepest K slice per work item for which the 256 x 128 product kernels run as a persistent grid (measured: 1-2 %
// faster up to here, 1-2 % slower at 16384; the 128 x 128 kernels are never faster as a persistent grid).
#ifndef ECGEMM_PERSISTENT_MAX_K
#define ECGEMM_PERSISTENT_MAX_K 4096
#endif
static_assert(SmallFp16Config::BK == Fp16Config::BK && SmallBf16Config::BK == Bf16Config::BK, "stage depths");


inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
// the ecgemm_mode_t values are the ProductMethod values
inline int parts_of(ecgemm_mode_t mode) { return parts_of_split(split_kind_of((int)mode)); }
inline bool valid_mode(int mode) { return mode >= ECGEMM_MODE_FP16_SPLIT && mode <= ECGEMM_MODE_FP16_OUTSIDE_ACC; }
inline int stage_depth_of(ecgemm_mode_t mode) { return mode == ECGEMM_MODE_BF16_FULL ? Bf16Config::BK : Fp16Config::BK; }
static_assert((int)ECGEMM_MODE_FP16_SPLIT == (int)kMethodFp16Split && (int)ECGEMM_MODE_BF16_FULL == (int)kMethodBf16Full &&
              (int)ECGEMM_MODE_FP16_MARKIDIS == (int)kMethodFp16Markidis &&
              (int)ECGEMM_MODE_FP16_UNSCALED == (int)kMethodFp16Unscaled &&
              (int)ECGEMM_MODE_FP16_PLAIN == (int)kMethodFp16Plain && (int)ECGEMM_MODE_BF16_PLAIN == (int)kMethodBf16Plain &&
              (int)ECGEMM_MODE_FP16_OUTSIDE_ACC == (int)kMethodFp16Outside,
              "mode numbering");
static_assert(PlainFp16Config::BK == Fp16Config::BK && MarkidisConfig::BK == Fp16Config::BK, "stage depths");
inline bool valid_op(int op) { return op == ECGEMM_OP_N || op == ECGEMM_OP_T; }

size_t packed_bytes(int64_t rows, int64_t depth, ecgemm_mode_t mode) {
  return (size_t)round_up(rows, kRowPad) * (size_t)round_up(depth, kDepthPad) * 2 * parts_of(mode);
}

struct Plan {
  bool small_tiles;  // 128 x 128, two workgroups per CU
  int bm, bn;
  int64_t Mp, Np, Kp;
  int tiles_m, tiles_n, k_tiles, k_splits;
  size_t a_bytes, b_bytes, partial_bytes, total_bytes;
};

// One tile shape per mode (256 x 128 x 32, 4 waves).  K is divided among blocks only when the output
// tiles alone cannot occupy the 256 CUs and K is deep enough to leave every block a long loop.
Plan make_plan(int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode) {
  Plan pl;
  pl.Mp = round_up(M, kRowPad);
  pl.Np = round_up(N, kRowPad);
  pl.Kp = round_up(K, kDepthPad);
  pl.small_tiles = (mode == ECGEMM_MODE_FP16_SPLIT || mode == ECGEMM_MODE_BF16_FULL) && pl.Kp <= ECGEMM_SMALL_TILE_MAX_K;
  pl.bm = pl.small_tiles ? 128 : 256;
  pl.bn = 128;
  pl.tiles_m = (int)((M + pl.bm - 1) / pl.bm);
  pl.tiles_n = (int)((N + pl.bn - 1) / pl.bn);
  pl.k_tiles = (int)(pl.Kp / stage_depth_of(mode));
  const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
  int splits = 1;
  if (tiles < 192) {
    splits = (int)((512 + tiles - 1) / tiles);
    const int max_by_depth = (int)(pl.Kp / 512);  // at least 512 of depth per block
    if (splits > max_by_depth) splits = max_by_depth;
    if (splits > 64) splits = 64;
    if (splits < 1) splits = 1;
  }
  pl.k_splits = splits;
  pl.a_bytes = align256(packed_bytes(M, K, mode));
  pl.b_bytes = align256(packed_bytes(N, K, mode));
  pl.partial_bytes = splits > 1 ? align256((size_t)splits * pl.Mp * pl.Np * sizeof(float)) : 0;
  pl.total_bytes = pl.a_bytes + pl.b_bytes + pl.partial_bytes;
  return pl;
}

ecgemm_status_t fail(ecgemm_handle_t h, ecgemm_status_t st, const std::string& what) {
  if (h) h->last_error = what;
  return st;
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
ecgemm_status_t launch_split(ecgemm_handle_t h, ecgemm_op_t op, int64_t rows, int64_t depth, const float* src,
                             int64_t ld, ecgemm_mode_t mode, void* packed, int log2_prescale = 0) {
  const float prescale = std::ldexp(1.0f, log2_prescale);
  const int64_t Rp = round_up(rows, kRowPad), Kp = round_up(depth, kDepthPad);
  const int64_t k_steps = Kp / 16;
  const int64_t blocks64 = (Kp / 32) * (Rp / 64);
  if (blocks64 > 0x7fffffff) return fail(h, ECGEMM_ERR_INVALID_ARG, "operand has more than 2^42 elements");
  const dim3 block(256), grid64((unsigned)blocks64), grid256((unsigned)(blocks64 / 4));
  const unsigned k_tiles = (unsigned)(Kp / 32);
  unsigned short* out = static_cast<unsigned short*>(packed);
  const bool k_contiguous = op == ECGEMM_OP_T;
  const bool vec = (ld % 4 == 0) && ((uintptr_t)src % 16 == 0);
#define ECGEMM_LAUNCH_SPLIT(KIND)                                                                                          \
  do {                                                                                                                     \
    if (!k_contiguous && vec)                                                                                              \
      hipLaunchKernelGGL((split_r_contiguous_wide<KIND>), grid256, block, 0, h->stream, src, ld, rows, depth, k_steps,     \
                         prescale, out, (unsigned)(Rp / 256));                                                             \
    else if (!k_contiguous)                                                                                                \
      hipLaunchKernelGGL((split_r_contiguous<KIND>), grid64, block, 0, h->stream, src, ld, rows, depth, k_steps, prescale, \
                         out, (unsigned)(Rp / 64));                                                                        \
    else if (vec)                                                                                                          \
      hipLaunchKernelGGL((split_k_contiguous<KIND, true>), grid64, block, 0, h->stream, src, ld, rows, depth, k_steps,     \
                         prescale, out, k_tiles);                                                                          \
    else                                                                                                                   \
      hipLaunchKernelGGL((split_k_contiguous<KIND, false>), grid64, block, 0, h->stream, src, ld, rows, depth, k_steps,    \
                         prescale, out, k_tiles);                                                                          \
  } while (0)
  switch (split_kind_of((int)mode)) {
    case kSplitFp16Scaled: ECGEMM_LAUNCH_SPLIT(kSplitFp16Scaled); break;
    case kSplitBf16x3: ECGEMM_LAUNCH_SPLIT(kSplitBf16x3); break;
    case kSplitFp16Unscaled: ECGEMM_LAUNCH_SPLIT(kSplitFp16Unscaled); break;
    case kSplitFp16Plain: ECGEMM_LAUNCH_SPLIT(kSplitFp16Plain); break;
    default: ECGEMM_LAUNCH_SPLIT(kSplitBf16Plain); break;
  }
#undef ECGEMM_LAUNCH_SPLIT
  ECGEMM_HIP(h, hipGetLastError());
  return ECGEMM_OK;
}

// Steps 2 and 3 on operands already in fragment order (padded as ecgemm_split pads them, or tighter).
ecgemm_status_t launch_product(ecgemm_handle_t h, const Plan& pl, int64_t M, int64_t N, float alpha, const void* a_packed,
                               const void* b_packed, float beta, float* C, int64_t ldc, ecgemm_mode_t mode, float* partials,
                               int log2_out_scale = 0) {
  ProductParams pp;
  pp.a_packed = static_cast<const char*>(a_packed);
  pp.b_packed = static_cast<const char*>(b_packed);
  pp.row_block_bytes = (pl.Kp / 16) * parts_of(mode) * 1024;
  pp.k_tiles = pl.k_tiles;
  pp.k_splits = pl.k_splits;
  pp.tiles_m = pl.tiles_m;
  pp.tiles_n = pl.tiles_n;
  pp.M = M;
  pp.N = N;
  pp.ldc = ldc;
  pp.alpha = alpha;
  pp.beta = beta;
  pp.out_scale = std::ldexp(1.0f, log2_out_scale);
  pp.C = C;
  pp.partials = partials;
  pp.Mp = pl.Mp;
  pp.Np = pl.Np;
  // Grid, always a multiple of the 8 XCDs.  Items of moderate depth on the 256 x 128 kernels: a persistent grid, one
  // block per CU, each block walking through several items with the next item's loads in flight during its epilogue.
  // Otherwise one block per item, handed out in order by the hardware as CUs free up, which keeps the tiles an XCD
  // works on at any time next to each other: blocks of a persistent grid drift apart over long items and lose L2
  // hits (72 % instead of 82 % at K = 16384), and two co-resident 128 x 128 blocks already cover each other's epilogue.
  const int64_t items = (int64_t)pl.tiles_m * pl.tiles_n * pl.k_splits;
  const int64_t slots = (int64_t)h->compute_units * (pl.small_tiles ? 2 : 1);
  const int64_t depth_per_item = (pl.Kp + pl.k_splits - 1) / pl.k_splits;
  const bool persistent = !pl.small_tiles && depth_per_item <= ECGEMM_PERSISTENT_MAX_K;
  const dim3 grid((unsigned)(items < slots || !persistent ? round_up(items, 8) : slots));
  if (pl.small_tiles) {
    if (mode == ECGEMM_MODE_BF16_FULL)
      hipLaunchKernelGGL(product_kernel<SmallBf16Config>, grid, dim3(SmallBf16Config::THREADS), 0, h->stream, pp);
    else
      hipLaunchKernelGGL(product_kernel<SmallFp16Config>, grid, dim3(SmallFp16Config::THREADS), 0, h->stream, pp);
  } else
  switch (mode) {
    case ECGEMM_MODE_FP16_SPLIT: hipLaunchKernelGGL(product_kernel<Fp16Config>, grid, dim3(Fp16Config::THREADS), 0, h->stream, pp); break;
    case ECGEMM_MODE_BF16_FULL: hipLaunchKernelGGL(product_kernel<Bf16Config>, grid, dim3(Bf16Config::THREADS), 0, h->stream, pp); break;
    case ECGEMM_MODE_FP16_MARKIDIS: hipLaunchKernelGGL(product_kernel<MarkidisConfig>, grid, dim3(MarkidisConfig::THREADS), 0, h->stream, pp); break;
    case ECGEMM_MODE_FP16_UNSCALED: hipLaunchKernelGGL(product_kernel<UnscaledConfig>, grid, dim3(UnscaledConfig::THREADS), 0, h->stream, pp); break;
    case ECGEMM_MODE_FP16_PLAIN: hipLaunchKernelGGL(product_kernel<PlainFp16Config>, grid, dim3(PlainFp16Config::THREADS), 0, h->stream, pp); break;
    case ECGEMM_MODE_BF16_PLAIN: hipLaunchKernelGGL(product_kernel<PlainBf16Config>, grid, dim3(PlainBf16Config::THREADS), 0, h->stream, pp); break;
    case ECGEMM_MODE_FP16_OUTSIDE_ACC: hipLaunchKernelGGL(product_kernel<OutsideConfig>, grid, dim3(OutsideConfig::THREADS), 0, h->stream, pp); break;
  }
  ECGEMM_HIP(h, hipGetLastError());
  if (pl.k_splits > 1) {
    const dim3 rgrid((unsigned)((M + 255) / 256), (unsigned)(N < 65535 ? N : 65535));
    hipLaunchKernelGGL(reduce_partials_kernel, rgrid, dim3(256), 0, h->stream, partials, pl.k_splits, pl.Mp, pl.Np, M, N, alpha,
                       beta, C, ldc);
    ECGEMM_HIP(h, hipGetLastError());
  }
  return ECGEMM_OK;
}

// Device memory for this call: the caller's workspace if one is set (never allocating), else the handle's own,
// grown on demand.
ecgemm_status_t acquire_workspace(ecgemm_handle_t h, size_t bytes, char** out) {
  *out = nullptr;
  if (bytes == 0) return ECGEMM_OK;
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

ecgemm_status_t check_sizes(ecgemm_handle_t h, int64_t M, int64_t N, int64_t K, ecgemm_mode_t mode) {
  // tile indices are 32-bit and the byte offset along K inside a row block is a 32-bit vector offset
  if (M > (int64_t)1 << 36 || N > (int64_t)1 << 36) return fail(h, ECGEMM_ERR_INVALID_ARG, "M or N too large");
  if ((round_up(K, kDepthPad) / 16) * parts_of(mode) * 1024 >= ((int64_t)1 << 32))
    return fail(h, ECGEMM_ERR_INVALID_ARG, "K too large: a packed row block must stay below 4 GiB");
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

ecgemm_status_t ecgemm_create(ecgemm_handle_t* handle) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  *handle = nullptr;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return ECGEMM_ERR_HIP;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return ECGEMM_ERR_HIP;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return ECGEMM_ERR_UNSUPPORTED;
  ecgemm_context* ctx = new (std::nothrow) ecgemm_context();
  if (!ctx) return ECGEMM_ERR_ALLOC;
  ctx->device = device;
  ctx->compute_units = prop.multiProcessorCount > 8 ? prop.multiProcessorCount / 8 * 8 : 8;
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

ecgemm_status_t ecgemm_workspace_size(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K,
                                      ecgemm_mode_t mode, size_t* bytes) {
  if (!bytes || M < 0 || N < 0 || K < 0 || !valid_mode(mode))
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_workspace_size: bad argument");
  *bytes = (M == 0 || N == 0 || K == 0) ? 0 : make_plan(M, N, K, mode).total_bytes;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_set_workspace(ecgemm_handle_t handle, void* device_buffer, size_t bytes) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if ((device_buffer == nullptr) != (bytes == 0) || ((uintptr_t)device_buffer % 256) != 0)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_set_workspace: buffer must be 256-byte aligned, or (NULL, 0)");
  handle->user_workspace = device_buffer;
  handle->user_bytes = bytes;
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
  if (!valid_op(op) || !valid_mode(mode) || rows < 0 || depth < 0)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_split: bad enum or negative size");
  if (rows == 0 || depth == 0) return ECGEMM_OK;
  if (!src || !packed || ((uintptr_t)packed % 16) != 0)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_split: null or misaligned pointer");
  if (ld < (op == ECGEMM_OP_N ? rows : depth))
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_split: leading dimension too small");
  return launch_split(handle, op, rows, depth, src, ld, mode, packed);
}

ecgemm_status_t ecgemm_set_scaling(ecgemm_handle_t handle, int log2_scale_a, int log2_scale_b) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (std::abs(log2_scale_a) > 126 || std::abs(log2_scale_b) > 126 || std::abs(log2_scale_a + log2_scale_b) > 126)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_set_scaling: exponents (and their sum) must stay within +-126");
  handle->log2_scale_a = log2_scale_a;
  handle->log2_scale_b = log2_scale_b;
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_exponent_range(ecgemm_handle_t handle, int64_t rows, int64_t cols, const float* src, int64_t ld,
                                      int* min_exponent, int* max_exponent) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!min_exponent || !max_exponent || rows < 0 || cols < 0)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_exponent_range: bad argument");
  int host[2] = {INT_MAX, INT_MIN};
  if (rows > 0 && cols > 0) {
    if (!src || ld < rows) return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_exponent_range: null source or ld < rows");
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

ecgemm_status_t ecgemm_choose_mode(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB, int64_t M, int64_t N,
                                   int64_t K, const float* A, int64_t lda, const float* B, int64_t ldb,
                                   ecgemm_mode_t* mode, int* log2_scale_a, int* log2_scale_b) {
  if (!handle) return ECGEMM_ERR_INVALID_ARG;
  if (!mode || !log2_scale_a || !log2_scale_b || !valid_op(transA) || !valid_op(transB) || M < 0 || N < 0 || K < 0)
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_choose_mode: bad argument");
  int lo[2] = {0, 0}, hi[2] = {0, 0};
  ecgemm_status_t st = ecgemm_exponent_range(handle, transA == ECGEMM_OP_N ? M : K, transA == ECGEMM_OP_N ? K : M, A, lda,
                                             &lo[0], &hi[0]);
  if (st != ECGEMM_OK) return st;
  st = ecgemm_exponent_range(handle, transB == ECGEMM_OP_N ? K : N, transB == ECGEMM_OP_N ? N : K, B, ldb, &lo[1], &hi[1]);
  if (st != ECGEMM_OK) return st;
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
  if (count < 0 || count > 0x7fffffff) return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_debug_mfma: bad count");
  if (count == 0) return ECGEMM_OK;
  if (!a || !b || !c || !d || ((uintptr_t)a % 16) || ((uintptr_t)b % 16) || ((uintptr_t)c % 64) || ((uintptr_t)d % 64))
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_debug_mfma: null or misaligned pointer");
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
  if (!operands || !sink || !flops || blocks <= 0 || iters <= 0 || ((uintptr_t)operands % 16))
    return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_debug_mfma_rate: bad argument");
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
  if (!calls || !split_ms || !product_ms) return fail(handle, ECGEMM_ERR_INVALID_ARG, "ecgemm_get_timing: null output");
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

ecgemm_status_t ecgemm_sgemm(ecgemm_handle_t handle, ecgemm_op_t transA, ecgemm_op_t transB,
                             int64_t M, int64_t N, int64_t K, float alpha,
                             const float* A, int64_t lda, const float* B, int64_t ldb,
                             float beta, float* C, int64_t ldc, ecgemm_mode_t mode) {
  ecgemm_handle_t h = handle;
  if (!h) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_op(transA) || !valid_op(transB) || !valid_mode(mode))
    return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: bad transA / transB / mode");
  if (M < 0 || N < 0 || K < 0) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: negative size");
  if (M == 0 || N == 0) return ECGEMM_OK;
  if (!C || ldc < M) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: C is null or ldc < M");

  const dim3 block256(256);
  if (K == 0 || alpha == 0.0f) {
    const dim3 grid((unsigned)((M + 255) / 256), (unsigned)(N < 65535 ? N : 65535));
    hipLaunchKernelGGL(scale_c_kernel, grid, block256, 0, h->stream, M, N, beta, C, ldc);
    ECGEMM_HIP(h, hipGetLastError());
    return ECGEMM_OK;
  }
  if (!A || !B) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: A or B is null");
  if (lda < (transA == ECGEMM_OP_N ? M : K)) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: lda too small");
  if (ldb < (transB == ECGEMM_OP_N ? K : N)) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: ldb too small");

  ecgemm_status_t st = check_sizes(h, M, N, K, mode);
  if (st != ECGEMM_OK) return st;
  const Plan pl = make_plan(M, N, K, mode);
  if ((int64_t)pl.tiles_m * pl.tiles_n * pl.k_splits > 0x7fffffffLL)
    return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_sgemm: too many tiles");
  char* ws = nullptr;
  st = acquire_workspace(h, pl.total_bytes, &ws);
  if (st != ECGEMM_OK) return st;
  char* a_packed = ws;
  char* b_packed = ws + pl.a_bytes;
  float* partials = pl.k_splits > 1 ? reinterpret_cast<float*>(ws + pl.a_bytes + pl.b_bytes) : nullptr;

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
  } lease{h};
  TimedCall& tc = lease.tc;
  if (h->timing) {
    tc.start = take_event(h);
    tc.split_done = take_event(h);
    tc.product_done = take_event(h);
    if (!tc.start || !tc.split_done || !tc.product_done) return fail(h, ECGEMM_ERR_HIP, "ecgemm_sgemm: hipEventCreate failed");
    ECGEMM_HIP(h, hipEventRecord(tc.start, h->stream));
  }

  // step 1: op(A) is M x K with rows m; op(B)^T is N x K with rows n.  For B the roles of N and T swap:
  // B stored K x N (transB == N) has k contiguous, i.e. it is the "T" case of the splitter.
  st = launch_split(h, transA, M, K, A, lda, mode, a_packed, h->log2_scale_a);
  if (st != ECGEMM_OK) return st;
  st = launch_split(h, transB == ECGEMM_OP_N ? ECGEMM_OP_T : ECGEMM_OP_N, N, K, B, ldb, mode, b_packed, h->log2_scale_b);
  if (st != ECGEMM_OK) return st;
  if (h->timing) ECGEMM_HIP(h, hipEventRecord(tc.split_done, h->stream));

  // steps 2 and 3
  st = launch_product(h, pl, M, N, alpha, a_packed, b_packed, beta, C, ldc, mode, partials,
                      -(h->log2_scale_a + h->log2_scale_b));
  if (st != ECGEMM_OK) return st;
  if (h->timing) {
    ECGEMM_HIP(h, hipEventRecord(tc.product_done, h->stream));
    h->timed.push_back(tc);
    lease.keep = true;
  }
  return ECGEMM_OK;
}

ecgemm_status_t ecgemm_product(ecgemm_handle_t handle, int64_t M, int64_t N, int64_t K, float alpha,
                               const void* packedA, const void* packedB, float beta, float* C, int64_t ldc,
                               ecgemm_mode_t mode) {
  ecgemm_handle_t h = handle;
  if (!h) return ECGEMM_ERR_INVALID_ARG;
  if (!valid_mode(mode)) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_product: bad mode");
  if (M < 0 || N < 0 || K < 0) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_product: negative size");
  if (M == 0 || N == 0) return ECGEMM_OK;
  if (!C || ldc < M) return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_product: C is null or ldc < M");
  if (K == 0 || alpha == 0.0f) {
    const dim3 grid((unsigned)((M + 255) / 256), (unsigned)(N < 65535 ? N : 65535));
    hipLaunchKernelGGL(scale_c_kernel, grid, dim3(256), 0, h->stream, M, N, beta, C, ldc);
    ECGEMM_HIP(h, hipGetLastError());
    return ECGEMM_OK;
  }
  if (!packedA || !packedB || ((uintptr_t)packedA % 16) != 0 || ((uintptr_t)packedB % 16) != 0)
    return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_product: packed operand is null or not 16-byte aligned");
  ecgemm_status_t st = check_sizes(h, M, N, K, mode);
  if (st != ECGEMM_OK) return st;
  const Plan pl = make_plan(M, N, K, mode);
  if ((int64_t)pl.tiles_m * pl.tiles_n * pl.k_splits > 0x7fffffffLL)
    return fail(h, ECGEMM_ERR_INVALID_ARG, "ecgemm_product: too many tiles");
  char* ws = nullptr;
  st = acquire_workspace(h, pl.partial_bytes, &ws);
  if (st != ECGEMM_OK) return st;
  return launch_product(h, pl, M, N, alpha, packedA, packedB, beta, C, ldc, mode, reinterpret_cast<float*>(ws));
}

}  // extern "C"
