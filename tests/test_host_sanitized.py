"""The host side of the library (argument checks, planner, workspace arithmetic, error strings) under
AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

A C program calls every entry point that can run without a GPU - and the others with arguments that must be refused
before any GPU work - against a build of the library whose host code is instrumented; any report from either sanitizer
ends the program with a non-zero status."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "ecgemm.h"
#include "ecgemm_debug.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t next(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }
#define CHECK(cond) do { if (!(cond)) { printf("line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
  size_t bytes = 0;
  ecgemm_plan_info_t info;
  int i, mode;
  /* names of every status, and of a value that is none */
  for (i = -1; i < 7; ++i) CHECK(strlen(ecgemm_status_string((ecgemm_status_t)i)) > 8);
  CHECK(strcmp(ecgemm_last_error_string(NULL), "null handle") == 0);
  CHECK(ecgemm_last_error_argument(NULL) == -1);
  /* sizes: valid, zero, negative, unknown mode, null output */
  for (mode = 0; mode <= 9; ++mode) {
    CHECK(ecgemm_split_size(1, 1, (ecgemm_mode_t)mode, &bytes) == ECGEMM_OK && bytes >= 256 * 32 * 2);
    CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_T, 300, 200, 100, (ecgemm_mode_t)mode, &bytes) == ECGEMM_OK);
    CHECK(ecgemm_plan_info(NULL, 300, 200, 100, (ecgemm_mode_t)mode, &info) == ECGEMM_OK && info.workspace_bytes == bytes);
  }
  CHECK(ecgemm_split_size(-1, 1, ECGEMM_MODE_FP16_SPLIT, &bytes) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_split_size(1, 1, ECGEMM_MODE_AUTO, &bytes) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_split_size(1, 1, (ecgemm_mode_t)11, &bytes) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_plan_info(NULL, 300, 200, 100, ECGEMM_MODE_AUTO, &info) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, (ecgemm_mode_t)11, &bytes) == ECGEMM_ERR_INVALID_ARG);
  { /* the automatic mode's workspace serves either candidate and holds its statistics */
    size_t fp16 = 0, bf16 = 0, both = 0;
    CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_T, 3000, 2000, 5000, ECGEMM_MODE_FP16_SPLIT, &fp16) == ECGEMM_OK);
    CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_T, 3000, 2000, 5000, ECGEMM_MODE_BF16_FULL, &bf16) == ECGEMM_OK);
    CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_T, 3000, 2000, 5000, ECGEMM_MODE_AUTO, &both) == ECGEMM_OK);
    CHECK(both > fp16 && both > bf16 && both % 256 == 0 && both < bf16 + fp16);
    CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_T, 0, 2000, 5000, ECGEMM_MODE_AUTO, &both) == ECGEMM_OK && both == 0);
  }
  CHECK(ecgemm_split_size(1, 1, ECGEMM_MODE_FP16_SPLIT, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, (ecgemm_op_t)2, ECGEMM_OP_N, 1, 1, 1, ECGEMM_MODE_FP16_SPLIT, &bytes) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, (ecgemm_mode_t)-1, &bytes) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, -1, 1, ECGEMM_MODE_FP16_SPLIT, &bytes) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, ECGEMM_MODE_FP16_SPLIT, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 0, 5, 5, ECGEMM_MODE_BF16_FULL, &bytes) == ECGEMM_OK && bytes == 0);
  CHECK(ecgemm_plan_info(NULL, 1, 1, 1, ECGEMM_MODE_FP16_SPLIT, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_plan_info(NULL, 0, 1, 1, ECGEMM_MODE_FP16_SPLIT, &info) == ECGEMM_ERR_INVALID_ARG);
  /* the limits of the 32-bit tile and offset arithmetic, from both sides */
  CHECK(ecgemm_plan_info(NULL, (int64_t)1 << 36, 1, 1, ECGEMM_MODE_FP16_SPLIT, &info) == ECGEMM_OK);
  CHECK(ecgemm_plan_info(NULL, ((int64_t)1 << 36) + 1, 1, 1, ECGEMM_MODE_FP16_SPLIT, &info) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_plan_info(NULL, (int64_t)1 << 22, (int64_t)1 << 22, 32, ECGEMM_MODE_BF16_FULL, &info) == ECGEMM_OK);
  CHECK(ecgemm_plan_info(NULL, (int64_t)1 << 23, (int64_t)1 << 23, 32, ECGEMM_MODE_BF16_FULL, &info) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_plan_info(NULL, 4, 4, ((int64_t)1 << 25) - 32, ECGEMM_MODE_FP16_SPLIT, &info) == ECGEMM_OK);
  CHECK(ecgemm_plan_info(NULL, 4, 4, (int64_t)1 << 25, ECGEMM_MODE_FP16_SPLIT, &info) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_plan_info(NULL, 4, 4, (int64_t)1 << 62, ECGEMM_MODE_FP16_SPLIT, &info) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_N, INT64_MAX, INT64_MAX, INT64_MAX, ECGEMM_MODE_FP16_SPLIT, &bytes) ==
        ECGEMM_ERR_INVALID_ARG);
  /* the planner on random problems, small to huge, every mode: tiles accounted for, sizes consistent */
  for (i = 0; i < 3000; ++i) {
    const int64_t M = 1 + (int64_t)(next() % (i % 7 == 0 ? 200000 : 9000));
    const int64_t N = 1 + (int64_t)(next() % (i % 11 == 0 ? 200000 : 9000));
    const int64_t K = 1 + (int64_t)(next() % (i % 5 == 0 ? 300000 : 20000));
    mode = (int)(next() % 10);
    CHECK(ecgemm_plan_info(NULL, M, N, K, (ecgemm_mode_t)mode, &info) == ECGEMM_OK);
    CHECK((int64_t)info.tiles_m * info.tiles_n == (int64_t)info.whole_tiles + info.sliced_tiles);
    CHECK(info.slices >= 1 && info.slices <= 64 && (int64_t)info.slices * info.sliced_tiles <= 1024);
    CHECK(info.grid > 0 && info.column_bands >= 1 && info.column_bands <= 8 && info.estimated_us > 0.0);
    CHECK(ecgemm_workspace_size(NULL, ECGEMM_OP_T, ECGEMM_OP_N, M, N, K, (ecgemm_mode_t)mode, &bytes) == ECGEMM_OK);
    if (info.shape >= 3) { /* one launch: one block per tile and slice of the depth, only partial sums in the workspace, small products only */
      CHECK(info.grid == (int64_t)info.tiles_m * info.tiles_n * info.slices && mode <= 1);
      CHECK(info.workspace_bytes == (info.slices > 1 ? (size_t)info.slices * info.sliced_tiles * info.tile_m * info.tile_n * 4 : 0));
      CHECK(info.slices == 1 || (info.grid <= 256 && K / info.slices >= 512 && info.sliced_tiles == info.tiles_m * info.tiles_n));
      CHECK(info.tile_m == (info.shape == 3 ? 64 : 32) && (K <= 8192 || info.slices > 1) && info.grid <= 4096);
    } else {
      CHECK(info.grid % 8 == 0 && bytes == info.workspace_bytes);
    }
  }
  /* everything that takes a handle refuses a null one without touching the GPU */
  CHECK(ecgemm_create(NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_destroy(NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_set_stream(NULL, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_set_workspace(NULL, NULL, 0) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_set_shape(NULL, ECGEMM_SHAPE_AUTO) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_set_scaling(NULL, 0, 0) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_debug_set_tile_order(NULL, 1, 0, 0) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_set_timing(NULL, 1) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_get_timing(NULL, &i, NULL, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_sgemm(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, 1.0f, NULL, 1, NULL, 1, 0.0f, NULL, 1, ECGEMM_MODE_FP16_SPLIT) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_sgemm_noalloc(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, 1.0f, NULL, 1, NULL, 1, 0.0f, NULL, 1, ECGEMM_MODE_FP16_SPLIT) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_sgemm_scaled(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, 1.0f, NULL, 1, NULL, 1, 0.0f, NULL, 1, ECGEMM_MODE_FP16_SPLIT, NULL, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_sgemm(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, 1.0f, NULL, 1, NULL, 1, 0.0f, NULL, 1, ECGEMM_MODE_AUTO) == ECGEMM_ERR_INVALID_ARG);
  { ecgemm_mode_t chosen; int scaled; CHECK(ecgemm_auto_choice(NULL, &chosen, &scaled) == ECGEMM_ERR_INVALID_ARG); }
  CHECK(ecgemm_product(NULL, 1, 1, 1, 1.0f, NULL, NULL, 0.0f, NULL, 1, ECGEMM_MODE_FP16_SPLIT) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_split(NULL, ECGEMM_OP_N, 1, 1, NULL, 1, ECGEMM_MODE_FP16_SPLIT, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_row_scales(NULL, ECGEMM_OP_N, 1, 1, NULL, 1, 14, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_exponent_range(NULL, 1, 1, NULL, 1, &i, &i) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_choose_mode(NULL, ECGEMM_OP_N, ECGEMM_OP_N, 1, 1, 1, NULL, 1, NULL, 1, NULL, NULL, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_debug_mfma(NULL, 0, 1, NULL, NULL, NULL, NULL) == ECGEMM_ERR_INVALID_ARG);
  CHECK(ecgemm_debug_mfma_rate(NULL, 0, NULL, NULL, 1, 1, NULL) == ECGEMM_ERR_INVALID_ARG);
  /* the tile order: reciprocal arithmetic against division over whole grids */
  {
    static int32_t tm[1 << 16], tn[1 << 16];
    int64_t bad = -1;
    for (i = 0; i < 200; ++i) {
      const int64_t M = 1 + (int64_t)(next() % 20000), N = 1 + (int64_t)(next() % 20000), K = 1 + (int64_t)(next() % 9000);
      mode = (int)(next() % 2);
      CHECK(ecgemm_plan_info(NULL, M, N, K, (ecgemm_mode_t)mode, &info) == ECGEMM_OK);
      if ((int64_t)info.tiles_m * info.tiles_n > (1 << 16)) continue;
      if (info.shape >= 3) {
        CHECK(ecgemm_debug_tile_order(NULL, M, N, K, (ecgemm_mode_t)mode, tm, tn, &bad) == ECGEMM_ERR_UNSUPPORTED);
        continue;
      }
      CHECK(ecgemm_debug_tile_order(NULL, M, N, K, (ecgemm_mode_t)mode, tm, tn, &bad) == ECGEMM_OK && bad == 0);
    }
    CHECK(ecgemm_debug_tile_order(NULL, 5, 5, 5, ECGEMM_MODE_FP16_SPLIT, NULL, tn, &bad) == ECGEMM_ERR_INVALID_ARG);
  }
  printf("host side clean\n");
  return 0;
}
'''


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    import importlib.util
    spec = importlib.util.spec_from_file_location("ecgemm_hip_build", os.path.join(ROOT, "paper_2203_03341_amd", "build.py"))
    hip_build = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(hip_build)
    clang = os.path.join(os.path.dirname(hip_build.CLANGXX), "clang")
    if not (os.path.exists(hip_build.HIPCC) and os.path.exists(clang)):
        pytest.skip("no ROCm compilers")
    lib = hip_build.build_host_sanitized()
    src = tmp_path / "host_driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "host_driver"
    lib_dir, lib_name = os.path.dirname(lib), os.path.basename(lib)[3:-3]
    build = subprocess.run([clang, "-std=c99", "-Wall", "-Werror", "-g", "-fsanitize=address,undefined", "-shared-libsan",
                            "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"), str(src), "-L", lib_dir,
                            "-l" + lib_name, "-Wl,-rpath," + lib_dir, "-o", str(exe)], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    rt_dir = os.path.dirname(subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True,
                                            text=True).stdout.strip())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               LD_LIBRARY_PATH=os.pathsep.join(p for p in (rt_dir, os.environ.get("LD_LIBRARY_PATH", "")) if p))
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.returncode, run.stdout[-2000:], run.stderr[-4000:])
    assert "host side clean" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
