"""The shared library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    """Every function declared in include/*.h (ecgemm.h: the production surface; ecgemm_debug.h: test and tuning knobs)."""
    import glob
    names = set()
    for header in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names.update(re.findall(r"\b(ecgemm_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_north_star_entry_points():
    names = _declared_functions()
    for required in ("ecgemm_create", "ecgemm_sgemm", "ecgemm_destroy"):
        assert required in names


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: a C99 program that includes the header, calls the entry points that need no GPU and
    links against the shared library must build with gcc and run."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        import pytest
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib_dir = os.path.join(root, "paper_2203_03341_amd")
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include <stdio.h>\n#include "ecgemm.h"\n'
        "int main(void) {\n"
        "  size_t bytes = 0; ecgemm_plan_info_t info;\n"
        "  if (ecgemm_workspace_size(NULL, ECGEMM_OP_N, ECGEMM_OP_T, 4096, 4096, 4096, ECGEMM_MODE_FP16_SPLIT, &bytes) != ECGEMM_OK) return 1;\n"
        "  if (ecgemm_plan_info(NULL, 4096, 4096, 4096, ECGEMM_MODE_BF16_FULL, &info) != ECGEMM_OK) return 2;\n"
        "  if (ecgemm_plan_info(NULL, 0, 1, 1, ECGEMM_MODE_BF16_FULL, &info) != ECGEMM_ERR_INVALID_ARG) return 3;\n"
        '  printf("%zu %d %s\\n", bytes, info.tile_m, ecgemm_status_string(ECGEMM_ERR_UNSUPPORTED));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "use_header"
    build = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), str(src),
                            "-L", lib_dir, "-lecgemm", "-Wl,-rpath," + lib_dir, "-o", str(exe)], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0, (run.returncode, run.stderr)
    assert run.stdout.split() == [str(2 * 4096 * 4096 * 4), "256", "ECGEMM_ERR_UNSUPPORTED"]


def test_library_exports_every_declared_symbol():
    from paper_2203_03341_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared_functions()


def test_status_strings_and_sizes_need_no_gpu():
    import paper_2203_03341_amd as ec
    assert ec.status_string(ec.OK) == "ECGEMM_OK"
    assert ec.status_string(ec.ERR_INVALID_ARG) == "ECGEMM_ERR_INVALID_ARG"
    # rows pad to 256, depth to 32, two (FP16) or three (BF16) 16-bit parts
    assert ec.split_size(1, 1, ec.MODE_FP16_SPLIT) == 256 * 32 * 2 * 2
    assert ec.split_size(257, 33, ec.MODE_BF16_FULL) == 512 * 64 * 2 * 3


def test_product_path_does_not_touch_the_oracle():
    """The package must not import, load or mention the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2203_03341_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_plan_of_the_baseline_configs():
    """Host logic: which kernel shape a problem gets, how its tiles become work items, how the kernel is launched."""
    import paper_2203_03341_amd as ec
    W4, X2 = ec.SHAPE_256x128_W4, ec.SHAPE_128x128_X2
    p = ec.plan_info(16384, 16384, 16384, ec.MODE_FP16_SPLIT)          # headline: 8192 whole tiles, one workgroup each
    assert (p["shape"], p["tile_m"], p["tile_n"], p["whole_tiles"], p["sliced_tiles"], p["persistent"], p["grid"]) == \
        (W4, 256, 128, 8192, 0, 0, 8192)
    assert p["workspace_bytes"] == 2 * 16384 * 16384 * 4
    # column bands of the tile order = how the 8 XCDs lie over the tile grid: as many rows of XCDs as keep the live A
    # panels (group_m tile rows x K, packed) within 128 MiB of the shared cache
    assert (p["group_m"], p["column_bands"]) == (4, 4)                  # 64 MiB panels: 2 x 4
    assert ec.plan_info(8192, 8192, 8192, ec.MODE_FP16_SPLIT)["column_bands"] == 2     # 32 MiB panels: 4 x 2
    assert ec.plan_info(8192, 8192, 8192, ec.MODE_BF16_FULL)["column_bands"] == 4      # 48 MiB panels: 2 x 4
    assert ec.plan_info(8192, 8192, 2048, ec.MODE_FP16_SPLIT)["column_bands"] == 1     # 8 MiB panels: 8 x 1
    assert ec.plan_info(4096, 4096, 4096, ec.MODE_FP16_SPLIT)["column_bands"] == 1     # four groups of 16 MiB
    assert ec.plan_info(2048, 8192, 32800, ec.MODE_FP16_SPLIT)["column_bands"] == 8    # one panel is 128 MiB: 1 x 8
    assert ec.plan_info(1024, 8192, 32800, ec.MODE_FP16_SPLIT)["column_bands"] == 1    # a single group of tile rows
    assert ec.plan_info(4096, 16384 + 128, 16384, ec.MODE_FP16_SPLIT)["column_bands"] == 4   # 129 tile columns: 33 + 3 x 32
    assert ec.plan_info(16384, 512, 16384, ec.MODE_FP16_SPLIT)["column_bands"] == 1    # 4 tile columns: narrower than a patch
    p = ec.plan_info(4096, 4096, 4096, ec.MODE_BF16_FULL)              # K <= 4096: persistent grid of one block per CU
    assert (p["shape"], p["whole_tiles"], p["persistent"], p["grid"]) == (W4, 512, 1, 256)
    p = ec.plan_info(16384, 16384, 256, ec.MODE_FP16_SPLIT)            # shallow K: 128 x 128 tiles, two blocks per CU
    assert (p["shape"], p["tile_m"], p["whole_tiles"], p["slices"], p["persistent"]) == (X2, 128, 128 * 128, 1, 0)
    assert (p["group_m"], p["column_bands"]) == (8, 1)
    p = ec.plan_info(1024, 1024, 65536, ec.MODE_FP16_SPLIT)            # 32 tiles: all cut into 8 slices = 256 items
    assert (p["shape"], p["whole_tiles"], p["sliced_tiles"], p["slices"], p["grid"]) == (W4, 0, 32, 8, 256)
    p = ec.plan_info(4095, 3001, 5003, ec.MODE_BF16_FULL)              # 384 tiles: 256 whole, 128 in two slices
    assert (p["shape"], p["tiles_m"], p["tiles_n"], p["whole_tiles"], p["sliced_tiles"], p["slices"]) == (W4, 16, 24, 256, 128, 2)
    p = ec.plan_info(1024, 1024, 1024, ec.MODE_BF16_FULL)              # one launch: 256 blocks of 64 x 64, one per compute unit
    assert (p["shape"], p["sliced_tiles"], p["slices"], p["grid"]) == (ec.SHAPE_64x64_FUSED, 0, 1, 256)
    p = ec.plan_info(1280, 1280, 1280, ec.MODE_BF16_FULL)              # 25 tiles x 2 slices would leave CUs idle: smaller tiles
    assert (p["shape"], p["sliced_tiles"], p["slices"], p["grid"]) == (X2, 100, 2, 200)
    p = ec.plan_info(640, 640, 16384, ec.MODE_BF16_FULL)               # 6 W4 tiles could not fill the chip: smaller tiles,
    assert (p["shape"], p["sliced_tiles"]) == (X2, 25) and 10 <= p["slices"] <= 21   # one or two slices per compute unit
    p = ec.plan_info(512, 512, 16384, ec.MODE_BF16_FULL)               # few enough tiles for one launch: 64 of 64 x 64 in 4 slices
    assert (p["shape"], p["sliced_tiles"], p["slices"], p["grid"]) == (ec.SHAPE_64x64_FUSED, 64, 4, 256)
    p = ec.plan_info(1792, 1792, 1792, ec.MODE_FP16_SPLIT)             # 196 tiles of 128 x 128, one per CU: slices would only add traffic
    assert (p["shape"], p["whole_tiles"], p["slices"]) == (X2, 196, 1)
    p = ec.plan_info(2048, 2048, 2048, ec.MODE_FP16_SPLIT)             # 256 tiles of 128 x 128 beat 128 of 256 x 128 in 2 slices
    assert (p["shape"], p["whole_tiles"], p["slices"]) == (X2, 256, 1)
    p = ec.plan_info(2304, 2304, 2304, ec.MODE_FP16_SPLIT)             # 162 tiles of 256 x 128 beat 324 of 128 x 128 (68 CUs with two)
    assert (p["shape"], p["whole_tiles"], p["slices"]) == (W4, 162, 1)
    p = ec.plan_info(960, 2304, 18688, ec.MODE_FP16_SPLIT)             # 72 deep tiles: 3 slices each, 216 items in one round
    assert (p["shape"], p["sliced_tiles"], p["slices"]) == (W4, 72, 3)
    p = ec.plan_info(300, 200, 100, ec.MODE_FP16_MARKIDIS)             # comparison methods: one shape
    assert (p["shape"], p["tiles_m"], p["tiles_n"]) == (W4, 2, 2)
    # small products: one launch that splits for itself, 32 x 32 tiles while those leave compute units idle, 64 x 64
    # after that, nothing in the workspace; deep products of few tiles: the same with the depth in slices of at least
    # 512 (all blocks in one round) and a reduction; the split-first shapes again once blocks crowd the units, or the
    # depth is beyond 8192 and the tiles are too many for slices
    F64, F32 = ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED
    for mode in (ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL):
        for (M, N, K, shape, sliced) in [(1, 1, 1, F32, False), (256, 256, 256, F32, False), (512, 512, 512, F32, False),
                                         (300, 200, 77, F32, False), (4096, 128, 128, (F32, F64), False), (1024, 1024, 256, F64, False),
                                         (1536, 1536, 1536, X2, None), (128, 128, 8256, (F32, F64), True), (1024, 1024, 8256, (W4, X2), None), (256, 256, 4096, (F32, F64), True),
                                         (128, 128, 4096, (F32, F64), True), (64, 64, 1023, (F32, F64), False)]:
            p = ec.plan_info(M, N, K, mode)
            assert p["shape"] == shape or (isinstance(shape, tuple) and p["shape"] in shape), (M, N, K, mode, p)
            if p["shape"] in (F64, F32):
                tile = 64 if p["shape"] == F64 else 32
                tiles = -(-M // tile) * -(-N // tile)
                assert (p["tile_m"], p["tile_n"]) == (tile, tile) and p["tiles_m"] * p["tiles_n"] == tiles and p["estimated_us"] > 4
                assert (p["slices"] > 1) == sliced and p["grid"] == tiles * p["slices"]
                if sliced:
                    assert p["sliced_tiles"] == tiles and p["grid"] <= 256 and K // p["slices"] >= 512
                    assert p["workspace_bytes"] == p["slices"] * tiles * tile * tile * 4
                else:
                    assert (p["sliced_tiles"], p["workspace_bytes"]) == (0, 0)
    for mode in (ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL):
        for (M, N, K) in [(1, 1, 1), (257, 129, 33), (5000, 7000, 900), (20000, 300, 70000)]:
            p = ec.plan_info(M, N, K, mode)
            assert p["tiles_m"] * p["tiles_n"] == p["whole_tiles"] + p["sliced_tiles"]
            assert p["tiles_m"] == -(-M // p["tile_m"]) and p["tiles_n"] == -(-N // p["tile_n"])
            assert (p["slices"] == 1) == (p["sliced_tiles"] == 0)
            if p["shape"] in (W4, X2):
                assert p["workspace_bytes"] == ec.workspace_size(ec.OP_N, ec.OP_N, M, N, K, mode)
            if p["slices"] > 1:
                assert -(-K // p["slices"]) >= 512 - 32                  # a slice is never shallower than 512 (padded)
    import pytest
    with pytest.raises(ec.EcgemmError):
        ec.plan_info(0, 1, 1, ec.MODE_FP16_SPLIT)
    # sizes whose tiles could not be counted in 32 bits, or whose packed row block would pass 4 GiB, are refused
    for bad in [(1 << 23, 1 << 23, 32), (1 << 37, 1, 1), (4, 4, 1 << 26)]:
        with pytest.raises(ec.EcgemmError) as err:
            ec.plan_info(*bad, ec.MODE_FP16_SPLIT)
        assert err.value.status == ec.ERR_INVALID_ARG
        with pytest.raises(ec.EcgemmError):
            ec.workspace_size(ec.OP_N, ec.OP_T, *bad, ec.MODE_FP16_SPLIT)
    assert ec.plan_info(1 << 22, 1 << 15, 32, ec.MODE_FP16_SPLIT)["tiles_m"] == 1 << 15     # 2^30 tiles of 128 x 128: still fine


def test_plans_of_random_problems_are_well_formed():
    """Host logic: whatever the cost estimate picks, every tile is accounted for once, slices are at least 512 deep
    and none is empty, there are at most 1024 of them, and the workspace holds the packed operands and the partial sums."""
    import random
    import paper_2203_03341_amd as ec
    rng = random.Random(7)
    for trial in range(400):
        M = int(2 ** rng.uniform(0, 15.5)) + rng.choice([0, 0, 1, 7])
        N = int(2 ** rng.uniform(0, 15.5)) + rng.choice([0, 0, 3])
        K = int(2 ** rng.uniform(0, 17.5)) + rng.choice([0, 0, 5])
        mode = rng.choice([ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL, ec.MODE_FP16_MARKIDIS, ec.MODE_FP32_MFMA])
        p = ec.plan_info(M, N, K, mode)
        case = (M, N, K, mode, p)
        assert p["tiles_m"] == -(-M // p["tile_m"]) and p["tiles_n"] == -(-N // p["tile_n"]), case
        assert p["whole_tiles"] + p["sliced_tiles"] == p["tiles_m"] * p["tiles_n"], case
        assert (p["slices"] == 1) == (p["sliced_tiles"] == 0), case
        assert 1 <= p["column_bands"] <= max(1, p["tiles_n"]) and p["group_m"] in (4, 8), case
        if p["shape"] in (ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED):      # one launch: nothing packed; every tile sliced or none
            tile = 64 if p["shape"] == 3 else 32
            assert p["tile_m"] == p["tile_n"] == tile, case
            assert mode in (ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL) and (K <= 8192 or p["slices"] > 1) and p["tiles_m"] * p["tiles_n"] <= 2048, case
            if p["slices"] == 1:
                assert p["workspace_bytes"] == 0, case
            else:
                tiles = p["tiles_m"] * p["tiles_n"]
                assert p["sliced_tiles"] == tiles and p["slices"] * tiles <= 256 and K // p["slices"] >= 512, case
                assert p["workspace_bytes"] == p["slices"] * tiles * tile * tile * 4, case
                chunks = -(-K // 64)
                per_slice = -(-(-(-chunks // p["slices"])) // 8) * 8          # equal shares rounded up to whole 512-deep runs
                assert per_slice * (p["slices"] - 1) < chunks, case            # the last slice is not empty
            continue
        Kp = -(-K // 32) * 32
        parts = {ec.MODE_FP16_SPLIT: 2, ec.MODE_BF16_FULL: 3, ec.MODE_FP16_MARKIDIS: 2, ec.MODE_FP32_MFMA: 2}[mode]
        packed = (-(-M // 256) * 256 + -(-N // 256) * 256) * Kp * 2 * parts
        partial = p["slices"] * p["sliced_tiles"] * p["tile_m"] * p["tile_n"] * 4 if p["slices"] > 1 else 0
        assert packed + partial <= p["workspace_bytes"] <= packed + partial + 3 * 256, case
        if p["slices"] > 1:
            slots = 256 * (2 if p["tile_m"] == 128 else 1)
            assert p["sliced_tiles"] == (p["tiles_m"] * p["tiles_n"]) % slots, case      # only the leftover tiles are sliced
            assert p["slices"] <= min(64, Kp // 512) and p["slices"] * p["sliced_tiles"] <= 1024, case
            stage = 16 if p["tile_m"] == 128 else 32                                        # depth of an LDS stage
            stages = Kp // stage
            per_slice = -(-stages // p["slices"])
            assert per_slice * (p["slices"] - 1) < stages, case                            # the last slice is not empty


def test_tile_order_reciprocal_arithmetic_agrees_with_division():
    """The kernels locate a tile with multiplications by reciprocals prepared on the host.  For grids of many shapes
    (bands of equal and unequal width, a shorter last group of tile rows, one row, one column, forced orders) every
    tile number must give the coordinates that plain division gives, and the order must visit every tile once."""
    import numpy as np
    import paper_2203_03341_amd as ec
    rng = np.random.default_rng(5)
    problems = [(1, 1, 32), (256, 128, 64), (300, 5000, 96), (5000, 300, 96), (16384, 16384, 256), (4095, 3001, 5003),
                (2304, 4224, 1536), (20000, 130, 40000), (129, 20000, 64), (8192, 8192, 8192)]
    problems += [(int(rng.integers(1, 12000)), int(rng.integers(1, 12000)), int(rng.integers(1, 20000))) for _ in range(60)]
    for mode in (ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL):
        for (M, N, K) in problems:
            p = ec.plan_info(M, N, K, mode)
            if p["shape"] in (ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED):   # one launch: no reciprocal arithmetic
                import pytest
                with pytest.raises(ec.EcgemmError):
                    ec.debug_tile_order(M, N, K, mode)
                continue
            tm, tn, bad = ec.debug_tile_order(M, N, K, mode)
            assert bad == 0, (M, N, K, mode)
            seen = np.zeros((p["tiles_m"], p["tiles_n"]), dtype=np.int32)
            np.add.at(seen, (tm, tn), 1)
            assert seen.min() == 1 and seen.max() == 1, (M, N, K, mode)


def test_workspace_plan_needs_no_gpu():
    """Host logic: operands padded to 256 rows x 32 depth, 2 / 3 / 1 sixteen-bit parts per element, and the output
    tiles left over after whole rounds of the chip's 256 CUs cut into slices along K (one partial tile per slice)."""
    import paper_2203_03341_amd as ec
    n = 16384
    assert ec.workspace_size(ec.OP_N, ec.OP_N, n, n, n, ec.MODE_FP16_SPLIT) == 2 * n * n * 4              # two packed operands, no split-K
    assert ec.workspace_size(ec.OP_N, ec.OP_N, n, n, n, ec.MODE_BF16_FULL) == 2 * n * n * 6
    assert ec.workspace_size(ec.OP_N, ec.OP_N, n, n, n, ec.MODE_FP16_PLAIN) == 2 * n * n * 2
    assert ec.workspace_size(ec.OP_N, ec.OP_N, 1, 1, 1, ec.MODE_FP16_PLAIN) == 2 * 256 * 32 * 2
    assert ec.workspace_size(ec.OP_N, ec.OP_N, 1, 1, 1, ec.MODE_FP16_SPLIT) == 0      # one launch on the FP32 operands
    assert ec.workspace_size(ec.OP_N, ec.OP_N, 0, 5, 5, ec.MODE_FP16_SPLIT) == 0
    # 32 output tiles of 256 x 128 on 256 CUs: every tile is cut into 8 slices along K, one partial tile per slice
    deep = ec.workspace_size(ec.OP_N, ec.OP_N, 1024, 1024, 65536, ec.MODE_FP16_SPLIT)
    assert deep == 2 * 1024 * 65536 * 4 + 8 * 32 * (256 * 128 * 4)
    # 16 x 24 = 384 tiles: 256 are done whole, the other 128 in two slices each
    odd = ec.workspace_size(ec.OP_N, ec.OP_N, 4095, 3001, 5003, ec.MODE_BF16_FULL)
    assert odd == (4096 + 3072) * 5024 * 6 + 2 * 128 * (256 * 128 * 4)
    # shallow K is never sliced
    assert ec.workspace_size(ec.OP_N, ec.OP_N, 4096, 4096, 512, ec.MODE_FP16_SPLIT) == 2 * 4096 * 512 * 4
    import pytest
    with pytest.raises(ec.EcgemmError):
        ec.workspace_size(ec.OP_N, ec.OP_N, -1, 1, 1, ec.MODE_FP16_SPLIT)
    with pytest.raises(ec.EcgemmError):
        ec.workspace_size(ec.OP_N, ec.OP_N, 1, 1, 1, 99)
