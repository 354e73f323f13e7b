"""The shared library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ecgemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ecgemm_[a-z_]+)\s*\(", text)))


def test_header_declares_the_north_star_entry_points():
    names = _declared_functions()
    for required in ("ecgemm_create", "ecgemm_sgemm", "ecgemm_destroy"):
        assert required in names


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


def test_workspace_plan_needs_no_gpu():
    """Host logic: operands padded to 256 rows x 32 depth, 2 / 3 / 1 sixteen-bit parts per element, and K divided
    among blocks (with one partial C per slice) only when the tiles alone cannot fill the chip."""
    import paper_2203_03341_amd as ec
    n = 16384
    assert ec.workspace_size(n, n, n, ec.MODE_FP16_SPLIT) == 2 * n * n * 4              # two packed operands, no split-K
    assert ec.workspace_size(n, n, n, ec.MODE_BF16_FULL) == 2 * n * n * 6
    assert ec.workspace_size(n, n, n, ec.MODE_FP16_PLAIN) == 2 * n * n * 2
    assert ec.workspace_size(1, 1, 1, ec.MODE_FP16_SPLIT) == 2 * 256 * 32 * 4
    assert ec.workspace_size(0, 5, 5, ec.MODE_FP16_SPLIT) == 0
    deep = ec.workspace_size(1024, 1024, 65536, ec.MODE_FP16_SPLIT)
    operands = 2 * 1024 * 65536 * 4
    slices = (deep - operands) // (1024 * 1024 * 4)
    assert deep > operands and (deep - operands) % (1024 * 1024 * 4) == 0 and 2 <= slices <= 64
    assert ec.workspace_size(4095, 3001, 5003, ec.MODE_BF16_FULL) == (4096 + 3072) * 5024 * 6
    import pytest
    with pytest.raises(ec.EcgemmError):
        ec.workspace_size(-1, 1, 1, ec.MODE_FP16_SPLIT)
    with pytest.raises(ec.EcgemmError):
        ec.workspace_size(1, 1, 1, 99)
