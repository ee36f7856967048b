"""Host-side checks that need no GPU: the library loads, exports every symbol the public
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import re
from pathlib import Path

import numpy as np
import pytest

from paper_2605_30325_amd import veda

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    if not veda.LIB_PATH.exists():
        from paper_2605_30325_amd import build
        build.build()
    return veda.load()


def test_every_declared_symbol_is_exported(lib):
    header = (ROOT / "include" / "veda.h").read_text()
    declared = set(re.findall(r"\b(veda_[a-z_]+)\s*\(", header))
    assert declared == set(veda.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_public_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, no C++ and no HIP types
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "veda.h"\nint main(void) { return (int)sizeof(veda_problem) == 0; }\n')
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", f"-I{ROOT / 'include'}",
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_status_strings(lib):
    assert lib.veda_status_string(0) == b"ok"
    assert b"workspace" in lib.veda_status_string(veda.VEDA_ERR_WORKSPACE)


def _problem(shape_rows, heads=2, tile_tokens=64, head_dim=64, dtype=0, T=4, H=8, W=8):
    arr = np.ascontiguousarray(shape_rows, np.int32)
    p = veda.veda_problem(1, heads, head_dim, T, H, W, tile_tokens,
                          arr.ctypes.data_as(C.POINTER(C.c_int32)), dtype)
    return p, arr


def test_plan_create_rejects_bad_problems(lib):
    out = C.c_void_p()
    bad = [
        _problem([[4, 4, 4], [4, 4, 2]]),                 # product != B
        _problem([[4, 4, 4], [0, 8, 8]]),                 # non-positive extent
        _problem([[4, 4, 4], [4, 4, 4]], T=0),            # empty grid
        _problem([[4, 4, 4], [4, 4, 4]], dtype=7),        # unknown dtype
    ]
    for p, keep in bad:
        assert lib.veda_plan_create(C.byref(p), C.byref(out)) == veda.VEDA_ERR_INVALID_ARG
        assert out.value is None
    p, keep = _problem([[4, 4, 8], [4, 4, 8]], tile_tokens=128)            # 128-token tiles are bf16 only
    assert lib.veda_plan_create(C.byref(p), C.byref(out)) == veda.VEDA_ERR_UNSUPPORTED
    p, keep = _problem([[4, 8, 8], [4, 8, 8]], tile_tokens=256, dtype=1)
    assert lib.veda_plan_create(C.byref(p), C.byref(out)) == veda.VEDA_ERR_UNSUPPORTED
    p, keep = _problem([[4, 4, 8], [4, 4, 4]], tile_tokens=128, dtype=1)   # product != B for head 1
    assert lib.veda_plan_create(C.byref(p), C.byref(out)) == veda.VEDA_ERR_INVALID_ARG
    p, keep = _problem([[4, 4, 4], [4, 4, 4]], head_dim=96)
    assert lib.veda_plan_create(C.byref(p), C.byref(out)) == veda.VEDA_ERR_UNSUPPORTED
    assert lib.veda_plan_create(None, C.byref(out)) == veda.VEDA_ERR_INVALID_ARG


def test_stage_calls_reject_null_plan(lib):
    s = veda.veda_strides(0, 0, 64)
    assert lib.veda_tile_layout(None, None, s, 0, None, None, None, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_score(None, None, None, None, None, None, 0.125, None, None, 0, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_select(None, None, None, None, None, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_sparse_attn_fwd(None, None, None, None, None, None, None, 0.125, None, s, None, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_layout_stats(None, None, s, None, None, None, None, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_sparse_attn_fwd_q_tokens(None, None, s, None, None, None, None, None, 0.125, None, s, None,
                                             None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_sparse_attn_fwd_qk_tokens(None, None, s, None, s, None, None, None, None, 0.125, None, s, None,
                                              None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_score_stats(None, None, None, None, None, 0.125, None, None, 0, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_score_closed_form(None, None, None, None, 0.5, None, None, 0, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_score_select(None, None, None, None, None, None, 0.125, None, None, None, None, 0,
                                      None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_score_select_stats(None, None, None, None, None, 0.125, None, None, None, None, 0,
                                            None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_plan_fused_workspace_bytes(None, None, None) == 0
    assert lib.veda_tile_heatmap(None, None, None, None, 0.125, None, 0, None, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_tile_recall(None, None, None, None, None, None, 0, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_output_sqerr(None, None, s, None, s, None, None, 0, None) == veda.VEDA_ERR_INVALID_ARG
    assert lib.veda_plan_tiles(None, 0) == -1 and lib.veda_plan_total_tiles(None) == -1
    lib.veda_plan_destroy(None)
