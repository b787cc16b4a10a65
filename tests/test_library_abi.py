"""The C-ABI library loads on a machine without a GPU and exports every symbol
that include/pkv.h declares; host-only entry points behave."""

import ctypes
import os
import re

import pytest

from paper_2602_02579_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pkv_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree_on_the_symbol_list():
    assert declared_symbols() == sorted(api.EXPORTED_SYMBOLS)
    for name in api.EXPORTED_SYMBOLS:
        assert hasattr(api, name)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(api.library_path()):
        pytest.skip("libpkv.so not built (run python -m paper_2602_02579_amd.build)")
    lib = ctypes.CDLL(api.library_path())
    for name in declared_symbols():
        assert getattr(lib, name) is not None


def test_host_only_entry_points():
    if not os.path.exists(api.library_path()):
        pytest.skip("libpkv.so not built")
    assert api.pkv_version() >= 100
    assert api.pkv_status_string(0) == "ok"
    assert "workspace" in api.pkv_status_string(4)
    cfg = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")
    assert api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, cfg, 32768, 128) % 256 == 0
    assert api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, cfg, 32768, 128) > 0
    assert api.pkv_workspace_bytes(api.CALL_TOPK_SELECT, cfg, 16384, 0) == 0
    assert api.pkv_workspace_bytes(api.CALL_TOPK_SELECT, cfg, 131072, 0) > 0
    bad = api.LayerCfg(32, 7, 128, 4096, 5e5, "bf16")
    assert api.pkv_workspace_bytes(api.CALL_QUERY_SCORE, bad, 32768, 128) == 0


def test_argument_errors_are_reported_without_a_gpu():
    """Null pointers and bad sizes are rejected on the host before any launch."""
    if not os.path.exists(api.library_path()):
        pytest.skip("libpkv.so not built")
    lib = api.load_library()
    c = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")._c()
    assert lib.pkv_rope_restore(ctypes.byref(c), None, None, None, 0, 5, None) == 1
    assert lib.pkv_rope_restore(ctypes.byref(c), None, None, None, 0, -1, None) == 2
    assert lib.pkv_rope_restore(ctypes.byref(c), None, None, None, 0, 0, None) == 0
    assert lib.pkv_rope_restore(None, None, None, None, 0, 5, None) == 1
    assert lib.pkv_topk_select(None, 10, 11, None, None, 0, None) == 2
    assert lib.pkv_topk_select(None, 10, 0, None, None, 0, None) == 0
    assert lib.pkv_topk_select(None, 10, 3, None, None, 0, None) == 1
    assert lib.pkv_scatter_kv(ctypes.byref(c), None, None, None, None, None, 5, 3, None) == 2
    assert lib.pkv_sparse_row_attn(ctypes.byref(c), None, None, None, None, None, None,
                                   0, 10, 0.0, None, 0, None) == 0
    assert lib.pkv_sparse_row_attn(ctypes.byref(c), None, None, None, None, None, None,
                                   4, 10, 0.0, None, 0, None) == 1
    c2 = api.LayerCfg(32, 8, 72, 4096, 5e5, "bf16")._c()
    assert lib.pkv_rope_restore(ctypes.byref(c2), None, None, None, 0, 5, None) == 3
    # sizes whose 32-bit byte offsets or column counts would wrap inside the kernels are
    # refused, not run: head_dim * keys * 2 bytes >= 2**32; (rows or query tokens) * heads
    # beyond 2**31 - 1
    assert lib.pkv_sparse_row_attn(ctypes.byref(c), None, None, None, None, None, None,
                                   4, 1 << 24, 0.0, None, 0, None) == 3
    assert lib.pkv_sparse_row_attn(ctypes.byref(c), None, None, None, None, None, None,
                                   4, (1 << 24) - 64, 0.0, None, 0, None) == 1
    assert lib.pkv_sparse_row_attn(ctypes.byref(c), None, None, None, None, None, None,
                                   1 << 27, 1024, 0.0, None, 0, None) == 3
    # the entry point with built-in scratch refuses what does not fit it, before any device call
    assert lib.pkv_query_score_static(None, None, None, None, 128, 32768, 0.0, 0, None) == 1
    assert lib.pkv_query_score_static(ctypes.byref(c), None, None, None, 256, 131072, 0.0, 0,
                                      None) == 4
    wide = api.LayerCfg(4096, 8, 128, 4096, 5e5, "bf16")._c()
    assert lib.pkv_query_score(ctypes.byref(wide), None, None, None, 1 << 20, 1024, 0.0, 0,
                               None, 0, None) == 3
    assert lib.pkv_query_score(ctypes.byref(wide), None, None, None, 1 << 10, 1024, 0.0, 0,
                               None, 0, None) == 1


def test_glue_and_variant_entry_points_check_their_arguments_on_the_host():
    if not os.path.exists(api.library_path()):
        pytest.skip("libpkv.so not built")
    import torch
    lib = api.load_library()
    bf = api.PKV_BF16
    # scratch sizing: split contractions (few rows) need fp32 partials, large launches and
    # fp32 storage do not; invalid sizes give 0
    few = api.pkv_glue_workspace_bytes(torch.bfloat16, 128, 4096, 14336)
    assert few > 0 and few % 256 == 0
    assert api.pkv_glue_workspace_bytes(torch.float32, 128, 4096, 14336) == 0
    assert api.pkv_glue_workspace_bytes(torch.bfloat16, 100000, 4096, 14336) == 0
    assert lib.pkv_glue_workspace_bytes(bf, -1, 4096, 14336) == 0
    # null pointers / sizes / dtype are refused before any launch; m == 0 is a no-op
    assert lib.pkv_rmsnorm_rows(bf, None, None, None, 1e-5, None, 4, 64, None) == 1
    assert lib.pkv_rmsnorm_rows(bf, None, None, None, 1e-5, None, 4, 60, None) == 3
    assert lib.pkv_rmsnorm_rows(bf, None, None, None, -1.0, None, 4, 64, None) == 2
    assert lib.pkv_rmsnorm_rows(9, None, None, None, 1e-5, None, 4, 64, None) == 3
    assert lib.pkv_rmsnorm_rows(bf, None, None, None, 1e-5, None, 0, 64, None) == 0
    assert lib.pkv_gather_rows(bf, None, None, None, 4, 64, None) == 1
    assert lib.pkv_gather_rows(bf, None, None, None, 4, 63, None) == 3
    assert lib.pkv_gather_rows(bf, None, None, None, -4, 64, None) == 2
    assert lib.pkv_linear_rows(bf, None, None, None, None, 4, 64, 64, None, 0, None) == 1
    assert lib.pkv_linear_rows(bf, None, None, None, None, 4, 0, 64, None, 0, None) == 2
    assert lib.pkv_swiglu_rows(bf, None, None, None, None, 0, 64, 64, None, 0, None) == 0
    c = api.LayerCfg(32, 8, 128, 4096, 5e5, "bf16")._c()
    var = api._CVariant(None, None, None, 1, None, 1e-6)      # q_norm without k_norm
    assert lib.pkv_gather_qkv_proj_ex(ctypes.byref(c), None, None, None, None, None, None,
                                      ctypes.byref(var), None, None, None, 4, None, 0, None) == 1
    assert lib.pkv_gather_qkv_proj_ex(ctypes.byref(c), None, None, None, None, None, None,
                                      None, None, None, None, 0, None, 0, None) == 0
    assert lib.pkv_gather_qkv_proj_scatter(ctypes.byref(c), None, None, None, None, None, None,
                                           None, None, None, None, None, 5, 3, None, 0,
                                           None) == 2          # more rows than cache rows
    assert lib.pkv_gather_qkv_proj_scatter(ctypes.byref(c), None, None, None, None, None, None,
                                           None, None, None, None, None, 3, 5, None, 0,
                                           None) == 1


def test_a_missing_library_fails_loudly_and_nothing_falls_back():
    """The binding has no CPU path: with the shared library absent, the first call
    raises (checked in a fresh interpreter so that this process keeps its library)."""
    import subprocess
    import sys
    code = (
        "import os, sys\n"
        "os.environ['PKV_LIBRARY'] = '/nonexistent/libpkv.so'\n"
        "import torch\n"
        "from paper_2602_02579_amd import api\n"
        "try:\n"
        "    api.pkv_topk_select(torch.zeros(8), 2, torch.zeros(2, dtype=torch.int32))\n"
        "except RuntimeError as e:\n"
        "    assert 'missing' in str(e) and 'no CPU fallback' in str(e), str(e)\n"
        "    sys.exit(0)\n"
        "sys.exit(1)\n")
    res = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True)
    assert res.returncode == 0, res.stdout + res.stderr
