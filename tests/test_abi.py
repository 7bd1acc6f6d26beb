"""The C-ABI library: it loads, exports every function the header declares, and its host-side
validation returns the documented statuses before anything is launched. CPU only: no call
here gets past validation."""
import ctypes
import os
import re

import pytest

from paper_2406_00023_amd import binding as B
from paper_2406_00023_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2406_00023_amd.build import build
        build()
    return B.load_library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "etr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(etr_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_config_struct_matches_header():
    assert ctypes.sizeof(B.EtrConfig) == 44
    assert [f[0] for f in B.EtrConfig._fields_] == ["T", "d", "E", "D", "k", "capacity", "H", "dtype", "mode", "cos",
                                                    "gate_norm"]


def test_status_strings(lib):
    texts = {lib.etr_status_string(i).decode() for i in range(8)}
    assert len(texts) == 8 and "ok" in texts


def test_workspace_queries(lib):
    for name, s in I.CONFIGS.items():
        cfg = B.make_config(s)
        total, sel, ffn = B.etr_workspace_bytes(cfg), B.etr_select_workspace_bytes(cfg), B.etr_ffn_workspace_bytes(cfg)
        elt = 4 if s.dtype == I.DT_F32 else 2
        assert ffn >= s.E * s.capacity * s.H * elt
        # yp always; the permuted token buffer only where the fused call cannot gather inside GEMM-1 (fp32 here)
        n_row_buffers = 2 if s.dtype == I.DT_F32 else 1
        assert total >= sel + ffn + n_row_buffers * s.E * s.capacity * s.d * elt
        assert total % 256 == 0
    big = B.etr_workspace_bytes(B.make_config(I.CONFIGS["cfg5"]))
    assert big < 8 * 2 ** 30


def _bad(**kw):
    return B.make_config(I.CONFIGS["cfg1"].with_(**kw))


@pytest.mark.parametrize("cfg,status", [
    (_bad(T=0), 2), (_bad(D=7), 2), (_bad(k=0), 2), (_bad(k=9), 2), (_bad(capacity=0), 2), (_bad(H=-8), 2),
    (_bad(E=65, d=65 * 8), 3), (_bad(d=260, D=4), 3), (_bad(H=508), 3), (_bad(dtype=2), 3), (_bad(mode=5), 3), (_bad(mode=-1), 3),
    (_bad(cos=2), 3), (_bad(d=32768, D=1, E=64), 3),
])
def test_invalid_configs(lib, cfg, status):
    assert B.etr_workspace_bytes(cfg) == 0
    null = ctypes.c_void_p(0)
    assert lib.etr_route(ctypes.byref(cfg), null, null, null, null, null) == status
    assert lib.etr_select(ctypes.byref(cfg), null, null, null, null, null, null, 0, null) == status
    assert lib.etr_moe_forward(ctypes.byref(cfg), *([null] * 13), 0, null) == status


def test_ecr_ignores_k(lib):
    cfg = B.make_config(I.CONFIGS["cfg1"].with_(k=0), mode=I.MODE_ECR)
    assert B.etr_workspace_bytes(cfg) > 0


def test_null_and_alignment(lib):
    cfg = B.make_config(I.CONFIGS["cfg1"])
    null, ok, odd = ctypes.c_void_p(0), ctypes.c_void_p(4096), ctypes.c_void_p(4100)
    c = ctypes.byref(cfg)
    assert lib.etr_route(None, ok, ok, ok, ok, null) == 1
    assert lib.etr_route(c, null, ok, ok, ok, null) == 1
    assert lib.etr_route(c, ok, ok, ok, odd, null) == 5
    assert lib.etr_dispatch(c, ok, ok, null, ok, null) == 1
    assert lib.etr_combine(c, ok, odd, ok, ok, null) == 5
    assert lib.etr_expert_ffn(c, ok, ok, ok, ok, ok, ok, null, 0, null) == 1
    # workspace too small is reported before any launch
    assert lib.etr_select(c, ok, null, ok, ok, ok, ok, 16, null) == 4
    assert lib.etr_expert_ffn(c, ok, ok, ok, ok, ok, ok, ok, 16, null) == 4
    assert lib.etr_moe_forward(c, ok, ok, ok, ok, ok, ok, *([null] * 6), ok, 16, null) == 4


def test_noalloc_select_validates_before_anything_else(lib):
    """The allocation-free entry point rejects bad arguments and oversized configurations on the host."""
    null, ok, odd = ctypes.c_void_p(0), ctypes.c_void_p(4096), ctypes.c_void_p(4100)
    cfg = B.make_config(I.CONFIGS["cfg1"])
    c = ctypes.byref(cfg)
    assert lib.etr_select_noalloc(None, ok, null, ok, ok, ok, null) == 1
    assert lib.etr_select_noalloc(c, null, null, ok, ok, ok, null) == 1
    assert lib.etr_select_noalloc(c, ok, null, ok, odd, ok, null) == 5
    limit = B.etr_select_noalloc_max_bytes()
    assert limit == 8 << 20
    for s in I.CONFIGS.values():                       # every benchmark workload fits
        assert B.etr_select_workspace_bytes(B.make_config(s)) <= limit
    big = B.make_config(I.CONFIGS["cfg5"].with_(T=1 << 20, capacity=1 << 20))
    assert B.etr_select_workspace_bytes(big) > limit
    assert lib.etr_select_noalloc(ctypes.byref(big), ok, null, ok, ok, ok, null) == 7


def test_binding_refuses_missing_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.load_library()
