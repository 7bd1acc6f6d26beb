"""ctypes front end of the CPU oracle (oracle/etr_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu-baseline leg; never by the product package.  Arguments are
numpy arrays (bf16 tensors travel as uint16 bit patterns).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "etr_ref.cpp")
_LIB = os.path.join(_HERE, "libetr_ref.so")

DT_F32, DT_BF16 = 0, 1
MODE_TCR, MODE_ECR, MODE_BIDIR, MODE_TCR_RANK, MODE_BIDIR_STRICT = 0, 1, 2, 3, 4
COS_FULL, COS_POOLED = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.etr_ref_double_to_bf16.restype = ctypes.c_uint16
        _lib.etr_ref_double_to_bf16.argtypes = [ctypes.c_double]
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _elem(dtype: int):
    return np.float32 if dtype == DT_F32 else np.uint16


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed with status {rc}")


def num_threads() -> int:
    return int(lib().etr_ref_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the oracle's loops use from now on (for the single-core timing of the benchmark)."""
    lib().etr_ref_set_num_threads(int(n))


def double_to_bf16(v: float) -> int:
    return int(lib().etr_ref_double_to_bf16(float(v)))


def route(x: np.ndarray, w_emb: np.ndarray, D: int, dtype: int, cos_mode: int = COS_FULL):
    T, d = x.shape
    E, P = w_emb.shape
    assert x.dtype == _elem(dtype) and w_emb.dtype == np.float32 and P * D == d
    score = np.empty((T, E), np.float32)
    gate = np.empty((T, E), np.float32)
    _check(lib().etr_ref_route(T, d, E, D, dtype, cos_mode, _p(x), _p(w_emb), _p(score), _p(gate)), "route")
    return score, gate


def select(score: np.ndarray, k: int, capacity: int, mode: int):
    T, E = score.shape
    assert score.dtype == np.float32
    topk = np.full((T, max(k, 1)), -1, np.int32)
    slot_of = np.empty((T, E), np.int32)
    slot_token = np.empty((E, capacity), np.int32)
    counts = np.empty((E,), np.int32)
    _check(lib().etr_ref_select(T, E, k, capacity, mode, _p(score), _p(topk), _p(slot_of), _p(slot_token),
                                _p(counts)), "select")
    return topk, slot_of, slot_token, counts


def select_adaptive(score: np.ndarray, k: int, capacity: int, mode: int, sum_threshold: float):
    T, E = score.shape
    assert score.dtype == np.float32
    topk = np.full((T, max(k, 1)), -1, np.int32)
    slot_of = np.empty((T, E), np.int32)
    slot_token = np.empty((E, capacity), np.int32)
    counts = np.empty((E,), np.int32)
    _check(lib().etr_ref_select_adaptive(T, E, k, capacity, mode, _p(score), ctypes.c_float(sum_threshold), _p(topk),
                                         _p(slot_of), _p(slot_token), _p(counts)), "select_adaptive")
    return topk, slot_of, slot_token, counts


def dispatch(x: np.ndarray, slot_token: np.ndarray, counts: np.ndarray, dtype: int):
    T, d = x.shape
    E, C = slot_token.shape
    xp = np.empty((E, C, d), _elem(dtype))
    _check(lib().etr_ref_dispatch(T, d, E, C, dtype, _p(x), _p(slot_token), _p(counts), _p(xp)), "dispatch")
    return xp


def ffn_rows(rows: np.ndarray, expert_of_row: np.ndarray, w_gate, w_up, w_down, dtype: int):
    n, d = rows.shape
    E, H, d2 = w_gate.shape
    assert d2 == d and w_down.shape == (E, d, H) and w_up.shape == (E, H, d)
    eid = np.ascontiguousarray(expert_of_row, np.int32)
    y = np.empty((n, d), np.float64)
    _check(lib().etr_ref_ffn_rows(n, d, H, dtype, _p(rows), _p(eid), _p(w_gate), _p(w_up), _p(w_down), _p(y)),
           "ffn_rows")
    return y


def expert_ffn(xp: np.ndarray, counts: np.ndarray, w_gate, w_up, w_down, dtype: int):
    E, C, d = xp.shape
    H = w_gate.shape[1]
    yp = np.empty((E, C, d), np.float64)
    _check(lib().etr_ref_expert_ffn(d, E, C, H, dtype, _p(xp), _p(counts), _p(w_gate), _p(w_up), _p(w_down),
                                    _p(yp)), "expert_ffn")
    return yp


def combine(yp: np.ndarray, gate: np.ndarray, slot_of: np.ndarray, dtype: int, gate_norm: int = 0):
    E, C, d = yp.shape
    T = gate.shape[0]
    assert yp.dtype == np.float64
    out = np.empty((T, d), _elem(dtype))
    _check(lib().etr_ref_combine(T, d, E, C, dtype, _p(yp), _p(gate), _p(slot_of), _p(out), gate_norm), "combine")
    return out


def moe_forward(x, w_emb, w_gate, w_up, w_down, *, D: int, k: int, capacity: int, dtype: int, mode: int,
                cos_mode: int = COS_FULL, score_in: Optional[np.ndarray] = None,
                tokens: Optional[np.ndarray] = None, gate_norm: int = 0):
    """Returns a dict: out (rows for `tokens`, or all T), score, gate, topk, slot_of, slot_token, counts."""
    T, d = x.shape
    E = w_emb.shape[0]
    H = w_gate.shape[1]
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, np.int32)
        n_tok = int(tokens.shape[0])
    else:
        n_tok = -1
    n_out = T if n_tok < 0 else n_tok
    res = dict(
        out=np.empty((n_out, d), _elem(dtype)),
        score=np.empty((T, E), np.float32), gate=np.empty((T, E), np.float32),
        topk=np.full((T, max(k, 1)), -1, np.int32), slot_of=np.empty((T, E), np.int32),
        slot_token=np.empty((E, capacity), np.int32), counts=np.empty((E,), np.int32))
    if score_in is not None:
        assert score_in.dtype == np.float32 and score_in.shape == (T, E)
    _check(lib().etr_ref_moe_forward(
        T, d, E, D, k, capacity, H, dtype, mode, cos_mode, _p(x), _p(w_emb), _p(w_gate), _p(w_up), _p(w_down),
        _p(score_in), _p(tokens), n_tok, _p(res["out"]), _p(res["score"]), _p(res["gate"]), _p(res["topk"]),
        _p(res["slot_of"]), _p(res["slot_token"]), _p(res["counts"]), gate_norm), "moe_forward")
    return res


def route_stats(gate: np.ndarray, slot_of: np.ndarray, counts: np.ndarray, target: np.ndarray):
    """Returns load[E], mean_gate[E] (float64), kl (float), n_unrouted (int)."""
    T, E = gate.shape
    assert gate.dtype == np.float32 and target.dtype == np.float32 and slot_of.dtype == np.int32
    load, mg = np.empty(E, np.float64), np.empty(E, np.float64)
    kl, un = np.zeros(1, np.float64), np.zeros(1, np.int32)
    _check(lib().etr_ref_route_stats(T, E, _p(gate), _p(slot_of), _p(np.ascontiguousarray(counts, np.int32)),
                                     _p(target), _p(load), _p(mg), _p(kl), _p(un)), "route_stats")
    return load, mg, float(kl[0]), int(un[0])


def capacity_lower_bound(score: np.ndarray, d: int):
    """Returns (dmax, capacity) of the Remark's C_min for this batch of scores."""
    T, E = score.shape
    assert score.dtype == np.float32
    dm, c = np.zeros(1, np.float32), np.zeros(1, np.int32)
    _check(lib().etr_ref_capacity_lower_bound(T, E, d, _p(score), _p(dm), _p(c)), "capacity_lower_bound")
    return float(dm[0]), int(c[0])


def backward_tokens(x, w_emb, w_gate, w_up, w_down, slot_of, dout, tokens, *, D: int, dtype: int,
                    cos_mode: int = COS_FULL, gate_norm: int = 0):
    """Per-token part of the layer's backward (routing tables fixed): dx[n][d], dgate[n][E], dscore[n][E], float64."""
    T, d = x.shape
    E, H = w_gate.shape[0], w_gate.shape[1]
    tokens = np.ascontiguousarray(tokens, np.int32)
    n = int(tokens.shape[0])
    assert slot_of.dtype == np.int32 and slot_of.shape == (T, E) and dout.shape == (T, d) and dout.dtype == x.dtype
    dx, dg, ds = np.empty((n, d), np.float64), np.empty((n, E), np.float64), np.empty((n, E), np.float64)
    _check(lib().etr_ref_backward_tokens(T, d, E, D, H, dtype, cos_mode, _p(x), _p(w_emb), _p(w_gate), _p(w_up),
                                         _p(w_down), _p(slot_of), _p(dout), _p(tokens), n, _p(dx), _p(dg), _p(ds),
                                         gate_norm),
           "backward_tokens")
    return dx, dg, ds


def backward_hidden_units(x, w_emb, w_gate, w_up, w_down, slot_of, dout, unit_expert, unit_index, *, D: int,
                          dtype: int, cos_mode: int = COS_FULL, gate_norm: int = 0):
    """Per-hidden-unit part of the backward: rows of dWg and dWu and columns of dWd, each [n][d] float64."""
    T, d = x.shape
    E, H = w_gate.shape[0], w_gate.shape[1]
    ue = np.ascontiguousarray(unit_expert, np.int32)
    ui = np.ascontiguousarray(unit_index, np.int32)
    n = int(ue.shape[0])
    assert ui.shape == ue.shape and slot_of.dtype == np.int32 and dout.dtype == x.dtype
    gw, uw, dw = (np.empty((n, d), np.float64) for _ in range(3))
    _check(lib().etr_ref_backward_hidden_units(T, d, E, D, H, dtype, cos_mode, _p(x), _p(w_emb), _p(w_gate), _p(w_up),
                                               _p(w_down), _p(slot_of), _p(dout), _p(ue), _p(ui), n, _p(gw), _p(uw),
                                               _p(dw), gate_norm), "backward_hidden_units")
    return gw, uw, dw


def moe_backward(x, w_emb, w_gate, w_up, w_down, slot_of, dout, *, D: int, dtype: int, cos_mode: int = COS_FULL,
                 gate_norm: int = 0):
    """Whole gradient (small sizes only): dict dx[T][d], dgate, dscore [T][E], dw_gate, dw_up [E][H][d], dw_down [E][d][H]."""
    T, d = x.shape
    E, H = w_gate.shape[0], w_gate.shape[1]
    dx, dg, ds = backward_tokens(x, w_emb, w_gate, w_up, w_down, slot_of, dout, np.arange(T), D=D, dtype=dtype,
                                 cos_mode=cos_mode, gate_norm=gate_norm)
    ue, ui = np.repeat(np.arange(E), H), np.tile(np.arange(H), E)
    gw, uw, dw = backward_hidden_units(x, w_emb, w_gate, w_up, w_down, slot_of, dout, ue, ui, D=D, dtype=dtype,
                                       cos_mode=cos_mode, gate_norm=gate_norm)
    return dict(dx=dx, dgate=dg, dscore=ds, dw_gate=gw.reshape(E, H, d), dw_up=uw.reshape(E, H, d),
                dw_down=np.ascontiguousarray(dw.reshape(E, H, d).transpose(0, 2, 1)))


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 values (pure bit reinterpretation)."""
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    return a.astype(np.float64) if dtype == DT_F32 else bf16_bits_to_f64(a)
