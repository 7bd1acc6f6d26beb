"""Thin ctypes binding of the C-ABI library declared in include/etr.h.

Argument marshalling only: torch tensors provide device memory and the current
stream; every step of the layer runs in the HIP kernels.  There is no CPU
fallback: if the shared library is missing or a status is non-zero the call
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .inputs import EtrShape

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libetr_hip.so")

EXPORTS = ("etr_workspace_bytes", "etr_select_workspace_bytes", "etr_ffn_workspace_bytes", "etr_status_string",
           "etr_route", "etr_select", "etr_dispatch", "etr_expert_ffn", "etr_combine", "etr_moe_forward",
           "etr_moe_forward_profiled", "etr_select_adaptive", "etr_stats_workspace_bytes", "etr_route_stats",
           "etr_capacity_lower_bound", "etr_backward_workspace_bytes", "etr_moe_backward",
           "etr_moe_forward_train", "etr_select_noalloc", "etr_select_noalloc_max_bytes")
N_STAGE_EVENTS = 7
STAGE_NAMES = ("route", "select", "dispatch", "ffn_gate_up", "ffn_down", "combine")


class EtrConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "E", "D", "k", "capacity", "H", "dtype", "mode", "cos",
                                             "gate_norm")]


class EtrError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn}: status {status} ({text})")
        self.status = status


_lib = None


def load_library():
    """Load libetr_hip.so (built in-tree by paper_2406_00023_amd/build.py). Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2406_00023_amd.build` "
                                "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, cp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(EtrConfig)
    for name in ("etr_workspace_bytes", "etr_select_workspace_bytes", "etr_ffn_workspace_bytes",
                 "etr_stats_workspace_bytes", "etr_backward_workspace_bytes"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [cp]
    lib.etr_select_noalloc_max_bytes.restype = sz
    lib.etr_select_noalloc_max_bytes.argtypes = []
    lib.etr_status_string.restype = ctypes.c_char_p
    lib.etr_status_string.argtypes = [ctypes.c_int]
    sigs = {
        "etr_route": [cp, vp, vp, vp, vp, vp],
        "etr_select": [cp, vp, vp, vp, vp, vp, vp, sz, vp],
        "etr_select_noalloc": [cp, vp, vp, vp, vp, vp, vp],
        "etr_dispatch": [cp, vp, vp, vp, vp, vp],
        "etr_expert_ffn": [cp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "etr_combine": [cp, vp, vp, vp, vp, vp],
        "etr_moe_forward": [cp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "etr_select_adaptive": [cp, vp, vp, ctypes.c_float, vp, vp, vp, vp, vp, sz, vp],
        "etr_route_stats": [cp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "etr_capacity_lower_bound": [cp, vp, vp, vp, vp, sz, vp],
        "etr_moe_backward": [cp] + [vp] * 20 + [sz, vp],
        "etr_moe_forward_train": [cp] + [vp] * 15 + [sz, vp],
        "etr_moe_forward_profiled": [cp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp,
                                     ctypes.POINTER(ctypes.c_void_p)],
    }
    for name, args in sigs.items():
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = args
    _lib = lib
    return lib


def make_config(shape: EtrShape, mode: Optional[int] = None, capacity: Optional[int] = None,
                cos: Optional[int] = None, gate_norm: int = 0) -> EtrConfig:
    return EtrConfig(shape.T, shape.d, shape.E, shape.D, shape.k,
                     shape.capacity if capacity is None else capacity, shape.H, shape.dtype,
                     shape.mode if mode is None else mode, shape.cos if cos is None else cos, gate_norm)


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn: str, status: int):
    if status != 0:
        raise EtrError(fn, status, load_library().etr_status_string(status).decode())


def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def etr_workspace_bytes(cfg: EtrConfig) -> int:
    return int(load_library().etr_workspace_bytes(ctypes.byref(cfg)))


def etr_select_workspace_bytes(cfg: EtrConfig) -> int:
    return int(load_library().etr_select_workspace_bytes(ctypes.byref(cfg)))


def etr_ffn_workspace_bytes(cfg: EtrConfig) -> int:
    return int(load_library().etr_ffn_workspace_bytes(ctypes.byref(cfg)))


def etr_route(cfg, x, w_emb, score, gate):
    _check("etr_route", load_library().etr_route(ctypes.byref(cfg), _ptr(x), _ptr(w_emb), _ptr(score), _ptr(gate),
                                                 _stream()))


def etr_select(cfg, score, topk_expert, slot_of, slot_token, counts, ws):
    _check("etr_select", load_library().etr_select(ctypes.byref(cfg), _ptr(score), _ptr(topk_expert), _ptr(slot_of),
                                                   _ptr(slot_token), _ptr(counts), _ptr(ws), _nbytes(ws), _stream()))


def etr_select_noalloc_max_bytes() -> int:
    return int(load_library().etr_select_noalloc_max_bytes())


def etr_select_noalloc(cfg, score, topk_expert, slot_of, slot_token, counts):
    _check("etr_select_noalloc", load_library().etr_select_noalloc(
        ctypes.byref(cfg), _ptr(score), _ptr(topk_expert), _ptr(slot_of), _ptr(slot_token), _ptr(counts), _stream()))


def etr_select_adaptive(cfg, score, capacity_dev, affinity_sum_threshold, topk_expert, slot_of, slot_token, counts, ws):
    _check("etr_select_adaptive", load_library().etr_select_adaptive(
        ctypes.byref(cfg), _ptr(score), _ptr(capacity_dev), ctypes.c_float(affinity_sum_threshold), _ptr(topk_expert),
        _ptr(slot_of), _ptr(slot_token), _ptr(counts), _ptr(ws), _nbytes(ws), _stream()))


def etr_stats_workspace_bytes(cfg: EtrConfig) -> int:
    return int(load_library().etr_stats_workspace_bytes(ctypes.byref(cfg)))


def etr_route_stats(cfg, gate, slot_of, counts, target, load_frac, mean_gate, kl, n_unrouted, ws):
    _check("etr_route_stats", load_library().etr_route_stats(
        ctypes.byref(cfg), _ptr(gate), _ptr(slot_of), _ptr(counts), _ptr(target), _ptr(load_frac), _ptr(mean_gate),
        _ptr(kl), _ptr(n_unrouted), _ptr(ws), _nbytes(ws), _stream()))


def etr_capacity_lower_bound(cfg, score, dmax, capacity, ws):
    _check("etr_capacity_lower_bound", load_library().etr_capacity_lower_bound(
        ctypes.byref(cfg), _ptr(score), _ptr(dmax), _ptr(capacity), _ptr(ws), _nbytes(ws), _stream()))


def etr_backward_workspace_bytes(cfg: EtrConfig) -> int:
    return int(load_library().etr_backward_workspace_bytes(ctypes.byref(cfg)))


def etr_moe_backward(cfg, x, w_emb, w_gate, w_up, w_down, score, gate, slot_of, slot_token, counts, dout, dx, dw_gate,
                     dw_up, dw_down, ws, dgate=None, dscore=None, a_saved=None, b_saved=None):
    _check("etr_moe_backward", load_library().etr_moe_backward(
        ctypes.byref(cfg), _ptr(x), _ptr(w_emb), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(score), _ptr(gate),
        _ptr(slot_of), _ptr(slot_token), _ptr(counts), _ptr(dout), _ptr(dx), _ptr(dw_gate), _ptr(dw_up), _ptr(dw_down),
        _ptr(dgate), _ptr(dscore), _ptr(a_saved), _ptr(b_saved), _ptr(ws), _nbytes(ws), _stream()))


def etr_moe_forward_train(cfg, x, w_emb, w_gate, w_up, w_down, out, a_save, b_save, ws, score=None, gate=None,
                          topk_expert=None, slot_of=None, slot_token=None, counts=None):
    _check("etr_moe_forward_train", load_library().etr_moe_forward_train(
        ctypes.byref(cfg), _ptr(x), _ptr(w_emb), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(score),
        _ptr(gate), _ptr(topk_expert), _ptr(slot_of), _ptr(slot_token), _ptr(counts), _ptr(a_save), _ptr(b_save),
        _ptr(ws), _nbytes(ws), _stream()))


def etr_dispatch(cfg, x, slot_token, counts, xp):
    _check("etr_dispatch", load_library().etr_dispatch(ctypes.byref(cfg), _ptr(x), _ptr(slot_token), _ptr(counts),
                                                       _ptr(xp), _stream()))


def etr_expert_ffn(cfg, xp, counts, w_gate, w_up, w_down, yp, ws):
    _check("etr_expert_ffn", load_library().etr_expert_ffn(ctypes.byref(cfg), _ptr(xp), _ptr(counts), _ptr(w_gate),
                                                           _ptr(w_up), _ptr(w_down), _ptr(yp), _ptr(ws), _nbytes(ws),
                                                           _stream()))


def etr_combine(cfg, yp, gate, slot_of, out):
    _check("etr_combine", load_library().etr_combine(ctypes.byref(cfg), _ptr(yp), _ptr(gate), _ptr(slot_of), _ptr(out),
                                                     _stream()))


def etr_moe_forward(cfg, x, w_emb, w_gate, w_up, w_down, out, ws, score=None, gate=None, topk_expert=None,
                    slot_of=None, slot_token=None, counts=None):
    _check("etr_moe_forward", load_library().etr_moe_forward(
        ctypes.byref(cfg), _ptr(x), _ptr(w_emb), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(score),
        _ptr(gate), _ptr(topk_expert), _ptr(slot_of), _ptr(slot_token), _ptr(counts), _ptr(ws), _nbytes(ws), _stream()))


class StageEvents:
    """ETR_N_STAGE_EVENTS HIP events owned by the caller, for etr_moe_forward_profiled.
    Created and read through the HIP runtime directly so that they are recorded on exactly
    the stream the kernels run on."""

    def __init__(self, only=None):
        """only: iterable of boundary indices to create (the others stay NULL and are not recorded)."""
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.handles = (ctypes.c_void_p * N_STAGE_EVENTS)()
        for i in (range(N_STAGE_EVENTS) if only is None else only):
            ev = ctypes.c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.handles[i] = ev

    def stage_ms(self):
        """Milliseconds of each stage (after the last event has completed)."""
        if self._hip.hipEventSynchronize(self.handles[N_STAGE_EVENTS - 1]) != 0:
            raise RuntimeError("hipEventSynchronize failed")
        out = []
        for i in range(N_STAGE_EVENTS - 1):
            ms = ctypes.c_float()
            if self._hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[i], self.handles[i + 1]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            out.append(float(ms.value))
        return out

    def __del__(self):
        try:
            for h in self.handles:
                if h:
                    self._hip.hipEventDestroy(h)
        except Exception:
            pass


def record_event(events: StageEvents, i: int):
    """Record event i of `events` on torch's current stream (measurement helper)."""
    hip = events._hip
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    if hip.hipEventRecord(events.handles[i], _stream()) != 0:
        raise RuntimeError("hipEventRecord failed")


def elapsed_ms(events: StageEvents, i: int, j: int) -> float:
    ms = ctypes.c_float()
    if events._hip.hipEventSynchronize(events.handles[j]) != 0:
        raise RuntimeError("hipEventSynchronize failed")
    if events._hip.hipEventElapsedTime(ctypes.byref(ms), events.handles[i], events.handles[j]) != 0:
        raise RuntimeError("hipEventElapsedTime failed")
    return float(ms.value)


def etr_moe_forward_profiled(cfg, x, w_emb, w_gate, w_up, w_down, out, ws, events: StageEvents, score=None, gate=None,
                             topk_expert=None, slot_of=None, slot_token=None, counts=None):
    _check("etr_moe_forward_profiled", load_library().etr_moe_forward_profiled(
        ctypes.byref(cfg), _ptr(x), _ptr(w_emb), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), _ptr(score),
        _ptr(gate), _ptr(topk_expert), _ptr(slot_of), _ptr(slot_token), _ptr(counts), _ptr(ws), _nbytes(ws), _stream(),
        events.handles))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch as a uint8 tensor (torch allocations are 256-byte aligned or better)."""
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)
