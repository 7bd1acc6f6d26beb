"""Helpers for the GPU parity tests: run the HIP stages through the Python binding and
hand identical bytes to the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

from paper_2406_00023_amd import binding as B
from paper_2406_00023_amd import inputs as I

# output tolerance: max |a-b| / max |b| over the whole output (scale-relative)
TOL_OUT = {I.DT_F32: 1e-4, I.DT_BF16: 2e-2}
# fp32 summation-order noise on a cosine in [-1, 1]
TOL_SCORE = 4e-6
TOL_GATE = 4e-6


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host numpy; bf16 travels as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def scale_rel_err(a: np.ndarray, b: np.ndarray) -> float:
    den = float(np.max(np.abs(b)))
    return float(np.max(np.abs(a - b))) / (den if den > 0 else 1.0)


def row_rel_err(a: np.ndarray, b: np.ndarray) -> float:
    """Largest per-row error, each row on its own scale: max_j |a-b| / max(max_j |b_row|, 1e-3 rms(b)).
    A row whose values are small (a low gate weight) cannot hide behind the largest row of the tensor;
    the floor keeps rows that are (nearly) zero from dividing by nothing."""
    a2, b2 = a.reshape(-1, a.shape[-1]), b.reshape(-1, b.shape[-1])
    floor = 1e-3 * float(np.sqrt(np.mean(b2 * b2)))
    den = np.maximum(np.max(np.abs(b2), axis=1), floor if floor > 0 else 1.0)
    return float(np.max(np.max(np.abs(a2 - b2), axis=1) / den))


def floored_elementwise_err(a: np.ndarray, b: np.ndarray) -> float:
    """Element-wise relative error with the floor atol = 1e-3 rms(b) (reported, not asserted: an element at a
    zero crossing of a row carries the rounding error of its neighbours)."""
    floor = 1e-3 * float(np.sqrt(np.mean(b * b)))
    return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), floor if floor > 0 else 1.0)))


class GpuLayer:
    """Owns the device tensors of one layer call and runs stages through the C ABI."""

    def __init__(self, shape: I.EtrShape, tensors=None, mode=None, capacity=None, cos=None, gate_norm=0):
        self.shape = shape
        self.cfg = B.make_config(shape, mode=mode, capacity=capacity, cos=cos, gate_norm=gate_norm)
        dev = "cuda"
        t = tensors if tensors is not None else I.make_inputs(shape, dev)
        self.t = {k: v.to(dev) for k, v in t.items()}
        T, E, C, d, k = shape.T, shape.E, self.cfg.capacity, shape.d, max(shape.k, 1)
        dt = shape.torch_dtype
        self.score = torch.empty(T, E, dtype=torch.float32, device=dev)
        self.gate = torch.empty(T, E, dtype=torch.float32, device=dev)
        self.topk = torch.full((T, k), -7, dtype=torch.int32, device=dev)
        self.slot_of = torch.full((T, E), -7, dtype=torch.int32, device=dev)
        self.slot_token = torch.full((E, C), -7, dtype=torch.int32, device=dev)
        self.counts = torch.full((E,), -7, dtype=torch.int32, device=dev)
        self.out = torch.empty(T, d, dtype=dt, device=dev)

    # ---- stage calls -------------------------------------------------------------
    def route(self):
        B.etr_route(self.cfg, self.t["x"], self.t["w_emb"], self.score, self.gate)

    def select(self, score=None):
        ws = B.alloc_workspace(B.etr_select_workspace_bytes(self.cfg))
        B.etr_select(self.cfg, self.score if score is None else score, self.topk, self.slot_of, self.slot_token,
                     self.counts, ws)

    def dispatch(self):
        E, C, d = self.shape.E, self.cfg.capacity, self.shape.d
        # poison so that rows the kernel must not touch are recognisable
        self.xp = torch.full((E, C, d), 7.0, dtype=self.shape.torch_dtype, device="cuda")
        B.etr_dispatch(self.cfg, self.t["x"], self.slot_token, self.counts, self.xp)

    def expert_ffn(self):
        E, C, d = self.shape.E, self.cfg.capacity, self.shape.d
        self.yp = torch.full((E, C, d), 7.0, dtype=self.shape.torch_dtype, device="cuda")
        ws = B.alloc_workspace(B.etr_ffn_workspace_bytes(self.cfg))
        B.etr_expert_ffn(self.cfg, self.xp, self.counts, self.t["w_gate"], self.t["w_up"], self.t["w_down"], self.yp, ws)

    def combine(self):
        B.etr_combine(self.cfg, self.yp, self.gate, self.slot_of, self.out)

    def forward(self, keep_tables=True):
        ws = B.alloc_workspace(B.etr_workspace_bytes(self.cfg))
        kw = dict(score=self.score, gate=self.gate, topk_expert=self.topk, slot_of=self.slot_of,
                  slot_token=self.slot_token, counts=self.counts) if keep_tables else {}
        B.etr_moe_forward(self.cfg, self.t["x"], self.t["w_emb"], self.t["w_gate"], self.t["w_up"], self.t["w_down"],
                          self.out, ws, **kw)
        torch.cuda.synchronize()

    # ---- host copies ---------------------------------------------------------------
    def host_inputs(self):
        return {k: to_np(v) for k, v in self.t.items()}


def check_routing_against_oracle(oracle, layer: GpuLayer, hx: dict, check_topk=True):
    """Staged parity of the routing half.  Returns the oracle's tables computed from the
    GPU's own fp32 scores (they must equal the GPU's tables byte for byte)."""
    s, cfg = layer.shape, layer.cfg
    g_score, g_gate = to_np(layer.score), to_np(layer.gate)
    o_score, o_gate = oracle.route(hx["x"], hx["w_emb"], s.D, s.dtype, cfg.cos)
    assert np.max(np.abs(g_score - o_score)) <= TOL_SCORE, np.max(np.abs(g_score - o_score))
    assert np.max(np.abs(g_gate - o_gate)) <= TOL_GATE, np.max(np.abs(g_gate - o_gate))
    topk, slot_of, slot_token, counts = oracle.select(g_score, s.k, cfg.capacity, cfg.mode)
    if check_topk and cfg.mode != I.MODE_ECR:
        np.testing.assert_array_equal(to_np(layer.topk), topk)
    np.testing.assert_array_equal(to_np(layer.counts), counts)
    np.testing.assert_array_equal(to_np(layer.slot_of), slot_of)
    np.testing.assert_array_equal(to_np(layer.slot_token), slot_token)
    # fully independent routing (oracle scores): differences can only come from near-ties
    _, so2, _, _ = oracle.select(o_score, s.k, cfg.capacity, cfg.mode)
    ndiff = int(((so2 >= 0) != (slot_of >= 0)).sum())
    return dict(score=g_score, gate=g_gate, slot_of=slot_of, slot_token=slot_token, counts=counts, ndiff=ndiff)


def check_output_against_oracle(oracle, layer: GpuLayer, hx: dict, g_score: np.ndarray, tokens=None):
    """Layer output vs the oracle continued from the GPU's scores, on all or on sampled tokens."""
    s, cfg = layer.shape, layer.cfg
    ref = oracle.moe_forward(hx["x"], hx["w_emb"], hx["w_gate"], hx["w_up"], hx["w_down"], D=s.D, k=s.k,
                             capacity=cfg.capacity, dtype=s.dtype, mode=cfg.mode, cos_mode=cfg.cos, score_in=g_score,
                             tokens=tokens, gate_norm=cfg.gate_norm)
    got = to_np(layer.out)
    if tokens is not None:
        got = got[np.asarray(tokens)]
    a, b = oracle.to_f64(got, s.dtype), oracle.to_f64(ref["out"], s.dtype)
    err = scale_rel_err(a, b)
    assert err <= TOL_OUT[s.dtype], err
    # the same bound for every row on its own scale (Eq. 1 gives each token its own gate weights)
    row_err = row_rel_err(a, b)
    assert row_err <= TOL_OUT[s.dtype], row_err
    layer.last_errors = dict(scale=err, per_row=row_err, elementwise_floored=floored_elementwise_err(a, b))
    # tokens kept by no expert give exact zero rows
    sel = ref["slot_of"] if tokens is None else ref["slot_of"][np.asarray(tokens)]
    dropped = (sel >= 0).sum(1) == 0
    assert np.all(a[dropped] == 0)
    return err
