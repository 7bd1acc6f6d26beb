"""Seeded synthetic inputs for the ETR MoE layer.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: no pooling, no scoring, no selection, no FFN.
It only produces tensors: tokens, orthonormal expert embeddings and FFN
weights, with the shapes and value structure of the five workloads.

Random numbers come from a counter-based generator written here (SplitMix64
finaliser over ``seed + index`` -> two 24-bit uniforms -> Box-Muller), so the
value at a given (seed, index) does not depend on chunking or on how many
values were drawn before it.  The integer part is bit-identical on every
device; the fp32 ``log``/``cos`` may differ in the last ulp between CPU and
GPU, which is why parity tests always hand the *same bytes* to both sides
(generated once, copied).

The inputs stand in for hidden states of a trained Mixtral-style model, which
the paper's experiments use (Sec. Experimental Setup) and which are not
available: isotropic tokens model the "before training" picture and clustered
tokens (same-cluster cosine about 0.8) the "after training" one (Appendix,
Token Feature Distribution).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import torch

MODE_TCR, MODE_ECR, MODE_BIDIR, MODE_TCR_RANK, MODE_BIDIR_STRICT = 0, 1, 2, 3, 4
COS_FULL, COS_POOLED = 0, 1
DT_F32, DT_BF16 = 0, 1

BASE_SEED = 2406000230

_STREAMS = {"tokens": 0, "emb": 1, "w_gate": 2, "w_up": 3, "w_down": 4, "bias": 5, "cluster": 6, "dout": 7}


@dataclass(frozen=True)
class EtrShape:
    """One workload: sizes, dtype, phase and the token recipe."""
    name: str
    cfg_id: int
    T: int
    d: int
    E: int
    D: int
    k: int
    capacity: int
    H: int
    dtype: int                  # DT_F32 / DT_BF16
    mode: int                   # MODE_*
    recipe: str                 # "iso" | "bias" | "cluster" | "zipf"
    n_centroids: int = 0
    E_global: int = 0           # > E when only a local share of experts is present
    cos: int = COS_FULL
    capacity_sweep: Tuple[int, ...] = field(default_factory=tuple)

    @property
    def P(self) -> int:
        return self.d // self.D

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == DT_F32 else torch.bfloat16

    def with_(self, **kw) -> "EtrShape":
        return replace(self, **kw)


def _ceil(a: float) -> int:
    return int(math.ceil(a - 1e-9))


CONFIGS: Dict[str, EtrShape] = {
    # tiny fp32 layer; run in all three phases by the tests
    "cfg1": EtrShape("cfg1", 1, T=512, d=256, E=8, D=8, k=1, capacity=_ceil(1.25 * 1 * 512 / 8), H=512,
                     dtype=DT_F32, mode=MODE_TCR, recipe="iso"),
    # bf16, token choice, skewed load so that some experts overflow
    "cfg2": EtrShape("cfg2", 2, T=8192, d=2048, E=16, D=16, k=2, capacity=_ceil(1.0 * 2 * 8192 / 16), H=5632,
                     dtype=DT_BF16, mode=MODE_TCR, recipe="bias"),
    # bf16, expert choice, clustered tokens
    "cfg3": EtrShape("cfg3", 3, T=16384, d=4096, E=16, D=32, k=1, capacity=int(1.25 * 16384 / 16), H=11008,
                     dtype=DT_BF16, mode=MODE_ECR, recipe="cluster", n_centroids=16),
    # bf16, bidirectional, capacity schedule
    "cfg4": EtrShape("cfg4", 4, T=32768, d=4096, E=32, D=32, k=2, capacity=2048, H=2816,
                     dtype=DT_BF16, mode=MODE_BIDIR, recipe="cluster", n_centroids=32,
                     capacity_sweep=(2048, 1792, 1536, 1280, 1024)),
    # bf16, the local 8 of 64 experts, Zipf-skewed
    "cfg5": EtrShape("cfg5", 5, T=65536, d=4096, E=8, D=64, k=4, capacity=_ceil(1.1 * 4 * 65536 / 8), H=1408,
                     dtype=DT_BF16, mode=MODE_BIDIR, recipe="zipf", E_global=64),
}


# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------
def _i64(v: int) -> int:
    """Reinterpret an unsigned 64-bit constant as a signed python int."""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _i64(0x9E3779B97F4A7C15)
_M1 = _i64(0xBF58476D1CE4E5B9)
_M2 = _i64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _splitmix64(counter: torch.Tensor) -> torch.Tensor:
    z = counter * _GOLDEN + _GOLDEN           # int64 arithmetic wraps: that is the intent
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def stream_seed(cfg_id: int, stream: str) -> int:
    return BASE_SEED + 10 * cfg_id + _STREAMS[stream]


def uniform_bits(seed: int, start: int, n: int, device) -> torch.Tensor:
    """n 64-bit words for counters start..start+n-1 of the stream `seed` (int64 tensor)."""
    idx = torch.arange(start, start + n, dtype=torch.int64, device=device)
    key = _i64((seed * 0xD6E8FEB86659FD93) & ((1 << 64) - 1))
    return _splitmix64(_splitmix64(idx ^ key) + idx)


def normal(seed: int, n: int, device="cpu", start: int = 0, chunk: int = 1 << 24) -> torch.Tensor:
    """n standard normals (fp32), value i depends only on (seed, start+i)."""
    out = torch.empty(n, dtype=torch.float32, device=device)
    for off in range(0, n, chunk):
        m = min(chunk, n - off)
        bits = uniform_bits(seed, start + off, m, device)
        u1 = ((_lsr(bits, 40) & 0xFFFFFF).to(torch.float32) + 1.0) * (1.0 / 16777216.0)   # (0,1]
        u2 = (_lsr(bits, 16) & 0xFFFFFF).to(torch.float32) * (1.0 / 16777216.0)           # [0,1)
        out[off:off + m] = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
    return out


def uniform01(seed: int, n: int, device="cpu", start: int = 0) -> torch.Tensor:
    bits = uniform_bits(seed, start, n, device)
    return (_lsr(bits, 11).to(torch.float64) * (1.0 / 9007199254740992.0))


# ----------------------------------------------------------------------------
# pieces
# ----------------------------------------------------------------------------
def orthonormal_embeddings(seed: int, E: int, P: int, E_global: int = 0) -> torch.Tensor:
    """Rows = orthonormal expert embeddings, fp32 [E][P] (CPU).

    A seeded Gaussian [P][n] is QR-factorised in fp64 (signs fixed so that
    diag(R) > 0); the embeddings are the first E columns of Q, transposed.
    With E_global > E the factorisation is done for all E_global experts and
    the first E rows are returned (the local share of a larger expert set).
    """
    n = max(E, E_global)
    if n > P:
        raise ValueError(f"{n} orthonormal rows do not exist in dimension {P}")
    a = normal(seed, P * n, "cpu").to(torch.float64).reshape(P, n)
    q, r = torch.linalg.qr(a, mode="reduced")
    sgn = torch.sign(torch.diagonal(r))
    sgn[sgn == 0] = 1.0
    q = q * sgn.unsqueeze(0)
    w = q.t().contiguous().to(torch.float32)[:E].contiguous()
    return w


def lifted_unit_directions(w_emb: torch.Tensor, D: int) -> torch.Tensor:
    """Unit vectors in R^d whose grouped mean is proportional to each embedding row:
    every pooled coordinate is repeated D times, then the row is normalised. fp32 [E][d]."""
    u = w_emb.to(torch.float64).repeat_interleave(D, dim=1)
    u = u / u.norm(dim=1, keepdim=True)
    return u.to(torch.float32)


def ffn_weight(seed: int, shape, dtype: torch.dtype, device, std: float = 0.02) -> torch.Tensor:
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(n, dtype=dtype, device=device)
    chunk = 1 << 26
    for off in range(0, n, chunk):
        m = min(chunk, n - off)
        out[off:off + m] = (normal(seed, m, device, start=off) * std).to(dtype)
    return out.reshape(*shape)


def make_tokens(shape: EtrShape, w_emb: torch.Tensor, device="cpu",
                T: Optional[int] = None) -> torch.Tensor:
    """Tokens [T][d] in the workload's dtype, by its recipe."""
    T = shape.T if T is None else T
    d, D, E = shape.d, shape.D, shape.E
    cid = shape.cfg_id
    z = normal(stream_seed(cid, "tokens"), T * d, device).reshape(T, d)
    if shape.recipe == "iso":
        x = z
    elif shape.recipe == "bias":
        # a fixed half-sigma-scale shift of each expert's projection: skewed load
        nu = normal(stream_seed(cid, "bias"), E, "cpu")
        u = lifted_unit_directions(w_emb, D)                       # [E][d]
        shift = (0.5 * nu).unsqueeze(1).mul(u).sum(0)               # [d]
        x = z + shift.to(device).unsqueeze(0)
    elif shape.recipe == "cluster":
        nc = shape.n_centroids
        mu = normal(stream_seed(cid, "bias"), nc * d, device).reshape(nc, d)
        c = (uniform01(stream_seed(cid, "cluster"), T, device) * nc).to(torch.int64).clamp_(max=nc - 1)
        x = mu[c] + 0.5 * z
    elif shape.recipe == "zipf":
        u = lifted_unit_directions(w_emb, D).to(device)             # [E][d]
        p = torch.tensor([(c + 1.0) ** -1.1 for c in range(E)], dtype=torch.float64)
        cdf = torch.cumsum(p / p.sum(), 0).to(device)
        r = uniform01(stream_seed(cid, "cluster"), T, device)
        c = torch.searchsorted(cdf, r).clamp_(max=E - 1)
        x = math.sqrt(d) * u[c] + z
    else:
        raise ValueError(shape.recipe)
    return x.to(shape.torch_dtype).contiguous()


def make_inputs(shape: EtrShape, device="cpu", with_weights: bool = True) -> Dict[str, torch.Tensor]:
    """All tensors of one layer call. x, w_gate, w_up, w_down in the workload's
    dtype; w_emb fp32. Layouts: x[T][d], w_emb[E][d/D], w_gate/w_up[E][H][d],
    w_down[E][d][H] (all row-major, contraction dimension contiguous)."""
    cid = shape.cfg_id
    w_emb = orthonormal_embeddings(stream_seed(cid, "emb"), shape.E, shape.P, shape.E_global)
    out = {"w_emb": w_emb.to(device), "x": make_tokens(shape, w_emb, device)}
    if with_weights:
        dt = shape.torch_dtype
        E, H, d = shape.E, shape.H, shape.d
        out["w_gate"] = ffn_weight(stream_seed(cid, "w_gate"), (E, H, d), dt, device)
        out["w_up"] = ffn_weight(stream_seed(cid, "w_up"), (E, H, d), dt, device)
        out["w_down"] = ffn_weight(stream_seed(cid, "w_down"), (E, d, H), dt, device)
    return out


def make_upstream_gradient(shape: EtrShape, device="cpu") -> torch.Tensor:
    """Upstream gradient d loss / d out for the backward pass: i.i.d. N(0, 1), [T][d] in the workload's dtype
    (what a following layer's backward hands over has no structure the method relies on)."""
    g = normal(stream_seed(shape.cfg_id, "dout"), shape.T * shape.d, device)
    return g.view(shape.T, shape.d).to(shape.torch_dtype)


def small_variant(shape: EtrShape, T: int, H: Optional[int] = None, d: Optional[int] = None) -> EtrShape:
    """Same recipe and expert structure at a reduced token count (and optionally
    reduced widths), with the capacity rescaled by T; used where the oracle has
    to finish in seconds."""
    cap = max(1, _ceil(shape.capacity * T / shape.T))
    kw = dict(T=T, capacity=cap, name=f"{shape.name}-T{T}")
    if H is not None:
        kw["H"] = H
    if d is not None:
        kw["d"] = d
    if shape.capacity_sweep:
        kw["capacity_sweep"] = tuple(max(1, _ceil(c * T / shape.T)) for c in shape.capacity_sweep)
    return shape.with_(**kw)
