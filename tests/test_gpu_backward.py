"""GPU parity of the backward pass (through the C ABI) against the CPU oracle on identical bytes.

The routing tables handed to the backward are the GPU's own (already byte-identical to the oracle's
selection on the GPU's scores); gradients are compared per tensor with max|a-b| / max|b|:
1e-4 for fp32, 2e-2 for bf16 (the tolerance of the forward output)."""
import numpy as np
import pytest
import torch

from paper_2406_00023_amd import binding as B
from paper_2406_00023_amd import inputs as I

pytestmark = pytest.mark.gpu

TCR, ECR, BIDIR = I.MODE_TCR, I.MODE_ECR, I.MODE_BIDIR
FULL, POOLED = I.COS_FULL, I.COS_POOLED


@pytest.fixture(scope="module")
def H():
    import gpu_helpers
    assert torch.cuda.is_available()
    B.load_library()
    return gpu_helpers


def _say(msg):
    print(msg, flush=True)


class Backward:
    """Runs forward routing + backward on the GPU and keeps the results."""

    def __init__(self, H, shape, mode, cos=None, gate_norm=0):
        self.H, self.shape = H, shape
        self.L = L = H.GpuLayer(shape, mode=mode, cos=cos, gate_norm=gate_norm)
        L.route(); L.select()
        dev, dt = "cuda", shape.torch_dtype
        E, Hh, d, T = shape.E, shape.H, shape.d, shape.T
        self.dout = I.make_upstream_gradient(shape, dev)
        # poisoned outputs: everything the call is meant to overwrite must be overwritten
        self.dx = torch.full((T, d), 7.0, dtype=dt, device=dev)
        self.dwg = torch.full((E, Hh, d), 7.0, dtype=dt, device=dev)
        self.dwu = torch.full((E, Hh, d), 7.0, dtype=dt, device=dev)
        self.dwd = torch.full((E, d, Hh), 7.0, dtype=dt, device=dev)
        self.dgate = torch.full((T, E), 7.0, dtype=torch.float32, device=dev)
        self.dscore = torch.full((T, E), 7.0, dtype=torch.float32, device=dev)
        ws = B.alloc_workspace(B.etr_backward_workspace_bytes(L.cfg))
        ws.fill_(0xFF)                    # NaN patterns: nothing may be read before it is written
        t = L.t
        B.etr_moe_backward(L.cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], L.score, L.gate, L.slot_of,
                           L.slot_token, L.counts, self.dout, self.dx, self.dwg, self.dwu, self.dwd, ws,
                           dgate=self.dgate, dscore=self.dscore)
        torch.cuda.synchronize()

    def host(self):
        hx = self.L.host_inputs()
        hx["dout"] = self.H.to_np(self.dout)
        hx["slot_of"] = self.H.to_np(self.L.slot_of)
        return hx


def _err(H, oracle, got, ref, dtype):
    a = oracle.to_f64(H.to_np(got), dtype) if got.dtype != torch.float32 or dtype == I.DT_F32 else H.to_np(got).astype(np.float64)
    return H.scale_rel_err(a, ref)


SMALL = {
    "cfg1": lambda: I.CONFIGS["cfg1"],
    "cfg2s": lambda: I.small_variant(I.CONFIGS["cfg2"], T=1100, d=512, H=704),
    "cfg3s": lambda: I.small_variant(I.CONFIGS["cfg3"], T=900, d=1024, H=1032),
    "cfg4s": lambda: I.small_variant(I.CONFIGS["cfg4"], T=1500, d=1024, H=328),
    "cfg5s": lambda: I.small_variant(I.CONFIGS["cfg5"], T=700, H=200),
    # whole column tiles (H % 128 == 0, d % 256 == 0): the recomputation and the training forward run on the
    # 64-wide persistent kernel (two-product and pre-activation-keeping epilogues, rows gathered through LDS)
    "cfg2w": lambda: I.small_variant(I.CONFIGS["cfg2"], T=1300, d=512, H=640),
    "cfg5w": lambda: I.small_variant(I.CONFIGS["cfg5"], T=900, H=256),
    # a capacity of 8192 rows and whole 256-column tiles for both u and the input gradient: the two products against
    # a weight matrix run on the row-major kernel with the weight transposed once (the overloaded experts of this
    # recipe keep a few thousand rows, the others few)
    "cfg2r": lambda: I.CONFIGS["cfg2"].with_(T=12000, d=256, H=256, capacity=8192, name="cfg2-rows"),
    # from that capacity on the weight-gradient products also fetch the rows of dOut and x through slot_token
    # themselves; here with a capacity that is no multiple of 64 (row numbers past the end of an expert's slot list),
    # a ragged last column tile of dW_down and experts of very different sizes
    "cfg2q": lambda: I.CONFIGS["cfg2"].with_(T=9000, d=256, H=200, capacity=8200, name="cfg2-rows-ragged"),
}


@pytest.mark.parametrize("name,mode,cos", [("cfg1", TCR, FULL), ("cfg1", ECR, POOLED), ("cfg1", BIDIR, FULL),
                                           ("cfg2s", TCR, FULL), ("cfg3s", ECR, FULL), ("cfg4s", BIDIR, POOLED),
                                           ("cfg5s", BIDIR, FULL), ("cfg2w", TCR, FULL), ("cfg5w", BIDIR, POOLED),
                                           ("cfg2r", TCR, FULL), ("cfg2r", BIDIR, POOLED), ("cfg2q", BIDIR, FULL),
                                           ("cfg2q", ECR, FULL)])
def test_backward_small_all_gradients(H, oracle, name, mode, cos):
    shape = SMALL[name]()
    _say(f"backward case {name} mode={mode} cos={cos} T={shape.T} d={shape.d} E={shape.E} C={shape.capacity} H={shape.H}")
    bw = Backward(H, shape, mode, cos)
    hx = bw.host()
    ref = oracle.moe_backward(hx["x"], hx["w_emb"], hx["w_gate"], hx["w_up"], hx["w_down"], hx["slot_of"], hx["dout"],
                              D=shape.D, dtype=shape.dtype, cos_mode=cos)
    tol = H.TOL_OUT[shape.dtype]
    errs = {
        "dx": _err(H, oracle, bw.dx, ref["dx"], shape.dtype),
        "dw_gate": _err(H, oracle, bw.dwg, ref["dw_gate"], shape.dtype),
        "dw_up": _err(H, oracle, bw.dwu, ref["dw_up"], shape.dtype),
        "dw_down": _err(H, oracle, bw.dwd, ref["dw_down"], shape.dtype),
        "dgate": H.scale_rel_err(H.to_np(bw.dgate).astype(np.float64), ref["dgate"]),
        "dscore": H.scale_rel_err(H.to_np(bw.dscore).astype(np.float64), ref["dscore"]),
    }
    _say(f"  errors {errs}")
    for k, v in errs.items():
        assert v <= tol, (k, v)
    # a token kept by no expert gets an exactly zero input gradient
    dropped = (hx["slot_of"] >= 0).sum(1) == 0
    assert np.all(oracle.to_f64(H.to_np(bw.dx), shape.dtype)[dropped] == 0)
    # experts that keep nothing get exactly zero weight gradients
    for e in np.nonzero(H.to_np(bw.L.counts) == 0)[0]:
        assert not H.to_np(bw.dwg)[e].any() and not H.to_np(bw.dwd)[e].any()


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_backward_full_size_sampled(H, oracle, name):
    """Full-size gradients on samples the oracle computes one by one, laid out over the tiles the grouped products
    schedule: one token in every 256-row tile of every expert's buffer (the last kept row included) plus a random
    sample for dx / dgate / dscore; one hidden unit in every 128-wide tile of H of every expert for the weight
    gradients (a row of dW_gate and dW_up and a column of dW_down each, all d entries)."""
    shape = I.CONFIGS[name]
    _say(f"backward full size {name}")
    bw = Backward(H, shape, shape.mode)
    hx = bw.host()
    rng = np.random.default_rng(7)
    counts, slot_token = H.to_np(bw.L.counts), H.to_np(bw.L.slot_token)
    toks = set(rng.choice(shape.T, 24, replace=False).tolist())
    for e in range(shape.E):
        n = int(counts[e])
        for lo in range(0, n, 256):
            toks.add(int(slot_token[e, int(rng.integers(lo, min(lo + 256, n)))]))
        if n:
            toks.add(int(slot_token[e, n - 1]))
    tokens = np.array(sorted(toks), np.int32)
    dx, dg, ds = oracle.backward_tokens(hx["x"], hx["w_emb"], hx["w_gate"], hx["w_up"], hx["w_down"], hx["slot_of"],
                                        hx["dout"], tokens, D=shape.D, dtype=shape.dtype)
    tol = H.TOL_OUT[shape.dtype]
    got_dx = oracle.to_f64(H.to_np(bw.dx), shape.dtype)[tokens]
    e1 = H.scale_rel_err(got_dx, dx)
    e1r = H.row_rel_err(got_dx, dx)
    e2 = H.scale_rel_err(H.to_np(bw.dgate).astype(np.float64)[tokens], dg)
    e3 = H.scale_rel_err(H.to_np(bw.dscore).astype(np.float64)[tokens], ds)
    _say(f"  {len(tokens)} tokens: dx {e1} (per row {e1r}) dgate {e2} dscore {e3}")
    assert e1 <= tol and e1r <= tol and e2 <= tol and e3 <= tol
    n_ht = (shape.H + 127) // 128
    ue = np.repeat(np.arange(shape.E), n_ht).astype(np.int32)
    lo = np.tile(np.arange(n_ht) * 128, shape.E)
    ui = (lo + rng.integers(0, 128, lo.shape[0])).clip(max=shape.H - 1).astype(np.int32)
    gw, uw, dw = oracle.backward_hidden_units(hx["x"], hx["w_emb"], hx["w_gate"], hx["w_up"], hx["w_down"], hx["slot_of"],
                                              hx["dout"], ue, ui, D=shape.D, dtype=shape.dtype)
    g_gw = oracle.to_f64(H.to_np(bw.dwg)[ue, ui], shape.dtype)
    g_uw = oracle.to_f64(H.to_np(bw.dwu)[ue, ui], shape.dtype)
    g_dw = oracle.to_f64(H.to_np(bw.dwd)[ue, :, ui], shape.dtype)
    e4, e5, e6 = H.scale_rel_err(g_gw, gw), H.scale_rel_err(g_uw, uw), H.scale_rel_err(g_dw, dw)
    _say(f"  {len(ue)} hidden units: dw_gate {e4} dw_up {e5} dw_down {e6}")
    assert e4 <= tol and e5 <= tol and e6 <= tol


@pytest.mark.parametrize("name", ["cfg1", "cfg2s", "cfg3s", "odd", "cfg2w", "cfg5w"])
def test_training_forward_keeps_pre_activations(H, oracle, name):
    """etr_moe_forward_train gives the bytes of etr_moe_forward, and the backward fed with the kept
    pre-activations gives the bytes of the backward that recomputes them."""
    shape = (I.small_variant(I.CONFIGS["cfg2"], T=300, d=272, H=328) if name == "odd" else SMALL[name]())
    _say(f"training forward {name} T={shape.T} d={shape.d} E={shape.E} C={shape.capacity} H={shape.H}")
    bw = Backward(H, shape, shape.mode)                 # recomputing backward on the routing of route + select
    L, cfg, t = bw.L, bw.L.cfg, bw.L.t
    dev, dt = "cuda", shape.torch_dtype
    T, E, C, d, Hh = shape.T, shape.E, cfg.capacity, shape.d, shape.H
    out_plain = torch.empty(T, d, dtype=dt, device=dev)
    out_train = torch.empty(T, d, dtype=dt, device=dev)
    a = torch.full((E, C, Hh), 7.0, dtype=dt, device=dev)
    b = torch.full((E, C, Hh), 7.0, dtype=dt, device=dev)
    ws = B.alloc_workspace(B.etr_workspace_bytes(cfg))
    B.etr_moe_forward(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out_plain, ws)
    slot_of = torch.empty_like(L.slot_of)
    B.etr_moe_forward_train(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], out_train, a, b, ws,
                            slot_of=slot_of)
    torch.cuda.synchronize()
    assert torch.equal(out_plain, out_train)
    assert torch.equal(slot_of, L.slot_of)
    # the kept values are W_gate x and W_up x of the kept rows (rows past counts[e] untouched)
    hx = bw.host()
    counts = H.to_np(L.counts)
    st = H.to_np(L.slot_token)
    e = int(np.argmax(counts))
    rows = hx["x"][st[e, :counts[e]]]
    xa = oracle.to_f64(rows, shape.dtype)
    ref_a = xa @ oracle.to_f64(hx["w_gate"][e], shape.dtype).T
    got_a = oracle.to_f64(H.to_np(a)[e, :counts[e]], shape.dtype)
    assert H.scale_rel_err(got_a, ref_a) <= H.TOL_OUT[shape.dtype]
    if counts[e] < C:
        assert torch.all(a[e, counts[e]:] == 7.0) and torch.all(b[e, counts[e]:] == 7.0)
    dx2, dwg2, dwu2, dwd2 = (torch.empty_like(v) for v in (bw.dx, bw.dwg, bw.dwu, bw.dwd))
    wsb = B.alloc_workspace(B.etr_backward_workspace_bytes(cfg))
    B.etr_moe_backward(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], L.score, L.gate, L.slot_of,
                       L.slot_token, L.counts, bw.dout, dx2, dwg2, dwu2, dwd2, wsb, a_saved=a, b_saved=b)
    torch.cuda.synchronize()
    for got, want, nm in ((dx2, bw.dx, "dx"), (dwg2, bw.dwg, "dw_gate"), (dwu2, bw.dwu, "dw_up"), (dwd2, bw.dwd, "dw_down")):
        assert torch.equal(got, want), nm


def test_backward_with_an_empty_and_a_one_row_expert(H, oracle):
    """Hand-edited routing tables on the shape that takes the transposition-free path: one expert keeps nothing
    (its weight gradients must be exact zeros), one keeps a single row."""
    shape = SMALL["cfg2s"]()
    _say("backward with edited tables (empty expert, one-row expert)")
    bw = Backward(H, shape, shape.mode)
    L, cfg, t = bw.L, bw.L.cfg, bw.L.t
    slot_of, slot_token, counts = (H.to_np(v).copy() for v in (L.slot_of, L.slot_token, L.counts))
    empty, single = 3, 5
    slot_of[:, empty] = -1; slot_token[empty, :] = -1; counts[empty] = 0
    keep = slot_token[single, 0]
    slot_of[:, single] = -1; slot_of[keep, single] = 0
    slot_token[single, :] = -1; slot_token[single, 0] = keep; counts[single] = 1
    d_slot_of, d_slot_token, d_counts = (torch.from_numpy(v).cuda() for v in (slot_of, slot_token, counts))
    ws = B.alloc_workspace(B.etr_backward_workspace_bytes(cfg))
    ws.fill_(0xFF)
    dgate = torch.empty_like(bw.dgate)
    B.etr_moe_backward(cfg, t["x"], t["w_emb"], t["w_gate"], t["w_up"], t["w_down"], L.score, L.gate, d_slot_of, d_slot_token,
                       d_counts, bw.dout, bw.dx, bw.dwg, bw.dwu, bw.dwd, ws, dgate=dgate)
    torch.cuda.synchronize()
    hx = bw.host()
    ref = oracle.moe_backward(hx["x"], hx["w_emb"], hx["w_gate"], hx["w_up"], hx["w_down"], slot_of, hx["dout"],
                              D=shape.D, dtype=shape.dtype)
    tol = H.TOL_OUT[shape.dtype]
    for got, key in ((bw.dx, "dx"), (bw.dwg, "dw_gate"), (bw.dwu, "dw_up"), (bw.dwd, "dw_down")):
        assert _err(H, oracle, got, ref[key], shape.dtype) <= tol, key
    assert H.scale_rel_err(H.to_np(dgate).astype(np.float64), ref["dgate"]) <= tol
    for g in (bw.dwg, bw.dwu, bw.dwd):
        assert not H.to_np(g)[empty].any()
    # the one-row expert: its gradient is that row's outer product, compare on its own scale
    for got, key in ((bw.dwg, "dw_gate"), (bw.dwd, "dw_down")):
        a = oracle.to_f64(H.to_np(got)[single], shape.dtype)
        assert H.scale_rel_err(a, ref[key][single]) <= tol, key
