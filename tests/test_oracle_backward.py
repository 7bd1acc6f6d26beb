"""Pins for the oracle's backward pass (chain rule through Eqs. 1-6 with the routing tables fixed): CPU only.

The gradient is pinned against (a) reverse-mode differentiation by torch (float64) of a forward
written with library ops, after that forward has been checked against the oracle's own forward
stages, (b) central finite differences of the oracle's forward stages, (c) closed forms."""
import numpy as np
import pytest
import torch

TCR, ECR, BIDIR = 0, 1, 2
FULL, POOLED = 0, 1


def _layer(seed, T=24, d=16, E=4, D=2, H=12, std=0.3):
    rng = np.random.default_rng(seed)
    P = d // D
    x = rng.standard_normal((T, d)).astype(np.float32)
    q, _ = np.linalg.qr(rng.standard_normal((P, E)))
    w_emb = np.ascontiguousarray((q.T * rng.uniform(0.5, 2.0, (E, 1))).astype(np.float32))   # norms != 1 on purpose
    wg = (rng.standard_normal((E, H, d)) * std).astype(np.float32)
    wu = (rng.standard_normal((E, H, d)) * std).astype(np.float32)
    wd = (rng.standard_normal((E, d, H)) * std).astype(np.float32)
    dout = rng.standard_normal((T, d)).astype(np.float32)
    return x, w_emb, wg, wu, wd, dout


def _torch_forward(x, w_emb, wg, wu, wd, slot_of, D, cos, gate_norm=0):
    """Layer forward with library ops in float64; routing tables are constants."""
    T, d = x.shape
    E, P = w_emb.shape
    g = x.reshape(T, P, D).mean(dim=2)
    if cos == FULL:
        score = (D ** 0.5) * (g @ w_emb.T) / (x.norm(dim=1, keepdim=True) * w_emb.norm(dim=1)[None, :])
    else:
        score = (g @ w_emb.T) / (g.norm(dim=1, keepdim=True) * w_emb.norm(dim=1)[None, :])
    gate = torch.softmax(score, dim=1)
    keep = torch.from_numpy(slot_of >= 0)
    weight = gate * keep
    if gate_norm:
        total = weight.sum(dim=1, keepdim=True)
        weight = weight / torch.where(total > 0, total, torch.ones_like(total))
    out = torch.zeros_like(x)
    for e in range(E):
        y = (torch.nn.functional.silu(x @ wg[e].T) * (x @ wu[e].T)) @ wd[e].T
        out = out + weight[:, e][:, None] * y
    return out, score, gate


def _tables(oracle, x, w_emb, D, k, C, mode, cos):
    score, gate = oracle.route(x, w_emb, D, oracle.DT_F32, cos)
    topk, slot_of, slot_token, counts = oracle.select(score, k, C, mode)
    return score, gate, slot_of, slot_token, counts


@pytest.mark.parametrize("mode", [TCR, ECR, BIDIR])
@pytest.mark.parametrize("cos", [FULL, POOLED])
def test_backward_matches_reverse_mode_differentiation(oracle, mode, cos):
    D, k, C = 2, 2, 8
    x, w_emb, wg, wu, wd, dout = _layer(10 + mode + 3 * cos)
    score, gate, slot_of, slot_token, counts = _tables(oracle, x, w_emb, D, k, C, mode, cos)
    assert (slot_of >= 0).sum() < x.shape[0] * w_emb.shape[0]          # something is dropped
    tx, twg, twu, twd = (torch.from_numpy(a.astype(np.float64)).requires_grad_(True) for a in (x, wg, wu, wd))
    out, tscore, tgate = _torch_forward(tx, torch.from_numpy(w_emb.astype(np.float64)), twg, twu, twd, slot_of, D, cos)
    # the library-op forward is the oracle's forward (stage by stage, so the two stay tied together)
    np.testing.assert_allclose(tscore.detach().numpy(), score, atol=2e-7)
    np.testing.assert_allclose(tgate.detach().numpy(), gate, atol=2e-7)
    xp = oracle.dispatch(x, slot_token, counts, oracle.DT_F32)
    yp = oracle.expert_ffn(xp, counts, wg, wu, wd, oracle.DT_F32)
    ref_out = oracle.combine(yp, gate, slot_of, oracle.DT_F32)
    np.testing.assert_allclose(out.detach().numpy(), ref_out, rtol=2e-6, atol=2e-6)
    tgate.retain_grad(); tscore.retain_grad()
    out.backward(torch.from_numpy(dout.astype(np.float64)))
    r = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32, cos_mode=cos)
    np.testing.assert_allclose(r["dx"], tx.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dw_gate"], twg.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dw_up"], twu.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dw_down"], twd.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dgate"], tgate.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(r["dscore"], tscore.grad.numpy(), rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("mode,cos", [(TCR, FULL), (BIDIR, POOLED)])
def test_backward_with_renormalised_gate(oracle, mode, cos):
    D, k, C = 2, 2, 8
    x, w_emb, wg, wu, wd, dout = _layer(80 + mode)
    score, gate, slot_of, slot_token, counts = _tables(oracle, x, w_emb, D, k, C, mode, cos)
    tx, twg, twu, twd = (torch.from_numpy(a.astype(np.float64)).requires_grad_(True) for a in (x, wg, wu, wd))
    out, tscore, tgate = _torch_forward(tx, torch.from_numpy(w_emb.astype(np.float64)), twg, twu, twd, slot_of, D, cos, 1)
    ref = oracle.moe_forward(x, w_emb, wg, wu, wd, D=D, k=k, capacity=C, dtype=oracle.DT_F32, mode=mode, cos_mode=cos,
                             gate_norm=1)
    np.testing.assert_array_equal(ref["slot_of"], slot_of)
    np.testing.assert_allclose(out.detach().numpy(), ref["out"], rtol=2e-6, atol=2e-6)
    tgate.retain_grad(); tscore.retain_grad()
    out.backward(torch.from_numpy(dout.astype(np.float64)))
    r = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32, cos_mode=cos, gate_norm=1)
    for name, t in (("dx", tx), ("dw_gate", twg), ("dw_up", twu), ("dw_down", twd), ("dgate", tgate), ("dscore", tscore)):
        np.testing.assert_allclose(r[name], t.grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=name)
    # and it is a different gradient from the plain gate's
    r0 = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32, cos_mode=cos)
    assert np.max(np.abs(r0["dx"] - r["dx"])) > 1e-3


def _oracle_out_f64(oracle, x, w_emb, wg, wu, wd, slot_of, slot_token, counts, D, cos):
    """The oracle's forward stages with fixed tables; the final sum is taken in float64 (no output rounding)."""
    _, gate = oracle.route(x, w_emb, D, oracle.DT_F32, cos)
    yp = oracle.expert_ffn(oracle.dispatch(x, slot_token, counts, oracle.DT_F32), counts, wg, wu, wd, oracle.DT_F32)
    out = np.zeros(x.shape, np.float64)
    for t, e in zip(*np.nonzero(slot_of >= 0)):
        out[t] += float(gate[t, e]) * yp[e, slot_of[t, e]]
    return out


@pytest.mark.parametrize("cos", [FULL, POOLED])
def test_backward_matches_finite_differences_of_the_forward(oracle, cos):
    D, k, C = 2, 2, 8
    x, w_emb, wg, wu, wd, dout = _layer(30 + cos)
    _, _, slot_of, slot_token, counts = _tables(oracle, x, w_emb, D, k, C, BIDIR, cos)
    r = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32, cos_mode=cos)
    rng = np.random.default_rng(5)
    eps = 2.0 ** -9
    f = lambda *a: float((_oracle_out_f64(oracle, *a, slot_of, slot_token, counts, D, cos) * dout).sum())
    for name, idx in (("dx", 0), ("dw_gate", 2), ("dw_up", 3), ("dw_down", 4)):
        args = [x, w_emb, wg, wu, wd]
        v = rng.integers(-2, 3, args[idx].shape).astype(np.float32)          # exactly representable direction
        plus, minus = list(args), list(args)
        plus[idx] = (args[idx] + np.float32(eps) * v).astype(np.float32)
        minus[idx] = (args[idx] - np.float32(eps) * v).astype(np.float32)
        step = plus[idx].astype(np.float64) - minus[idx].astype(np.float64)   # the step actually taken
        fd = f(*plus) - f(*minus)
        analytic = float((r[name] * step).sum())
        assert abs(fd - analytic) <= 2e-4 * max(1.0, abs(analytic)), (name, fd, analytic)


def test_backward_closed_forms(oracle):
    # one token, one expert kept (ECR with C = T), one path x_2 -> hidden 3 -> output 4
    d, H, E, D = 6, 5, 2, 1
    x = (np.arange(1, d + 1, dtype=np.float32) / 4).reshape(1, d)
    w_emb = np.eye(E, d, dtype=np.float32)
    wg = np.zeros((E, H, d), np.float32); wu = np.zeros_like(wg); wd = np.zeros((E, d, H), np.float32)
    a, b, c = 0.75, -1.5, 2.0
    wg[1, 3, 2] = a; wu[1, 3, 2] = b; wd[1, 4, 3] = c
    slot_of = np.array([[-1, 0]], np.int32)                      # only expert 1 keeps the token
    dout = np.zeros((1, d), np.float32); dout[0, 4] = 1.0
    r = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32)
    score, gate = oracle.route(x, w_emb, D, oracle.DT_F32)
    g1 = float(gate[0, 1])
    x2 = float(x[0, 2]); z = a * x2; sg = 1 / (1 + np.exp(-z))
    silu, dsilu = z * sg, sg * (1 + z * (1 - sg))
    h = silu * b * x2
    np.testing.assert_allclose(r["dw_down"][1, 4, 3], g1 * h, rtol=1e-6)
    np.testing.assert_allclose(r["dw_gate"][1, 3, 2], g1 * c * (b * x2) * dsilu * x2, rtol=1e-6)
    np.testing.assert_allclose(r["dw_up"][1, 3, 2], g1 * c * silu * x2, rtol=1e-6)
    np.testing.assert_allclose(r["dgate"][0], [0.0, c * h], rtol=1e-12)
    # da and db live on hidden unit 3 only: dW_gate and dW_up are that unit's row, an outer product with x
    np.testing.assert_allclose(r["dw_gate"][1, 3], g1 * c * (b * x2) * dsilu * x[0], rtol=1e-6)
    np.testing.assert_allclose(r["dw_up"][1, 3], g1 * c * silu * x[0], rtol=1e-6)
    assert np.count_nonzero(r["dw_down"]) == 1 and np.count_nonzero(r["dw_gate"]) == d and np.count_nonzero(r["dw_up"]) == d
    assert not r["dw_gate"][0].any() and not r["dw_down"][0].any()   # expert 0 keeps nothing
    # dscore = gate .* (dgate - <dgate, gate>)
    dg = r["dgate"][0]; gt = gate[0].astype(np.float64)
    np.testing.assert_allclose(r["dscore"][0], gt * (dg - (dg * gt).sum()), rtol=1e-6)
    # the affinity is invariant under x -> alpha x, so its gradient is orthogonal to x: what is left of <dx, x>
    # is the expert path, c * d/dalpha [SiLU(a alpha x2) b alpha x2] at alpha = 1, times the gate
    np.testing.assert_allclose(float((r["dx"][0] * x[0]).sum()), g1 * c * (dsilu * z * b * x2 + silu * b * x2), rtol=1e-6)


def test_backward_of_a_dropped_token_and_zero_down_projection(oracle):
    D, k, C = 2, 1, 3
    x, w_emb, wg, wu, wd, dout = _layer(50)
    _, gate, slot_of, slot_token, counts = _tables(oracle, x, w_emb, D, k, C, TCR, FULL)
    dropped = np.nonzero((slot_of < 0).all(axis=1))[0]
    assert dropped.size > 0
    r = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32)
    assert not r["dx"][dropped].any() and not r["dgate"][dropped].any()
    # W_down = 0: y = 0, so nothing flows to x, W_gate, W_up; dW_down = sum gate * dout (x) h stays
    r0 = oracle.moe_backward(x, w_emb, wg, wu, np.zeros_like(wd), slot_of, dout, D=D, dtype=oracle.DT_F32)
    assert not r0["dx"].any() and not r0["dw_gate"].any() and not r0["dw_up"].any() and not r0["dgate"].any()
    np.testing.assert_allclose(r0["dw_down"], r["dw_down"], rtol=1e-12)
    # linear in the upstream gradient
    r2 = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, (2 * dout).astype(np.float32), D=D, dtype=oracle.DT_F32)
    for key in ("dx", "dw_gate", "dw_up", "dw_down", "dgate", "dscore"):
        np.testing.assert_allclose(r2[key], 2 * r[key], rtol=1e-12, atol=1e-300)


def test_backward_bf16_inputs_are_widened_exactly(oracle):
    D, k, C = 2, 2, 8
    x, w_emb, wg, wu, wd, dout = _layer(60)
    to_bits = lambda a: torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    widen = lambda b: (b.astype(np.uint32) << 16).view(np.float32)
    bits = [to_bits(a) for a in (x, wg, wu, wd, dout)]
    xb, wgb, wub, wdb, db = bits
    xw, wgw, wuw, wdw, dw = (widen(b) for b in bits)
    _, _, slot_of, _, _ = _tables(oracle, xw, w_emb, D, k, C, BIDIR, FULL)
    r16 = oracle.moe_backward(xb, w_emb, wgb, wub, wdb, slot_of, db, D=D, dtype=oracle.DT_BF16)
    r32 = oracle.moe_backward(xw, w_emb, wgw, wuw, wdw, slot_of, dw, D=D, dtype=oracle.DT_F32)
    for key in r16:
        np.testing.assert_array_equal(r16[key], r32[key])


def test_sampled_parts_agree_with_the_whole(oracle):
    D, k, C = 2, 2, 8
    x, w_emb, wg, wu, wd, dout = _layer(70)
    _, _, slot_of, _, _ = _tables(oracle, x, w_emb, D, k, C, BIDIR, FULL)
    r = oracle.moe_backward(x, w_emb, wg, wu, wd, slot_of, dout, D=D, dtype=oracle.DT_F32)
    tok = np.array([5, 0, 17], np.int32)
    dx, dg, ds = oracle.backward_tokens(x, w_emb, wg, wu, wd, slot_of, dout, tok, D=D, dtype=oracle.DT_F32)
    np.testing.assert_array_equal(dx, r["dx"][tok])
    ue, ui = np.array([3, 1], np.int32), np.array([7, 0], np.int32)
    gw, uw, dw = oracle.backward_hidden_units(x, w_emb, wg, wu, wd, slot_of, dout, ue, ui, D=D, dtype=oracle.DT_F32)
    np.testing.assert_array_equal(gw, r["dw_gate"][ue, ui]); np.testing.assert_array_equal(uw, r["dw_up"][ue, ui])
    np.testing.assert_array_equal(dw, r["dw_down"][ue, :, ui])
