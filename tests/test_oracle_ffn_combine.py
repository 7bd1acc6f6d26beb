"""Pins for the oracle's dispatch, expert FFN, combine and whole-layer chain: CPU only."""
import numpy as np
import pytest
import torch

TCR, ECR, BIDIR = 0, 1, 2


def _swiglu_torch(x, wg, wu, wd):
    """Textbook SwiGLU MLP with library matmuls in float64 (independent formulation)."""
    x, wg, wu, wd = (torch.from_numpy(np.asarray(a, np.float64)) for a in (x, wg, wu, wd))
    return (torch.nn.functional.silu(x @ wg.T) * (x @ wu.T) @ wd.T).numpy()


def _bf16_bits(a32):
    return torch.from_numpy(np.ascontiguousarray(a32, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _rand_layer(rng, T, d, E, H, P, std=0.2):
    x = rng.standard_normal((T, d)).astype(np.float32)
    q, _ = np.linalg.qr(rng.standard_normal((P, E)))
    w_emb = np.ascontiguousarray(q.T.astype(np.float32))
    wg = (rng.standard_normal((E, H, d)) * std).astype(np.float32)
    wu = (rng.standard_normal((E, H, d)) * std).astype(np.float32)
    wd = (rng.standard_normal((E, d, H)) * std).astype(np.float32)
    return x, w_emb, wg, wu, wd


def test_ffn_matches_library_matmul(oracle):
    rng = np.random.default_rng(0)
    n, d, H, E = 19, 24, 40, 3
    x, _, wg, wu, wd = _rand_layer(rng, n, d, E, H, 8)
    eid = rng.integers(0, E, n).astype(np.int32)
    y = oracle.ffn_rows(x, eid, wg, wu, wd, oracle.DT_F32)
    for r in range(n):
        e = eid[r]
        np.testing.assert_allclose(y[r], _swiglu_torch(x[r:r + 1], wg[e], wu[e], wd[e])[0], rtol=1e-11, atol=1e-12)


def test_ffn_closed_forms(oracle):
    d, H, E = 6, 5, 2
    x = np.arange(1, d + 1, dtype=np.float32).reshape(1, d) / 4
    wg = np.zeros((E, H, d), np.float32); wu = np.zeros((E, H, d), np.float32); wd = np.zeros((E, d, H), np.float32)
    eid = np.array([1], np.int32)
    # zero gate projection: SiLU(0) = 0, so the output vanishes whatever the other weights are
    wu[:] = 1.0; wd[:] = 1.0
    assert np.all(oracle.ffn_rows(x, eid, wg, wu, wd, 0) == 0)
    # a single path x_2 -> hidden 3 -> output 4 in expert 1: y_4 = c * SiLU(a x_2) * (b x_2)
    wu[:] = 0; wd[:] = 0
    a, b, c = 0.75, -1.5, 2.0
    wg[1, 3, 2] = a; wu[1, 3, 2] = b; wd[1, 4, 3] = c
    y = oracle.ffn_rows(x, eid, wg, wu, wd, 0)
    z = a * float(x[0, 2])
    expect = np.zeros(d); expect[4] = c * (z / (1 + np.exp(-z))) * (b * float(x[0, 2]))
    np.testing.assert_allclose(y[0], expect, rtol=1e-14)
    # the same weights in expert 0 must not leak into expert 1
    assert np.all(oracle.ffn_rows(x, np.array([0], np.int32), wg, wu, wd, 0) == 0)
    # transposed-operand guard: non-square, asymmetric weights against the library
    rng = np.random.default_rng(1)
    wg = rng.standard_normal((E, H, d)).astype(np.float32); wu = rng.standard_normal((E, H, d)).astype(np.float32)
    wd = rng.standard_normal((E, d, H)).astype(np.float32)
    y1 = oracle.ffn_rows(x, eid, wg, wu, wd, 0)
    np.testing.assert_allclose(y1[0], _swiglu_torch(x, wg[1], wu[1], wd[1])[0], rtol=1e-12)
    # linear in W_down
    y2 = oracle.ffn_rows(x, eid, wg, wu, (2 * wd).astype(np.float32), 0)
    np.testing.assert_allclose(y2, 2 * y1, rtol=1e-14)


def test_bf16_rounding_ties_to_even(oracle):
    rng = np.random.default_rng(2)
    v = np.concatenate([rng.standard_normal(4000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 4000),
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0, 3.3895313892515355e38],
                                 np.float32)]).astype(np.float32)
    bits = v.view(np.uint32).astype(np.uint64)
    expect = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)    # integer RNE on fp32 bits
    got = np.array([oracle.double_to_bf16(float(t)) for t in v], np.uint16)
    np.testing.assert_array_equal(got, expect)
    # a double that lies just above a bf16 half-way point must round up even though
    # rounding to fp32 first would land on the tie and then round to even (down)
    assert oracle.double_to_bf16(1.00390625 + 2.0 ** -40) == 0x3F81
    assert oracle.double_to_bf16(1.00390625) == 0x3F80


def test_dispatch_copies_rows(oracle):
    rng = np.random.default_rng(3)
    T, d, E, C = 50, 16, 4, 9
    x = rng.standard_normal((T, d)).astype(np.float32)
    S = rng.uniform(-1, 1, (T, E)).astype(np.float32)
    _, slot_of, slot_token, counts = oracle.select(S, 2, C, BIDIR)
    xp = oracle.dispatch(x, slot_token, counts, 0)
    for e in range(E):
        for s in range(C):
            if s < counts[e]:
                np.testing.assert_array_equal(xp[e, s], x[slot_token[e, s]])
            else:
                assert np.all(xp[e, s] == 0)
    xb = _bf16_bits(x)
    xpb = oracle.dispatch(xb, slot_token, counts, 1)
    np.testing.assert_array_equal(xpb[0, 0], xb[slot_token[0, 0]])


def test_combine_is_weighted_sum(oracle):
    rng = np.random.default_rng(4)
    T, d, E, C = 30, 8, 3, 12
    S = rng.uniform(-1, 1, (T, E)).astype(np.float32)
    _, slot_of, slot_token, counts = oracle.select(S, 2, C, TCR)
    gate = rng.uniform(0, 1, (T, E)).astype(np.float32)
    yp = rng.standard_normal((E, C, d))
    out = oracle.combine(yp, gate, slot_of, 0)
    for t in range(T):
        acc = np.zeros(d)
        for e in range(E):
            if slot_of[t, e] >= 0:
                assert slot_token[e, slot_of[t, e]] == t
                acc += float(gate[t, e]) * yp[e, slot_of[t, e]]
        np.testing.assert_allclose(out[t], acc.astype(np.float32), rtol=1e-6, atol=1e-7)
        if not (slot_of[t] >= 0).any():
            assert np.all(out[t] == 0)
    assert ((slot_of >= 0).sum(1) == 0).any(), "the case must contain a fully dropped token"


@pytest.mark.parametrize("mode", [TCR, ECR, BIDIR])
def test_layer_equals_chain_and_subset(oracle, mode):
    rng = np.random.default_rng(5)
    T, d, E, H, D, k, C = 40, 32, 4, 24, 4, 2, 12
    x, w_emb, wg, wu, wd = _rand_layer(rng, T, d, E, H, d // D)
    full = oracle.moe_forward(x, w_emb, wg, wu, wd, D=D, k=k, capacity=C, dtype=0, mode=mode)
    score, gate = oracle.route(x, w_emb, D, 0)
    topk, slot_of, slot_token, counts = oracle.select(score, k, C, mode)
    xp = oracle.dispatch(x, slot_token, counts, 0)
    yp = oracle.expert_ffn(xp, counts, wg, wu, wd, 0)
    out = oracle.combine(yp, gate, slot_of, 0)
    np.testing.assert_array_equal(full["score"], score)
    np.testing.assert_array_equal(full["slot_of"], slot_of)
    np.testing.assert_array_equal(full["slot_token"], slot_token)
    np.testing.assert_array_equal(full["counts"], counts)
    np.testing.assert_allclose(full["out"], out, rtol=1e-6, atol=1e-7)
    toks = np.array([3, 17, 0, 39], np.int32)
    sub = oracle.moe_forward(x, w_emb, wg, wu, wd, D=D, k=k, capacity=C, dtype=0, mode=mode, tokens=toks)
    np.testing.assert_array_equal(sub["out"], full["out"][toks])
    # externally supplied scores replace the route step
    ext = oracle.moe_forward(x, w_emb, wg, wu, wd, D=D, k=k, capacity=C, dtype=0, mode=mode, score_in=score)
    np.testing.assert_array_equal(ext["slot_of"], slot_of)
    np.testing.assert_allclose(ext["out"], out, rtol=1e-5, atol=1e-6)


def test_dense_special_case(oracle):
    """Capacity >= T, every token lists every expert, all experts identical:
    Eq. 1 collapses to FFN(x) * sum_e gate = FFN(x), because the gate row sums to 1."""
    rng = np.random.default_rng(6)
    T, d, E, H, D = 25, 16, 4, 12, 2
    x, w_emb, wg, wu, wd = _rand_layer(rng, T, d, E, H, d // D)
    wg[:] = wg[0]; wu[:] = wu[0]; wd[:] = wd[0]
    expect = _swiglu_torch(x, wg[0], wu[0], wd[0])
    for mode, k in ((TCR, E), (BIDIR, E), (ECR, 1)):
        res = oracle.moe_forward(x, w_emb, wg, wu, wd, D=D, k=k, capacity=T, dtype=0, mode=mode)
        assert np.all(res["slot_of"] >= 0)
        np.testing.assert_allclose(res["out"], expect, rtol=2e-6, atol=1e-6)


def test_layer_bf16_path(oracle):
    rng = np.random.default_rng(7)
    T, d, E, H, D, k, C = 24, 32, 4, 16, 8, 1, 5
    x, w_emb, wg, wu, wd = _rand_layer(rng, T, d, E, H, d // D)
    xb, wgb, wub, wdb = (_bf16_bits(a) for a in (x, wg, wu, wd))
    widen = lambda b: np.ascontiguousarray((b.astype(np.uint32) << 16).view(np.float32))
    rb = oracle.moe_forward(xb, w_emb, wgb, wub, wdb, D=D, k=k, capacity=C, dtype=1, mode=TCR)
    rf = oracle.moe_forward(widen(xb), w_emb, widen(wgb), widen(wub), widen(wdb), D=D, k=k, capacity=C, dtype=0,
                            mode=TCR)
    np.testing.assert_array_equal(rb["slot_of"], rf["slot_of"])
    # the bf16 output is the fp32-path output rounded once more (double -> bf16 vs double -> fp32)
    np.testing.assert_allclose(oracle.bf16_bits_to_f64(rb["out"]), rf["out"].astype(np.float64), rtol=2 ** -8, atol=1e-30)
    assert ((rf["slot_of"] >= 0).sum(1) == 0).any() and np.all(rb["out"][(rf["slot_of"] >= 0).sum(1) == 0] == 0)


def test_renormalised_gate_variant(oracle):
    """gate_norm = 1: a token's weights are renormalised over the experts that kept it, so they sum to one and
    equal experts give out = FFN(x) for every token that is kept at all, whatever subset kept it."""
    rng = np.random.default_rng(21)
    T, d, E, H, D = 40, 16, 4, 12, 2
    x, w_emb, wg, wu, wd = _rand_layer(rng, T, d, E, H, d // D)
    wg[:] = wg[0]; wu[:] = wu[0]; wd[:] = wd[0]
    r = oracle.moe_forward(x, w_emb, wg, wu, wd, D=D, k=2, capacity=9, dtype=oracle.DT_F32, mode=BIDIR, gate_norm=1)
    kept = (r["slot_of"] >= 0).sum(1)
    assert 0 < (kept == 0).sum() and (kept == 1).any() and (kept == 2).any()
    ffn = _swiglu_torch(x, wg[0], wu[0], wd[0])
    np.testing.assert_allclose(r["out"][kept > 0], ffn[kept > 0], rtol=2e-6, atol=2e-6)
    assert not r["out"][kept == 0].any()
    # the stage function agrees with the chain, and differs from the plain gate exactly by the per-token factor
    xp = oracle.dispatch(x, r["slot_token"], r["counts"], oracle.DT_F32)
    yp = oracle.expert_ffn(xp, r["counts"], wg, wu, wd, oracle.DT_F32)
    np.testing.assert_array_equal(oracle.combine(yp, r["gate"], r["slot_of"], oracle.DT_F32, gate_norm=1), r["out"])
    plain = oracle.combine(yp, r["gate"], r["slot_of"], oracle.DT_F32).astype(np.float64)
    s = np.where(r["slot_of"] >= 0, r["gate"].astype(np.float64), 0).sum(1)
    np.testing.assert_allclose(plain[kept > 0] / s[kept > 0, None], r["out"][kept > 0], rtol=3e-6, atol=1e-7)
