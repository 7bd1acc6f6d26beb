"""Pins for the oracle's route step (GrAP, cosine affinity, gate): CPU only.

Each check compares the oracle with something fixed by the paper's equations
or by plain mathematics, written here independently of the oracle's code.
"""
import numpy as np
import pytest
import torch

from conftest import load_golden


def _bf16_bits(a32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_worked_example(oracle):
    g = load_golden("route_worked_example.json")
    x = np.array([g["x"]], np.float32)
    w = np.eye(g["E"], dtype=np.float32)
    s_full, gate = oracle.route(x, w, g["D"], oracle.DT_F32, oracle.COS_FULL)
    s_pool, _ = oracle.route(x, w, g["D"], oracle.DT_F32, oracle.COS_POOLED)
    np.testing.assert_allclose(s_full[0], g["score_full"], atol=1e-7)
    np.testing.assert_allclose(s_pool[0], g["score_pooled"], atol=1e-7)
    np.testing.assert_allclose(gate[0], g["gate_full"], atol=2e-6)


def test_grap_is_group_mean(oracle):
    # With identity embeddings, score_full * |x| / sqrt(D) is the pooled feature itself.
    rng = np.random.default_rng(1)
    T, D, P = 37, 8, 12
    x = rng.standard_normal((T, D * P)).astype(np.float32)
    s, _ = oracle.route(x, np.eye(P, dtype=np.float32), D, oracle.DT_F32, oracle.COS_FULL)
    means = x.astype(np.float64).reshape(T, P, D).mean(-1)
    got = s.astype(np.float64) * np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True) / np.sqrt(D)
    np.testing.assert_allclose(got, means, atol=2e-6)


def test_block_indicator_closed_form(oracle):
    # Eqs. 2-4: w_i = (n/d) on group i, 0 elsewhere; delta_ti = cos(x_t, w_i) in R^d.
    rng = np.random.default_rng(2)
    T, n, d = 50, 8, 256
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wfull = np.zeros((n, d))
    for i in range(n):
        Wfull[i, i * d // n:(i + 1) * d // n] = n / d
    xd = x.astype(np.float64)
    expect = (xd @ Wfull.T) / (np.linalg.norm(xd, axis=1, keepdims=True) * np.linalg.norm(Wfull, axis=1))
    s, _ = oracle.route(x, np.eye(n, dtype=np.float32), d // n, oracle.DT_F32, oracle.COS_FULL)
    np.testing.assert_allclose(s, expect, atol=1e-7)
    # and the closed form quoted for this special case: sum of the group / (sqrt(d/n) |x|)
    closed = xd.reshape(T, n, d // n).sum(-1) / (np.sqrt(d / n) * np.linalg.norm(xd, axis=1, keepdims=True))
    np.testing.assert_allclose(s, closed, atol=1e-7)


@pytest.mark.parametrize("D,P,E", [(4, 16, 5), (16, 8, 8), (1, 24, 7)])
def test_full_equals_cosine_in_Rd_with_lifted_embedding(oracle, D, P, E):
    rng = np.random.default_rng(3)
    T, d = 41, D * P
    x = rng.standard_normal((T, d)).astype(np.float32)
    w = rng.standard_normal((E, P)).astype(np.float32)            # not normalised on purpose
    lifted = np.repeat(w.astype(np.float64), D, axis=1) / D       # pooling transpose
    xd = x.astype(np.float64)
    expect = (xd @ lifted.T) / (np.linalg.norm(xd, axis=1, keepdims=True) * np.linalg.norm(lifted, axis=1))
    s, gate = oracle.route(x, w, D, oracle.DT_F32, oracle.COS_FULL)
    np.testing.assert_allclose(s, expect, atol=1e-7)
    # pooled variant: cosine between group means and embedding
    g = xd.reshape(T, P, D).mean(-1)
    wd = w.astype(np.float64)
    expect_p = (g @ wd.T) / (np.linalg.norm(g, axis=1, keepdims=True) * np.linalg.norm(wd, axis=1))
    sp, _ = oracle.route(x, w, D, oracle.DT_F32, oracle.COS_POOLED)
    np.testing.assert_allclose(sp, expect_p, atol=1e-7)
    # gate = softmax over experts of the score row
    sm = torch.softmax(torch.from_numpy(expect), dim=1).numpy()
    np.testing.assert_allclose(gate, sm, atol=1e-7)
    np.testing.assert_allclose(gate.sum(1), 1.0, atol=1e-6)


def test_range_scaling_permutation_zero(oracle):
    rng = np.random.default_rng(4)
    T, D, P, E = 64, 8, 32, 8
    x = rng.standard_normal((T, D * P)).astype(np.float32)
    q, _ = np.linalg.qr(rng.standard_normal((P, E)))
    w = np.ascontiguousarray(q.T.astype(np.float32))
    for cm in (oracle.COS_FULL, oracle.COS_POOLED):
        s, g = oracle.route(x, w, D, oracle.DT_F32, cm)
        assert np.all(np.abs(s) <= 1.0 + 1e-6)
        s2, _ = oracle.route((x * 4.0).astype(np.float32), w, D, oracle.DT_F32, cm)   # power of two: exact
        np.testing.assert_array_equal(s, s2)
        perm = rng.permutation(T)
        s3, g3 = oracle.route(np.ascontiguousarray(x[perm]), w, D, oracle.DT_F32, cm)
        np.testing.assert_array_equal(s3, s[perm])
        np.testing.assert_array_equal(g3, g[perm])
    # FULL <= POOLED in magnitude (Jensen: |g| <= |x|/sqrt(D)), same sign
    sf, _ = oracle.route(x, w, D, oracle.DT_F32, oracle.COS_FULL)
    sp, _ = oracle.route(x, w, D, oracle.DT_F32, oracle.COS_POOLED)
    assert np.all(np.abs(sf) <= np.abs(sp) + 1e-7)
    assert np.all(np.sign(sf) == np.sign(sp))
    # zero token: all scores 0, uniform gate
    x[5] = 0
    s, g = oracle.route(x, w, D, oracle.DT_F32, oracle.COS_FULL)
    assert np.all(s[5] == 0) and np.allclose(g[5], 1.0 / E)


def test_bf16_input_is_widened_exactly(oracle):
    rng = np.random.default_rng(5)
    T, D, P, E = 33, 16, 8, 4
    x32 = rng.standard_normal((T, D * P)).astype(np.float32)
    bits = _bf16_bits(x32)
    xr = (bits.astype(np.uint32) << 16).view(np.float32)          # the values the bf16 bits stand for
    w = rng.standard_normal((E, P)).astype(np.float32)
    s_b, g_b = oracle.route(bits, w, D, oracle.DT_BF16)
    s_f, g_f = oracle.route(np.ascontiguousarray(xr), w, D, oracle.DT_F32)
    np.testing.assert_array_equal(s_b, s_f)
    np.testing.assert_array_equal(g_b, g_f)


def test_bad_shape_is_rejected(oracle):
    x = np.zeros((2, 10), np.float32)
    w = np.zeros((2, 3), np.float32)
    with pytest.raises(AssertionError):
        oracle.route(x, w, 3, oracle.DT_F32)
