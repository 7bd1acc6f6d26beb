"""The seeded input generators: determinism, structure, and that each recipe produces
the load pattern its workload is meant to have. CPU only."""
import numpy as np
import pytest
import torch

from paper_2406_00023_amd import inputs as I


def test_generator_is_counter_based():
    a = I.normal(123, 1000)
    b = torch.cat([I.normal(123, 300), I.normal(123, 700, start=300)])
    c = I.normal(123, 1000, chunk=64)
    assert torch.equal(a, b) and torch.equal(a, c)
    assert not torch.equal(a, I.normal(124, 1000))
    z = I.normal(5, 400000)
    assert abs(float(z.mean())) < 0.01 and abs(float(z.std()) - 1) < 0.01
    assert abs(float((z ** 3).mean())) < 0.03 and abs(float((z ** 4).mean()) - 3) < 0.1
    assert torch.isfinite(z).all()
    u = I.uniform01(9, 100000)
    assert float(u.min()) >= 0 and float(u.max()) < 1 and abs(float(u.mean()) - 0.5) < 0.01


@pytest.mark.parametrize("name", list(I.CONFIGS))
def test_embeddings_are_orthonormal(name):
    s = I.CONFIGS[name]
    w = I.orthonormal_embeddings(I.stream_seed(s.cfg_id, "emb"), s.E, s.P, s.E_global).double()
    assert w.shape == (s.E, s.P)
    assert float((w @ w.T - torch.eye(s.E, dtype=torch.float64)).abs().max()) < 1e-6
    u = I.lifted_unit_directions(w.float(), s.D).double()
    assert float((u @ u.T - torch.eye(s.E, dtype=torch.float64)).abs().max()) < 1e-6   # lifting keeps orthogonality


def test_config_table():
    c = I.CONFIGS
    assert (c["cfg1"].capacity, c["cfg2"].capacity, c["cfg3"].capacity, c["cfg5"].capacity) == (80, 1024, 1280, 36045)
    assert c["cfg4"].capacity_sweep == (2048, 1792, 1536, 1280, 1024)
    for s in c.values():
        assert s.d % s.D == 0 and s.E <= s.P and s.d % 8 == 0


def test_make_inputs_shapes_and_dtype():
    s = I.small_variant(I.CONFIGS["cfg2"], T=64, H=32, d=256)
    t = I.make_inputs(s)
    assert t["x"].shape == (64, 256) and t["x"].dtype == torch.bfloat16
    assert t["w_gate"].shape == (16, 32, 256) and t["w_down"].shape == (16, 256, 32)
    assert abs(float(t["w_gate"].float().std()) - 0.02) < 0.002
    t2 = I.make_inputs(s)
    assert all(torch.equal(t[k], t2[k]) for k in t)


def test_cluster_recipe_gives_cosine_point_eight():
    # sigma = 0.5 around unit-variance centroids: same-cluster cosine = 1/(1+sigma^2) = 0.8
    s = I.small_variant(I.CONFIGS["cfg3"], T=256)
    t = I.make_inputs(s, with_weights=False)
    x = t["x"].double()
    c = (I.uniform01(I.stream_seed(3, "cluster"), 256) * 16).long()
    xn = x / x.norm(dim=1, keepdim=True)
    cos = xn @ xn.T
    same = (c[:, None] == c[None, :]) & ~torch.eye(256, dtype=torch.bool)
    assert abs(float(cos[same].mean()) - 0.8) < 0.02
    assert abs(float(cos[c[:, None] != c[None, :]].mean())) < 0.05


def _top_counts(oracle, s, t):
    xb = t["x"].view(torch.int16).numpy().view(np.uint16) if s.dtype == I.DT_BF16 else t["x"].numpy()
    score, _ = oracle.route(np.ascontiguousarray(xb), t["w_emb"].numpy(), s.D, s.dtype)
    order = np.argsort(-score, axis=1, kind="stable")[:, :s.k]
    return np.bincount(order.ravel(), minlength=s.E)


def test_bias_recipe_overflows_some_experts(oracle):
    s = I.small_variant(I.CONFIGS["cfg2"], T=2048)
    n = _top_counts(oracle, s, I.make_inputs(s, with_weights=False))
    assert (n > s.capacity).any() and (n < s.capacity).any()


def test_zipf_recipe_is_skewed(oracle):
    s = I.small_variant(I.CONFIGS["cfg5"], T=2048)
    t = I.make_inputs(s, with_weights=False)
    first = _top_counts(oracle, s.with_(k=1), t)          # every token's best expert follows the Zipf law
    p = np.array([(c + 1.0) ** -1.1 for c in range(s.E)]); p /= p.sum()
    assert np.all(np.abs(first / s.T - p) < 0.04)
    n = _top_counts(oracle, s, t)                          # top-4 load is still visibly skewed
    assert n[0] > 1.3 * n[-1] and n.sum() == s.k * s.T
