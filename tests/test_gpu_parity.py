"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical bytes.

Routing tables are compared byte for byte with the oracle's selection run on the GPU's
own fp32 scores; scores and gates within 4e-6; outputs within max-abs-error / max-abs
1e-4 (fp32) or 2e-2 (bf16).
"""
import numpy as np
import pytest
import torch

from paper_2406_00023_amd import binding as B
from paper_2406_00023_amd import inputs as I

pytestmark = pytest.mark.gpu

TCR, ECR, BIDIR = I.MODE_TCR, I.MODE_ECR, I.MODE_BIDIR


@pytest.fixture(scope="module")
def H():
    import gpu_helpers
    assert torch.cuda.is_available()
    B.load_library()
    return gpu_helpers


def _say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------------------
# whole layer, small enough for the oracle to do every row
# ---------------------------------------------------------------------------------------
SMALL = {
    "cfg1": lambda: I.CONFIGS["cfg1"],
    "cfg2s": lambda: I.small_variant(I.CONFIGS["cfg2"], T=1100, d=512, H=704),
    "cfg3s": lambda: I.small_variant(I.CONFIGS["cfg3"], T=900, d=1024, H=1032),
    "cfg4s": lambda: I.small_variant(I.CONFIGS["cfg4"], T=1500, d=1024, H=328),
    "cfg5s": lambda: I.small_variant(I.CONFIGS["cfg5"], T=700, H=200),     # full d: 64 pooled features for 64 global experts
    # widths on whole column tiles of both GEMMs (H % 128 == 0, d % 256 == 0): the four-wave persistent kernel,
    # with the token rows gathered inside GEMM-1 in the fused call
    "cfg2w": lambda: I.small_variant(I.CONFIGS["cfg2"], T=1300, d=512, H=640),
    "cfg5w": lambda: I.small_variant(I.CONFIGS["cfg5"], T=900, H=256),
}


@pytest.mark.parametrize("name,mode", [("cfg1", TCR), ("cfg1", ECR), ("cfg1", BIDIR), ("cfg2s", TCR), ("cfg3s", ECR),
                                       ("cfg4s", BIDIR), ("cfg5s", BIDIR), ("cfg2w", TCR), ("cfg5w", BIDIR)])
def test_layer_stage_by_stage_and_fused(H, oracle, name, mode):
    shape = SMALL[name]()
    _say(f"case {name} mode={mode} T={shape.T} d={shape.d} E={shape.E} C={shape.capacity} H={shape.H}")
    L = H.GpuLayer(shape, mode=mode)
    hx = L.host_inputs()
    # stage by stage
    L.route(); L.select(); L.dispatch(); L.expert_ffn(); L.combine()
    torch.cuda.synchronize()
    r = H.check_routing_against_oracle(oracle, L, hx)
    # dispatch: kept rows byte-equal, other rows untouched
    xp = H.to_np(L.xp)
    poison = H.to_np(torch.full((1,), 7.0, dtype=shape.torch_dtype))[0]
    for e in range(shape.E):
        n = r["counts"][e]
        np.testing.assert_array_equal(xp[e, :n], hx["x"][r["slot_token"][e, :n]])
        assert np.all(xp[e, n:] == poison)
        assert np.all(H.to_np(L.yp)[e, n:] == poison)
    err = H.check_output_against_oracle(oracle, L, hx, r["score"])
    staged = L.out.clone()
    tables = [t.clone() for t in (L.score, L.gate, L.topk, L.slot_of, L.slot_token, L.counts)]
    # fused call: same kernels on one stream -> identical bits
    for t in (L.score, L.gate, L.out):
        t.zero_()
    for t in (L.topk, L.slot_of, L.slot_token, L.counts):
        t.fill_(-9)
    L.forward()
    assert torch.equal(L.out, staged)
    for a, b in zip(tables, (L.score, L.gate, L.topk, L.slot_of, L.slot_token, L.counts)):
        if a is tables[2] and mode == ECR:
            continue
        assert torch.equal(a, b)
    # fused call without the optional outputs
    L.out.zero_()
    L.forward(keep_tables=False)
    assert torch.equal(L.out, staged)
    _say(f"  out err {err:.3e}; decisions differing from the fully independent oracle: {r['ndiff']}")
    assert r["ndiff"] <= 4


def test_capacity_sweep_small(H, oracle):
    shape = SMALL["cfg4s"]()
    t = I.make_inputs(shape, "cuda")
    for cap in shape.capacity_sweep:
        _say(f"case cfg4s capacity={cap}")
        L = H.GpuLayer(shape, tensors=t, capacity=cap)
        L.forward()
        hx = L.host_inputs()
        r = H.check_routing_against_oracle(oracle, L, hx)
        H.check_output_against_oracle(oracle, L, hx, r["score"], tokens=np.arange(0, shape.T, 7, dtype=np.int32))


# ---------------------------------------------------------------------------------------
# route
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,d,E,D,dtype,cos", [
    (257, 256, 8, 8, I.DT_F32, I.COS_FULL),       # fp32, two 16-byte chunks per group
    (130, 512, 5, 16, I.DT_BF16, I.COS_POOLED),   # E not a power of two, pooled norm
    (65, 384, 3, 6, I.DT_BF16, I.COS_FULL),       # group size not a multiple of the vector: scalar walk
    (33, 264, 33, 8, I.DT_BF16, I.COS_FULL),      # P = 33 = E, one lane per expert
    (1, 4096, 64, 64, I.DT_BF16, I.COS_FULL),     # single token, 64 experts
    (300, 1024, 16, 1, I.DT_F32, I.COS_POOLED),   # D = 1: no pooling at all
    (9000, 2048, 16, 16, I.DT_BF16, I.COS_FULL),  # more tokens than one grid pass
])
def test_route(H, oracle, T, d, E, D, dtype, cos):
    _say(f"case route T={T} d={d} E={E} D={D} dtype={dtype} cos={cos}")
    shape = I.EtrShape("r", 1, T=T, d=d, E=E, D=D, k=1, capacity=4, H=8, dtype=dtype, mode=TCR, recipe="iso", cos=cos)
    w = I.orthonormal_embeddings(77, E, d // D)
    w = (w * torch.linspace(0.5, 2.0, E).unsqueeze(1)).contiguous()     # norms are computed, not assumed
    x = I.make_tokens(shape, w, "cuda")
    if T > 2:
        x[T // 2] = 0                                                    # zero-norm token
    L = H.GpuLayer(shape, tensors={"x": x, "w_emb": w})
    L.route()
    torch.cuda.synchronize()
    o_score, o_gate = oracle.route(H.to_np(x), w.numpy(), D, dtype, cos)
    assert np.max(np.abs(H.to_np(L.score) - o_score)) <= H.TOL_SCORE
    assert np.max(np.abs(H.to_np(L.gate) - o_gate)) <= H.TOL_GATE
    if T > 2:
        assert np.all(H.to_np(L.score)[T // 2] == 0)


# ---------------------------------------------------------------------------------------
# select on externally supplied scores (ties, odd sizes, every mode)
# ---------------------------------------------------------------------------------------
def _scores(seed, T, E, levels):
    rng = np.random.default_rng(seed)
    if levels:
        s = rng.integers(-levels, levels + 1, size=(T, E)) / levels
        s[rng.random((T, E)) < 0.05] = -0.0
        return s.astype(np.float32)
    return rng.uniform(-1, 1, size=(T, E)).astype(np.float32)


@pytest.mark.parametrize("T,E,k,C,levels", [
    (1, 1, 1, 1, None), (6, 3, 2, 2, 4), (64, 8, 1, 5, 3), (1000, 17, 4, 123, 7), (1000, 17, 17, 2000, None),
    (4097, 64, 8, 300, 50), (5000, 2, 1, 1, 2), (20000, 16, 2, 2500, 1000), (70001, 8, 3, 9000, 200),
    (3000, 33, 5, 3000, None),
    # chunk lengths 16 and 64 of the per-expert search (64 with idle waves at the end of the column); four lanes
    # per token over many workgroups; 64 lanes per token
    (12000, 5, 2, 3000, 64), (40000, 4, 2, 15000, None), (33000, 40, 3, 1500, 500),
])
def test_select_external_scores(H, oracle, T, E, k, C, levels):
    S = _scores(T * 31 + E, T, E, levels)
    for mode in (TCR, ECR, BIDIR, I.MODE_TCR_RANK, I.MODE_BIDIR_STRICT):
        _say(f"case select T={T} E={E} k={k} C={C} levels={levels} mode={mode}")
        shape = I.EtrShape("s", 1, T=T, d=8 * E, E=E, D=8, k=k, capacity=C, H=8, dtype=I.DT_F32, mode=mode, recipe="iso")
        L = H.GpuLayer(shape, tensors={})
        L.select(score=torch.from_numpy(S).cuda())
        torch.cuda.synchronize()
        topk, slot_of, slot_token, counts = oracle.select(S, k, C, mode)
        if mode != ECR:
            np.testing.assert_array_equal(H.to_np(L.topk), topk)
        np.testing.assert_array_equal(H.to_np(L.counts), counts)
        np.testing.assert_array_equal(H.to_np(L.slot_of), slot_of)
        np.testing.assert_array_equal(H.to_np(L.slot_token), slot_token)
        # same call again: bit-reproducible
        first = (L.slot_of.clone(), L.slot_token.clone())
        L.select(score=torch.from_numpy(S).cuda())
        assert torch.equal(first[0], L.slot_of) and torch.equal(first[1], L.slot_token)


# ---------------------------------------------------------------------------------------
# expert FFN alone: ragged counts, an empty expert, K and N tails
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,E,C,d,H_,counts", [
    (I.DT_BF16, 3, 300, 264, 328, [300, 0, 37]),       # K not a multiple of the k-tile, N tails in both GEMMs
    (I.DT_BF16, 2, 130, 512, 128, [129, 1]),
    (I.DT_F32, 4, 70, 72, 40, [70, 3, 0, 64]),
    (I.DT_BF16, 1, 513, 1024, 704, [513]),            # pipelined kernels: row tail of 1, column tail in GEMM-1
    (I.DT_BF16, 2, 40, 64, 64, [40, 7]),               # pipelined kernels with only two k-tiles
    (I.DT_BF16, 1, 300, 128, 192, [300]),              # four and six k-tiles: prologue meets drain
    (I.DT_BF16, 3, 600, 2048, 512, [600, 256, 257]),   # counts on and just past a row-tile boundary
    # more live tiles than CUs with only two k-tiles: every persistent workgroup runs on from one tile into the next
    # while it is still inside the first tile's prologue (GEMM-1 in the first case, GEMM-2 in the second)
    (I.DT_BF16, 8, 2048, 128, 1024, [2048, 1500, 2048, 300, 2047, 1025, 2048, 1800]),
    (I.DT_BF16, 8, 2048, 2048, 128, [2048, 1500, 0, 300, 2047, 1025, 2048, 1800]),
    # whole column tiles in both GEMMs (the 64-wide persistent kernel): an odd number of k-tiles, an empty expert between
    # live ones, one-row and one-past-a-tile experts; then more live tiles than CUs with a long second contraction
    (I.DT_BF16, 6, 900, 768, 1152, [900, 0, 513, 1, 899, 256]),
    (I.DT_BF16, 8, 1100, 256, 2816, [1100, 700, 1, 1024, 0, 1025, 300, 1100]),
    # sixteen and more row tiles per expert: the tile list is cut into 8 x 4 super-tiles in the second GEMM
    # (d = 1024: four column tiles) and into one super-tile per row band in the first (H = 384: three column tiles)
    (I.DT_BF16, 2, 4200, 1024, 384, [4200, 3333]),
])
def test_expert_ffn(H, oracle, dtype, E, C, d, H_, counts):
    _say(f"case ffn dtype={dtype} E={E} C={C} d={d} H={H_} counts={counts}")
    dt = torch.float32 if dtype == I.DT_F32 else torch.bfloat16
    shape = I.EtrShape("f", 1, T=C, d=d, E=E, D=8, k=1, capacity=C, H=H_, dtype=dtype, mode=TCR, recipe="iso")
    xp = I.normal(1, E * C * d, "cuda").reshape(E, C, d).to(dt)
    wg = I.ffn_weight(2, (E, H_, d), dt, "cuda", std=0.05)
    wu = I.ffn_weight(3, (E, H_, d), dt, "cuda", std=0.05)
    wd = I.ffn_weight(4, (E, d, H_), dt, "cuda", std=0.05)
    cnt = torch.tensor(counts, dtype=torch.int32, device="cuda")
    yp = torch.full((E, C, d), 7.0, dtype=dt, device="cuda")
    cfg = B.make_config(shape)
    ws = B.alloc_workspace(B.etr_ffn_workspace_bytes(cfg))
    B.etr_expert_ffn(cfg, xp, cnt, wg, wu, wd, yp, ws)
    torch.cuda.synchronize()
    ref = oracle.expert_ffn(H.to_np(xp), np.array(counts, np.int32), H.to_np(wg), H.to_np(wu), H.to_np(wd), dtype)
    got = oracle.to_f64(H.to_np(yp), dtype)
    for e in range(E):
        n = counts[e]
        assert np.all(got[e, n:] == 7.0)
        if n:
            assert H.scale_rel_err(got[e, :n], ref[e, :n]) <= H.TOL_OUT[dtype]


# ---------------------------------------------------------------------------------------
# combine alone
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,T,E,C,d,k,mode", [(I.DT_BF16, 700, 8, 200, 520, 3, TCR), (I.DT_F32, 300, 5, 40, 264, 2, ECR)])
def test_combine(H, oracle, dtype, T, E, C, d, k, mode):
    _say(f"case combine dtype={dtype} T={T} E={E} C={C} d={d} mode={mode}")
    dt = torch.float32 if dtype == I.DT_F32 else torch.bfloat16
    S = _scores(5, T, E, None)
    _, slot_of, _, _ = oracle.select(S, k, C, mode)
    gate = np.random.default_rng(6).uniform(0, 1, (T, E)).astype(np.float32)
    yp = I.normal(8, E * C * d, "cuda").reshape(E, C, d).to(dt)
    shape = I.EtrShape("c", 1, T=T, d=d, E=E, D=8, k=k, capacity=C, H=8, dtype=dtype, mode=mode, recipe="iso")
    out = torch.empty(T, d, dtype=dt, device="cuda")
    B.etr_combine(B.make_config(shape), yp, torch.from_numpy(gate).cuda(), torch.from_numpy(slot_of).cuda(), out)
    torch.cuda.synchronize()
    ref = oracle.combine(oracle.to_f64(H.to_np(yp), dtype), gate, slot_of, dtype)
    a, b = oracle.to_f64(H.to_np(out), dtype), oracle.to_f64(ref, dtype)
    # fp32 accumulation of <= E terms, one rounding: a couple of ulps of the output type
    assert H.scale_rel_err(a, b) <= (2e-6 if dtype == I.DT_F32 else 2 ** -7)
    assert np.all(a[(slot_of >= 0).sum(1) == 0] == 0)


# ---------------------------------------------------------------------------------------
# argument validation reaches the caller as a status (nothing is launched)
# ---------------------------------------------------------------------------------------
def test_error_statuses_on_device(H):
    shape = I.CONFIGS["cfg1"]
    L = H.GpuLayer(shape)
    with pytest.raises(B.EtrError) as ei:
        B.etr_select(L.cfg, L.score, L.topk, L.slot_of, L.slot_token, L.counts, B.alloc_workspace(64))
    assert ei.value.status == 4
    with pytest.raises(B.EtrError) as ei:
        B.etr_route(L.cfg, L.t["x"].view(torch.uint8).flatten()[4:].view(torch.float32)[: shape.T * shape.d - 4],
                    L.t["w_emb"], L.score, L.gate)
    assert ei.value.status == 5
