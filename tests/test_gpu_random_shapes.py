"""Seeded random small shapes through the fused forward and the backward: the tile schedules, the ragged and empty
experts, the column tails and the kernel fall-backs all depend on the shape, so a spread of shapes is checked
against the oracle (every token, every gradient)."""
import numpy as np
import pytest
import torch

from paper_2406_00023_amd import binding as B
from paper_2406_00023_amd import inputs as I

pytestmark = pytest.mark.gpu


def _shape(seed):
    rng = np.random.default_rng(9000 + seed)
    D = int(rng.choice([4, 8, 16, 32]))
    # contraction lengths on and off the 64 / 128 boundaries that select the GEMM kernel
    d = int(rng.choice([64, 128, 192, 256, 320, 384, 512])) if seed % 3 else int(rng.choice([72, 136, 264]))
    while d % D:
        D //= 2
    P = d // D
    E = int(rng.integers(1, min(P, 24) + 1))
    H = int(rng.choice([64, 128, 200, 256, 328, 384, 576]))
    T = int(rng.integers(40, 700))
    mode = int(rng.integers(0, 5))
    k = int(rng.integers(1, min(E, 4) + 1))
    C = int(rng.integers(1, max(2, (2 * k * T) // E)))
    dtype = I.DT_BF16 if seed % 4 else I.DT_F32
    recipe = ["iso", "bias", "cluster", "zipf"][seed % 4] if E >= 2 else "iso"
    return I.EtrShape(f"rand{seed}", 7, T=T, d=d, E=E, D=D, k=k, capacity=C, H=H, dtype=dtype, mode=mode, recipe=recipe,
                      n_centroids=max(2, E))


@pytest.mark.parametrize("seed", range(16))
def test_random_shape_forward_and_backward(oracle, seed):
    import gpu_helpers as H
    from test_gpu_backward import Backward, _err
    B.load_library()
    shape = _shape(seed)
    print(f"random shape {seed}: T={shape.T} d={shape.d} E={shape.E} D={shape.D} k={shape.k} C={shape.capacity} H={shape.H} "
          f"dtype={shape.dtype} mode={shape.mode} recipe={shape.recipe}", flush=True)
    gate_norm = seed % 2
    L = H.GpuLayer(shape, gate_norm=gate_norm)
    hx = L.host_inputs()
    L.forward()
    r = H.check_routing_against_oracle(oracle, L, hx)
    H.check_output_against_oracle(oracle, L, hx, r["score"])
    bw = Backward(H, shape, shape.mode, gate_norm=gate_norm)
    hb = bw.host()
    ref = oracle.moe_backward(hb["x"], hb["w_emb"], hb["w_gate"], hb["w_up"], hb["w_down"], hb["slot_of"], hb["dout"],
                              D=shape.D, dtype=shape.dtype, gate_norm=gate_norm)
    tol = H.TOL_OUT[shape.dtype]
    for got, key in ((bw.dx, "dx"), (bw.dwg, "dw_gate"), (bw.dwu, "dw_up"), (bw.dwd, "dw_down")):
        if np.max(np.abs(ref[key])) == 0:
            assert not H.to_np(got).any(), key
        else:
            assert _err(H, oracle, got, ref[key], shape.dtype) <= tol, key


def _many_rows_shape(seed):
    """Capacities from 8192 on: the backward's weight-gradient products fetch their rows through slot_token, and the
    products against a weight matrix take the row-major kernel with ragged last column tiles."""
    rng = np.random.default_rng(9500 + seed)
    D = int(rng.choice([8, 16, 32]))
    d = int(rng.choice([128, 256, 320]))
    E = int(rng.integers(1, 5))
    H = int(rng.choice([64, 200, 264, 328]))
    T = int(rng.integers(8300, 13000))
    mode = int(rng.integers(0, 5))
    k = int(rng.integers(1, E + 1))
    C = int(rng.integers(8192, 8192 + 700))
    recipe = ["iso", "bias", "cluster", "zipf"][seed % 4] if E >= 2 else "iso"
    return I.EtrShape(f"rows{seed}", 7, T=T, d=d, E=E, D=D, k=k, capacity=C, H=H, dtype=I.DT_BF16, mode=mode, recipe=recipe,
                      n_centroids=max(2, E))


@pytest.mark.parametrize("seed", range(6))
def test_random_shape_backward_many_rows(oracle, seed):
    import gpu_helpers as H
    from test_gpu_backward import Backward, _err
    B.load_library()
    shape = _many_rows_shape(seed)
    print(f"many-rows shape {seed}: T={shape.T} d={shape.d} E={shape.E} D={shape.D} k={shape.k} C={shape.capacity} H={shape.H} "
          f"mode={shape.mode} recipe={shape.recipe}", flush=True)
    gate_norm = seed % 2
    bw = Backward(H, shape, shape.mode, gate_norm=gate_norm)
    hb = bw.host()
    ref = oracle.moe_backward(hb["x"], hb["w_emb"], hb["w_gate"], hb["w_up"], hb["w_down"], hb["slot_of"], hb["dout"],
                              D=shape.D, dtype=shape.dtype, gate_norm=gate_norm)
    tol = H.TOL_OUT[shape.dtype]
    for got, key in ((bw.dx, "dx"), (bw.dwg, "dw_gate"), (bw.dwu, "dw_up"), (bw.dwd, "dw_down")):
        if np.max(np.abs(ref[key])) == 0:
            assert not H.to_np(got).any(), key
        else:
            err = _err(H, oracle, got, ref[key], shape.dtype)
            print(f"  {key}: {err:.2e}", flush=True)
            assert err <= tol, key
