"""GPU parity of the fused forward against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs, mhffn
from tests.helpers import TOL, check_parity, device_inputs, relerr, small_workload, to_host

pytestmark = pytest.mark.gpu


def run_forward(w, seed=0, route_weights=False):
    import torch
    d = inputs.make_inputs(w, seed=seed, with_dy=False, route_weights=route_weights)
    g = device_inputs(d, w.dtype)
    if route_weights:
        Y = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["R"], w.eps,
                          mhffn.ROUTE_WEIGHTS)
    else:
        Y = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps)
    torch.cuda.synchronize()
    return d, to_host(Y)


def oracle_forward(d, w, rows=None, route_weights=False):
    X = d["X"] if rows is None else d["X"][rows]
    if route_weights:
        R = d["R"] if rows is None else d["R"][rows]
        return orc.forward(X, d["W_gate"], d["W_up"], d["W_down"], R, w.eps, orc.ROUTE_WEIGHTS)
    return orc.forward(X, d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)


def test_tiny_f32_config():
    w = inputs.WORKLOADS["tiny_f32"]
    d, Y = run_forward(w)
    assert relerr(Y, oracle_forward(d, w)) <= TOL["f32"]


@pytest.mark.parametrize("N", [1, 31, 63, 65, 257, 600])
def test_f32_ragged_and_generic_shapes(N):
    w = inputs.Workload("f32_generic", N, 3, 72, 5, 40, "f32", w_std=0.1, route_scale=3.0)
    d, Y = run_forward(w, seed=N)
    assert relerr(Y, oracle_forward(d, w)) <= TOL["f32"]


@pytest.mark.parametrize("N,H,E,de", [(256, 2, 4, 128), (1, 1, 1, 32), (63, 2, 3, 64),
                                       (65, 1, 5, 32), (257, 3, 2, 96), (1000, 2, 33, 32),
                                       (300, 1, 64, 32),
                                       # more than 64 sub-networks: the non-pipelined kernels
                                       (300, 1, 80, 32), (100, 2, 96, 32), (1500, 1, 70, 64)])
def test_bf16_small_shapes_params_mode(N, H, E, de):
    w = small_workload("bf16_small", N, H, E, de, "bf16")
    d, Y = run_forward(w, seed=N + E)
    assert relerr(Y, oracle_forward(d, w)) <= TOL["bf16"]


@pytest.mark.parametrize("N,H,E,de,weights", [
    (1, 1, 1, 32, False), (17, 3, 5, 64, False), (32, 16, 44, 128, False), (33, 2, 64, 32, False),
    (64, 16, 44, 128, False), (64, 5, 7, 384, True), (65, 2, 3, 96, False), (100, 6, 16, 128, True),
    (128, 16, 22, 384, False), (96, 1, 33, 32, True),
    # more heads than workgroup slots: one workgroup per head, no partial outputs
    (5, 300, 2, 32, False), (40, 260, 1, 64, True)])
def test_bf16_decode_sized_inputs(N, H, E, de, weights):
    """Up to 128 tokens at d_h = 128: the weight-streaming kernel (one to four token blocks,
    tiles of a batch worked on side by side, partial sums over tile groups and over
    workgroups), every row against the oracle."""
    w = small_workload("bf16_decode", N, H, E, de, "bf16")
    d, Y = run_forward(w, seed=N + E, route_weights=weights)
    check_parity({"Y": Y}, {"Y": oracle_forward(d, w, route_weights=weights)}, TOL["bf16"], 128,
                 "decode N=%d" % N)


def test_decode_sized_strided_rows_and_run_to_run():
    import torch
    w = small_workload("decode_strided", 50, 4, 9, 64, "bf16")
    d = inputs.make_inputs(w, seed=21, with_dy=False)
    g = device_inputs(d, w.dtype)
    dm = w.d_model
    Xp = torch.zeros(w.n_tokens, dm + 64, dtype=torch.bfloat16, device="cuda")
    Xp[:, :dm] = g["X"]
    out = []
    for _ in range(2):
        Yp = torch.full((w.n_tokens, dm + 128), 7.0, dtype=torch.bfloat16, device="cuda")
        mhffn.forward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps, out=Yp[:, :dm])
        torch.cuda.synchronize()
        assert torch.all(Yp[:, dm:] == 7.0)
        out.append(to_host(Yp[:, :dm]))
    assert np.array_equal(out[0], out[1])
    check_parity({"Y": out[0]}, {"Y": oracle_forward(d, w)}, TOL["bf16"], 128, "decode strided")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_weights_mode(dtype):
    w = small_workload("weights_mode", 333, 2, 6, 64, dtype)
    d, Y = run_forward(w, seed=5, route_weights=True)
    assert relerr(Y, oracle_forward(d, w, route_weights=True)) <= TOL[dtype]


def test_rows_beyond_n_untouched_and_strided_rows():
    """ld_x / ld_y larger than d_model: the padding columns are never written."""
    import torch
    w = small_workload("strided", 130, 2, 3, 64, "bf16")
    d = inputs.make_inputs(w, seed=9, with_dy=False)
    g = device_inputs(d, w.dtype)
    dm = w.d_model
    Xp = torch.zeros(w.n_tokens, dm + 64, dtype=torch.bfloat16, device="cuda")
    Xp[:, :dm] = g["X"]
    Yp = torch.full((w.n_tokens, dm + 128), 7.0, dtype=torch.bfloat16, device="cuda")
    mhffn.forward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps, out=Yp[:, :dm])
    torch.cuda.synchronize()
    assert torch.all(Yp[:, dm:] == 7.0)
    assert relerr(to_host(Yp[:, :dm]), oracle_forward(d, w)) <= TOL["bf16"]


@pytest.mark.parametrize("name", ["128m_fwd", "370m_fwdbwd", "1p3b_fwdbwd"])
def test_full_size_forward_on_sampled_tokens(name):
    """Full-size configuration in the launch shape the bench times; the oracle
    evaluates a seeded sample of token rows (tokens are independent)."""
    w = inputs.WORKLOADS[name]
    d, Y = run_forward(w)
    rows = np.sort(np.random.default_rng(1).choice(w.n_tokens, size=192, replace=False))
    rows[:3] = [0, 1, w.n_tokens - 1]
    rows = np.unique(rows)
    assert np.all(np.isfinite(Y))
    assert relerr(Y[rows], oracle_forward(d, w, rows)) <= TOL["bf16"]


@pytest.mark.parametrize("N", inputs.SWEEP_TOKENS)
def test_inference_sweep_peaked_weights(N):
    w = inputs.WORKLOADS["1p3b_sweep"].with_tokens(N)
    d, Y = run_forward(w)
    rows = np.unique(np.random.default_rng(2).choice(N, size=min(N, 128), replace=False))
    assert relerr(Y[rows], oracle_forward(d, w, rows)) <= TOL["bf16"]


def test_deterministic_run_to_run():
    w = small_workload("det", 700, 2, 4, 128, "bf16")
    _, Y1 = run_forward(w, seed=3)
    _, Y2 = run_forward(w, seed=3)
    assert np.array_equal(Y1, Y2)
