"""The unfused GPU baseline against the oracle, the fused path against the
unfused one on random shapes, and the activation-memory comparison."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs, mhffn
from tests.helpers import TOL, device_inputs, relerr, small_workload, to_host

pytestmark = pytest.mark.gpu
GRADS = ("dX", "dW_gate", "dW_up", "dW_down", "d_route")


def run_unfused(w, seed, route_weights=False, backward=True):
    import torch
    d = inputs.make_inputs(w, seed=seed, with_dy=True, route_weights=route_weights)
    g = device_inputs(d, w.dtype)
    route, mode = (g["R"], mhffn.ROUTE_WEIGHTS) if route_weights else (g["W_r"], mhffn.ROUTE_PARAMS)
    res = mhffn.reference_unfused(g["X"], g["W_gate"], g["W_up"], g["W_down"], route, w.eps, mode,
                                  dY=g["dY"] if backward else None)
    torch.cuda.synchronize()
    if backward:
        return d, g, to_host(res[0]), {k: to_host(v) for k, v in res[1].items()}
    return d, g, to_host(res), None


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,H,dh,E,de", [(256, 2, 128, 4, 128), (1, 1, 8, 1, 3), (77, 3, 72, 5, 40),
                                          (300, 2, 64, 2, 200), (129, 1, 256, 3, 33)])
def test_unfused_matches_oracle(dtype, N, H, dh, E, de):
    w = small_workload("unf", N, H, E, de, dtype, dh=dh, backward=True)
    d, _, Y, grads = run_unfused(w, seed=N)
    tol = TOL[dtype] * (3 if dtype == "bf16" else 1)  # intermediates rounded to bf16 several times
    assert relerr(Y, orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)) <= tol
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    errs = {k: relerr(grads[k], ref[k]) for k in GRADS}
    if E == 1:
        errs.pop("d_route")   # O(eps) quantity, see the fused backward test
    assert all(e <= tol for e in errs.values()), str(errs)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_unfused_weights_mode(dtype):
    w = small_workload("unf_w", 200, 2, 5, 64, dtype, backward=True)
    d, _, Y, grads = run_unfused(w, seed=2, route_weights=True)
    tol = TOL[dtype] * (3 if dtype == "bf16" else 1)
    assert relerr(Y, orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["R"], w.eps,
                                 orc.ROUTE_WEIGHTS)) <= tol
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["R"], d["dY"], w.eps,
                       orc.ROUTE_WEIGHTS)
    errs = {k: relerr(grads[k], ref[k]) for k in GRADS}
    assert all(e <= tol for e in errs.values()), str(errs)


def test_unfused_strided_rows():
    """X and dY as column slices of wider buffers: Y takes dY's row stride, dX takes X's, and
    the padding columns of caller-provided outputs stay untouched."""
    import torch
    w = small_workload("unf_strided", 130, 2, 3, 64, "bf16", backward=True)
    d = inputs.make_inputs(w, seed=9, with_dy=True)
    g = device_inputs(d, w.dtype)
    dm = w.d_model
    Xp = torch.zeros(w.n_tokens, dm + 64, dtype=torch.bfloat16, device="cuda")
    Xp[:, :dm] = g["X"]
    dYp = torch.zeros(w.n_tokens, dm + 128, dtype=torch.bfloat16, device="cuda")
    dYp[:, :dm] = g["dY"]
    Yp = torch.full((w.n_tokens, dm + 128), 7.0, dtype=torch.bfloat16, device="cuda")
    dXp = torch.full((w.n_tokens, dm + 64), 9.0, dtype=torch.bfloat16, device="cuda")
    Y, grads = mhffn.reference_unfused(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps,
                                       dY=dYp[:, :dm], out={"Y": Yp[:, :dm], "dX": dXp[:, :dm]})
    torch.cuda.synchronize()
    assert torch.all(Yp[:, dm:] == 7.0) and torch.all(dXp[:, dm:] == 9.0)
    tol = 3 * TOL["bf16"]
    assert relerr(to_host(Y), orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)) <= tol
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    errs = {k: relerr(to_host(grads[k]), ref[k]) for k in GRADS}
    assert all(e <= tol for e in errs.values()), str(errs)
    # outputs allocated by the binding: Y with dY's stride, dX with X's
    Y2, g2 = mhffn.reference_unfused(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps,
                                     dY=dYp[:, :dm], want=("dX",))
    torch.cuda.synchronize()
    assert Y2.stride(0) == dm + 128 and g2["dX"].stride(0) == dm + 64
    assert torch.equal(Y2, Y) and torch.equal(g2["dX"], grads["dX"])


@pytest.mark.parametrize("seed", range(6))
def test_fused_agrees_with_unfused_on_random_shapes(seed):
    import torch
    rng = np.random.default_rng(100 + seed)
    N = int(rng.integers(1, 1500))
    H = int(rng.integers(1, 5))
    E = int(rng.integers(1, 40))
    de = 32 * int(rng.integers(1, 7))
    w = small_workload("prop", N, H, E, de, "bf16", backward=True)
    d, g, Yu, gu = run_unfused(w, seed=seed)
    Yf = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps)
    gf = mhffn.backward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], g["dY"], w.eps)
    torch.cuda.synchronize()
    assert relerr(to_host(Yf), Yu) <= 4 * TOL["bf16"], (N, H, E, de)
    for k in GRADS:
        if k == "d_route" and E == 1:
            continue
        assert relerr(to_host(gf[k]), gu[k]) <= 4 * TOL["bf16"], (k, N, H, E, de)


def test_activation_memory_fused_vs_unfused():
    """The fused forward needs no scratch at all; the unfused one materialises three
    [N][H][d_ff] tensors.  Checked from the workspace query and from the allocator."""
    import torch
    w = inputs.WORKLOADS["370m_fwdbwd"]
    d = inputs.make_inputs(w, seed=0, with_dy=False)
    g = device_inputs(d, w.dtype)
    desc = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_PARAMS, w.eps)
    inter = w.n_tokens * w.n_heads * w.d_ff * 2
    assert mhffn.workspace_bytes(desc, mhffn.OP_FORWARD) == 0
    need = mhffn.workspace_bytes(desc, mhffn.OP_UNFUSED_FORWARD)
    # the three intermediates, R and Z, and at most 64 MB of split-k partial tiles of the
    # product kernel (per-head outputs are only d_h wide, so their contraction is split)
    assert 3 * inter <= need <= 3 * inter + 2 * w.n_tokens * w.n_heads * (w.n_sub + 2) * 4 + (64 << 20)
    assert mhffn.workspace_bytes(desc, mhffn.OP_UNFUSED_BACKWARD) >= 4 * inter
    # fused backward: R and dp as [H][E][N] fp32, partial sums of dW_r, and (this shape's
    # weights alone fill a round of the chip badly) fp32 partial weight gradients of at most 8
    # token segments -- a multiple of the weights' size, not of the token count
    bwd = mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD)
    n_weights = 3 * w.n_heads * w.d_ff * w.d_head
    assert bwd < inter // 4
    assert bwd <= 2 * w.n_tokens * w.n_heads * w.n_sub * 4 + 8 * n_weights * 4 + (16 << 20)

    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    Yf = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps)
    torch.cuda.synchronize()
    fused_peak = torch.cuda.max_memory_allocated() - base
    del Yf
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    Yu = mhffn.reference_unfused(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps)
    torch.cuda.synchronize()
    unfused_peak = torch.cuda.max_memory_allocated() - base
    y_bytes = w.n_tokens * w.d_model * 2
    assert fused_peak <= y_bytes + (1 << 20)            # the output and nothing else
    assert unfused_peak >= y_bytes + 3 * inter
    assert unfused_peak / fused_peak > 3 * w.d_ff * w.n_heads / w.d_model
    del Yu


def test_unfused_rejects_small_workspace():
    import ctypes
    import torch
    w = small_workload("unf_ws", 64, 1, 2, 32, "bf16")
    d = inputs.make_inputs(w, seed=0, with_dy=False)
    g = device_inputs(d, w.dtype)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(mhffn.MhffnError) as ei:
        mhffn.reference_unfused(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps,
                                workspace=small)
    assert ei.value.status == 5


def test_dense_swiglu_is_the_one_head_one_subnetwork_case():
    """H = 1, E = 1, unit weights, a head as wide as the model (beyond what the gating kernel
    keeps in LDS, so the weights are given): the dense SwiGLU FFN that bench.py --module times
    beside the module.  Checked against a plain numpy SwiGLU and its hand-written gradients."""
    import torch
    N, dm, dff = 300, 2048, 384
    w = small_workload("swiglu", N, 1, 1, dff, "bf16", dh=dm, w_std=0.02, backward=True)
    d = inputs.make_inputs(w, seed=5, with_dy=True)
    g = device_inputs(d, "bf16")
    ones = torch.ones(N, 1, 1, device="cuda", dtype=torch.float32)
    Y, grads = mhffn.reference_unfused(g["X"], g["W_gate"], g["W_up"], g["W_down"], ones, 0.0,
                                       mhffn.ROUTE_WEIGHTS, dY=g["dY"],
                                       want=("dX", "dW_gate", "dW_up", "dW_down"))
    torch.cuda.synchronize()
    X, dY = d["X"].astype(np.float64), d["dY"].astype(np.float64)
    K, U, V = (d[k][0, 0].astype(np.float64) for k in ("W_gate", "W_up", "W_down"))
    G, Up = X @ K.T, X @ U.T
    sg = 1.0 / (1.0 + np.exp(-G))
    A = G * sg * Up
    dA = dY @ V.T
    dG = dA * Up * (sg + G * sg * (1.0 - sg))
    dU = dA * G * sg
    ref = {"Y": A @ V, "dX": dG @ K + dU @ U, "dW_gate": dG.T @ X, "dW_up": dU.T @ X, "dW_down": A.T @ dY}
    tol = 3 * TOL["bf16"]
    assert relerr(to_host(Y), ref["Y"]) <= tol
    for k in ("dX", "dW_gate", "dW_up", "dW_down"):
        got = to_host(grads[k])
        assert relerr(got.reshape(ref[k].shape), ref[k]) <= tol, k
