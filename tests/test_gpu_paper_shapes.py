"""The paper's own shapes (sub-networks of width 384 / 256, E = 7, 8, 15, 22) through the
fused kernels: forward on sampled tokens, backward on one whole head, against the oracle."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs, mhffn
from tests.helpers import TOL, device_inputs, relerr, to_host
from tests.test_gpu_backward import GRADS, check_all, head_slice

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["paper_128m", "paper_370m", "paper_1p3b", "paper_bench"])
def test_forward_on_sampled_tokens(name):
    import torch
    w = inputs.WORKLOADS[name]
    d = inputs.make_inputs(w, seed=0, with_dy=False)
    g = device_inputs(d, w.dtype)
    Y = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps)
    torch.cuda.synchronize()
    Y = to_host(Y)
    rows = np.unique(np.random.default_rng(3).choice(w.n_tokens, size=160, replace=False))
    ref = orc.forward(d["X"][rows], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)
    assert np.all(np.isfinite(Y))
    assert relerr(Y[rows], ref) <= TOL["bf16"]


@pytest.mark.parametrize("name,head", [("paper_370m", 2), ("paper_1p3b", 9)])
def test_backward_on_one_whole_head(name, head):
    import torch
    w = inputs.WORKLOADS[name]
    d = inputs.make_inputs(w, seed=0, with_dy=True)
    g = device_inputs(d, w.dtype)
    out = mhffn.backward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], g["dY"], w.eps)
    torch.cuda.synchronize()
    got = {k: to_host(v) for k, v in out.items()}
    s = head_slice(d, w, head)
    ref = orc.backward(s["X"], s["W_gate"], s["W_up"], s["W_down"], s["W_r"], s["dY"], w.eps)
    cols = slice(head * w.d_head, (head + 1) * w.d_head)
    mine = {"dX": got["dX"][:, cols], "dW_gate": got["dW_gate"][head:head + 1],
            "dW_up": got["dW_up"][head:head + 1], "dW_down": got["dW_down"][head:head + 1],
            "d_route": got["d_route"][head:head + 1]}
    check_all(mine, ref, TOL["bf16"])


def test_empty_batch_gives_zero_weight_gradients():
    """N = 0: nothing to read, dX empty, weight gradients are exactly zero."""
    import torch
    H, E, de, dh = 2, 3, 64, 128
    X = torch.empty(0, H * dh, dtype=torch.bfloat16, device="cuda")
    W = [torch.randn(H, E, de, dh, device="cuda").to(torch.bfloat16) for _ in range(3)]
    Wr = torch.randn(H, dh, E, device="cuda").to(torch.bfloat16)
    Y = mhffn.forward(X, *W, Wr)
    assert Y.shape == (0, H * dh)
    out = {k: torch.full_like(t, 3.0) for k, t in (("dW_gate", W[0]), ("dW_up", W[1]),
                                                   ("dW_down", W[2]), ("d_route", Wr))}
    out["dX"] = torch.empty_like(X)
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    res = mhffn.backward(X, *W, Wr, X.clone(), workspace=ws, out=out)
    torch.cuda.synchronize()
    for k in ("dW_gate", "dW_up", "dW_down", "d_route"):
        assert torch.count_nonzero(res[k]) == 0, k
