"""Degenerate gates and extreme pre-activations on the GPU, forward and backward, for all
three head widths of the bf16 kernels and for the fp32 companions: one-hot, zero and negative
weights given as input, saturated gating logits, eps = 0 and a large eps, and gate
pre-activations far beyond the range where 2^(-m log2 e) is finite in fp32.  Every case is
compared with the fp64 oracle under the Frobenius and the per-row bound."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs, mhffn
from paper_2512_06989_amd.device import device_inputs, to_host
from tests.helpers import TOL, check_parity, small_workload

pytestmark = pytest.mark.gpu
GRADS = ("dX", "dW_gate", "dW_up", "dW_down", "d_route")
# (dtype, d_h, d_e): sub-network widths of the paper's head-width ablation, scaled down
KERNELS = [("bf16", 64, 96), ("bf16", 128, 64), ("bf16", 256, 96), ("f32", 128, 64), ("f32", 72, 40)]


def run_both(w, d, route_weights, eps):
    import torch
    g = device_inputs(d, w.dtype)
    route, mode, omode = ((g["R"], mhffn.ROUTE_WEIGHTS, orc.ROUTE_WEIGHTS) if route_weights
                          else (g["W_r"], mhffn.ROUTE_PARAMS, orc.ROUTE_PARAMS))
    Y = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], route, eps, mode)
    grads = mhffn.backward(g["X"], g["W_gate"], g["W_up"], g["W_down"], route, g["dY"], eps, mode)
    torch.cuda.synchronize()
    oroute = d["R"] if route_weights else d["W_r"]
    ref_y = orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], oroute, eps, omode)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], oroute, d["dY"], eps, omode)
    got = {k: to_host(v) for k, v in grads.items()}
    return to_host(Y), ref_y, got, ref


def workload(dtype, dh, de, N=300, H=2, E=5):
    return small_workload("edge", N, H, E, de, dtype, dh=dh, backward=True)


@pytest.mark.parametrize("dtype,dh,de", KERNELS)
@pytest.mark.parametrize("kind", ["one_hot", "zeros_and_negatives"])
def test_weights_given_as_input(dtype, dh, de, kind):
    """MHFFN_ROUTE_WEIGHTS with rows of R that are one-hot (a single sub-network per token
    and head, the others exactly 0), or a mix of exact zeros and negative values: the kernels
    divide by R nowhere (1/R is clamped where it is used as a factor)."""
    w = workload(dtype, dh, de)
    d = inputs.make_inputs(w, seed=11, with_dy=True, route_weights=True)
    rng = np.random.default_rng(5)
    R = np.zeros_like(d["R"])
    if kind == "one_hot":
        pick = rng.integers(0, w.n_sub, size=R.shape[:2])
        np.put_along_axis(R, pick[..., None], 1.0, axis=-1)
    else:
        R = rng.standard_normal(R.shape).astype(np.float32)
        R[rng.random(R.shape) < 0.3] = 0.0
    d["R"] = R
    Y, ref_y, got, ref = run_both(w, d, True, w.eps)
    check_parity({"Y": Y}, {"Y": ref_y}, TOL[dtype], dh, kind)
    check_parity(got, ref, TOL[dtype], dh, kind, route_weights=True)


@pytest.mark.parametrize("dtype,dh,de", KERNELS)
@pytest.mark.parametrize("eps", [0.0, 0.3])
def test_eps_zero_and_large(dtype, dh, de, eps):
    w = workload(dtype, dh, de)
    d = inputs.make_inputs(w, seed=12, with_dy=True)
    Y, ref_y, got, ref = run_both(w, d, False, eps)
    check_parity({"Y": Y}, {"Y": ref_y}, TOL[dtype], dh, "eps=%g" % eps)
    check_parity(got, ref, TOL[dtype], dh, "eps=%g" % eps)


@pytest.mark.parametrize("dtype,dh,de", KERNELS)
def test_saturated_gating_logits(dtype, dh, de):
    """Logits of eq:routing with a standard deviation of 40: most sigmoids are 0 or 1 to fp32
    precision (1 - s = 0 beyond |p| = 17), some are not.  The derivative through a saturated
    sigmoid is below fp32 resolution, so dW_r is compared on the scale of the un-saturated
    entries (whole-tensor bound) and not row by row."""
    w = workload(dtype, dh, de)
    d = inputs.make_inputs(w, seed=13, with_dy=True)
    wr = np.random.default_rng(6).standard_normal(d["W_r"].shape).astype(np.float32)
    d["W_r"] = inputs.round_to(wr * np.float32(40.0 / np.sqrt(dh)), dtype)
    Y, ref_y, got, ref = run_both(w, d, False, w.eps)
    p = np.einsum("lhj,hje->lhe", d["X"].reshape(w.n_tokens, w.n_heads, dh).astype(np.float64),
                  d["W_r"].astype(np.float64))
    assert np.mean(np.abs(p) > 17) > 0.5 and np.abs(p).max() > 80
    check_parity({"Y": Y}, {"Y": ref_y}, TOL[dtype], dh, "saturated")
    check_parity(got, ref, TOL[dtype], dh, "saturated", skip=("d_route",))
    scale = np.linalg.norm(ref["d_route"])
    assert np.all(np.isfinite(got["d_route"]))
    assert np.linalg.norm(got["d_route"] - ref["d_route"]) <= TOL[dtype] * scale


@pytest.mark.parametrize("dtype,dh,de", KERNELS)
def test_gate_preactivations_beyond_exp2_range(dtype, dh, de):
    """W_gate scaled so that the gate pre-activations have a standard deviation above 100:
    2^(-m log2 e) overflows to +inf for m < -89 and underflows to 0 for m > 104 in fp32;
    SiLU and its derivative must come out as 0 / m / 1 there, with no NaN."""
    w = workload(dtype, dh, de)
    d = inputs.make_inputs(w, seed=14, with_dy=True)
    wg = np.random.default_rng(7).standard_normal(d["W_gate"].shape).astype(np.float32)
    d["W_gate"] = inputs.round_to(wg * np.float32(110.0 / np.sqrt(dh)), dtype)
    m = np.einsum("lhj,hecj->lhec", d["X"].reshape(w.n_tokens, w.n_heads, dh).astype(np.float64),
                  d["W_gate"].astype(np.float64))
    assert m.min() < -300 and m.max() > 300
    Y, ref_y, got, ref = run_both(w, d, False, w.eps)
    check_parity({"Y": Y}, {"Y": ref_y}, TOL[dtype], dh, "large M")
    check_parity(got, ref, TOL[dtype], dh, "large M")
