"""Full-size parity in the launch shapes the bench times: every token row and every head of
the 128M / 370M / 1.3B configurations and of the inference sweep against the fp64 oracle,
with the whole-tensor Frobenius bound and the per-row bound (tests/helpers.py)."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs
from tests.helpers import TOL, check_parity
from tests.test_gpu_backward import run_backward
from tests.test_gpu_forward import run_forward

pytestmark = pytest.mark.gpu


def _report(name, figs):
    print("  %s: " % name + ", ".join("%s %.2e/%.2e" % (k, f, r) for k, (f, r) in figs.items()),
          flush=True)


@pytest.mark.parametrize("name", ["128m_fwd", "370m_fwdbwd", "1p3b_fwdbwd"])
def test_forward_every_row(name):
    w = inputs.WORKLOADS[name]
    d, Y = run_forward(w)
    ref = orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)
    _report(name, check_parity({"Y": Y}, {"Y": ref}, TOL["bf16"], w.d_head, name))


@pytest.mark.parametrize("N", inputs.SWEEP_TOKENS)
def test_inference_sweep_every_row(N):
    w = inputs.WORKLOADS["1p3b_sweep"].with_tokens(N)
    d, Y = run_forward(w)
    ref = orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)
    _report(w.name, check_parity({"Y": Y}, {"Y": ref}, TOL["bf16"], w.d_head, w.name))


@pytest.mark.parametrize("name", ["370m_fwdbwd", "1p3b_fwdbwd"])
def test_backward_every_head(name):
    w = inputs.WORKLOADS[name]
    d, got = run_backward(w)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    _report(name, check_parity(got, ref, TOL["bf16"], w.d_head, name))
