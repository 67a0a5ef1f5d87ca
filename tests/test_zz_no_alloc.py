"""mhffn_forward_static (the forward for callers that cannot allocate: its scratch is a static
device buffer of the library) against mhffn_forward, through the C ABI: two calls in a row, the
second with a smaller input, each bit-identical to the allocating entry point; a shape that
needs no scratch; and the refusal of a problem whose scratch exceeds the static buffer."""
import ctypes

import pytest

from paper_2512_06989_amd import inputs, mhffn
from paper_2512_06989_amd.device import device_inputs
from tests.helpers import small_workload

ARGS = ("X", "W_gate", "W_up", "W_down", "W_r")


@pytest.mark.gpu
def test_two_calls_in_a_row_second_one_smaller():
    import torch
    for N, seed in ((1000, 1), (64, 2), (300, 3)):   # split forward: partials go through the scratch
        w = small_workload("static", N, 4, 6, 128, "bf16")
        desc_w = inputs.make_inputs(w, seed=seed, with_dy=False)
        g = device_inputs(desc_w, "bf16")
        a = [g[k] for k in ARGS]
        d = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_PARAMS, w.eps)
        assert 0 < mhffn.workspace_bytes(d, mhffn.OP_FORWARD) <= (40 << 20)
        want = mhffn.forward(*a, w.eps)
        got = torch.full_like(g["X"], 7.0)
        # number of allocation requests the caching allocator has served so far (monotonic: a
        # tensor freed by the garbage collector in between does not change it)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        mhffn.forward_static(*a, got, w.eps)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        torch.cuda.synchronize()
        assert torch.equal(got, want), N


@pytest.mark.gpu
def test_weights_mode_and_a_shape_without_scratch():
    import torch
    w = small_workload("static_big", 9000, 16, 3, 64, "bf16")    # 36 token tiles x 16 heads: no split
    d_in = inputs.make_inputs(w, seed=4, with_dy=False, route_weights=True)
    g = device_inputs(d_in, "bf16")
    d = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_WEIGHTS, w.eps)
    assert mhffn.workspace_bytes(d, mhffn.OP_FORWARD) == 0
    want = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["R"], w.eps, mhffn.ROUTE_WEIGHTS)
    got = torch.empty_like(g["X"])
    mhffn.forward_static(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["R"], got, w.eps, mhffn.ROUTE_WEIGHTS)
    torch.cuda.synchronize()
    assert torch.equal(got, want)


def test_refuses_more_scratch_than_the_static_buffer():
    """d_h = 256, 1024 tokens, 8 heads: 8 splits x 1024 x 2048 fp32 partials = 64 MiB.  Checked
    on the host before anything is launched (runs without a GPU)."""
    d = mhffn.Desc(1024, 8, 256, 8, 704, 0, 0, mhffn.BF16, mhffn.ROUTE_PARAMS, 1e-6)
    assert mhffn.workspace_bytes(d, mhffn.OP_FORWARD) > (40 << 20)
    fake = ctypes.c_void_p(0x10000)
    rc = mhffn.load().mhffn_forward_static(ctypes.byref(d), *([fake] * 6), None)
    assert rc == 7 and "static" in mhffn.status_string(rc)
