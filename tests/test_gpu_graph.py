"""The entry points only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no host-side state after the first call), so they can be recorded into a
HIP graph.  Each replay is compared with the eager result, with eager work and
synchronisations between the replays."""
import pytest

from paper_2512_06989_amd import inputs, mhffn
from tests.helpers import device_inputs, small_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N", [64, 700])     # split forward (partials + reduce kernel) and plain
def test_forward_and_backward_replay_from_a_graph(N):
    import torch
    w = small_workload("graph", N, 4, 6, 128, "bf16", backward=True)
    d = inputs.make_inputs(w, seed=N, with_dy=True)
    g = device_inputs(d, "bf16")
    args = [g[k] for k in ("X", "W_gate", "W_up", "W_down", "W_r")]
    desc = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_PARAMS, w.eps)
    fws = torch.empty(max(mhffn.workspace_bytes(desc, mhffn.OP_FORWARD), 256), dtype=torch.uint8, device="cuda")
    bws = torch.empty(max(mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD), 256), dtype=torch.uint8, device="cuda")
    names = ("dX", "dW_gate", "dW_up", "dW_down", "d_route")
    like = dict(zip(names, args))

    def run(Y, grads):
        mhffn.forward(*args, w.eps, out=Y, workspace=fws)
        mhffn.backward(*args, g["dY"], w.eps, workspace=bws, out=grads)

    Y0, G0 = torch.empty_like(g["X"]), {k: torch.empty_like(v) for k, v in like.items()}
    run(Y0, G0)                                  # eager (also the first call: function attributes get set)
    torch.cuda.synchronize()
    Y1, G1 = torch.empty_like(g["X"]), {k: torch.empty_like(v) for k, v in like.items()}
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run(Y1, G1)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        Y1.fill_(7.0)
        for v in G1.values():
            v.fill_(7.0)
        scratch = torch.randn(1 << 20, device="cuda").sum()    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y1, Y0), rep
        for k in names:
            assert torch.equal(G1[k], G0[k]), (rep, k)
        del scratch


def test_first_call_may_be_captured_after_init():
    """mhffn_init raises every kernel's LDS limit, so a shape whose kernels may never have run
    in this process can be recorded into a graph without an eager call first."""
    import torch
    mhffn.init()
    w = small_workload("graph_init", 300, 3, 5, 192, "bf16", dh=64, backward=True)
    d = inputs.make_inputs(w, seed=2, with_dy=True)
    g = device_inputs(d, "bf16")
    args = [g[k] for k in ("X", "W_gate", "W_up", "W_down", "W_r")]
    desc = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_PARAMS, w.eps)
    fws = torch.empty(max(mhffn.workspace_bytes(desc, mhffn.OP_FORWARD), 256), dtype=torch.uint8, device="cuda")
    bws = torch.empty(max(mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD), 256), dtype=torch.uint8, device="cuda")
    names = ("dX", "dW_gate", "dW_up", "dW_down", "d_route")
    like = dict(zip(names, args))
    Y1, G1 = torch.empty_like(g["X"]), {k: torch.empty_like(v) for k, v in like.items()}
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            mhffn.forward(*args, w.eps, out=Y1, workspace=fws)
            mhffn.backward(*args, g["dY"], w.eps, workspace=bws, out=G1)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    Y0 = mhffn.forward(*args, w.eps, workspace=fws)
    G0 = mhffn.backward(*args, g["dY"], w.eps, workspace=bws)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y0)
    for k in names:
        assert torch.equal(G1[k], G0[k]), k
