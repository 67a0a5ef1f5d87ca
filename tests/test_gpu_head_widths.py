"""GPU parity of the fused bf16 kernels for the other head widths of the paper's ablation
(d_h = 64 and 256), forward and backward, against the fp64 oracle through the C ABI."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs, mhffn
from tests.helpers import TOL, device_inputs, relerr, small_workload, to_host
from tests.test_gpu_backward import GRADS, check_all, head_slice, run_backward
from tests.test_gpu_forward import oracle_forward, run_forward

pytestmark = pytest.mark.gpu

# (N, H, d_h, E, d_e): ragged token counts, one and several tiles, the split path of the
# forward (few tokens), more than 32 sub-networks, the paper's sub-network widths
SHAPES = [(1, 1, 64, 1, 32), (63, 2, 64, 3, 96), (300, 2, 64, 5, 64), (1000, 3, 64, 14, 192),
          (257, 1, 64, 40, 32), (130, 2, 64, 70, 32),
          # 96 sub-networks, the most the bf16 kernels take: W_r^T then fills a whole weight
          # stage of the token-major backward during its gating prologue
          (140, 1, 64, 96, 32),
          (1, 1, 256, 1, 32), (63, 2, 256, 3, 96), (300, 2, 256, 3, 64), (700, 1, 256, 4, 704),
          (257, 1, 256, 40, 32),
          # the token-major backward at d_h = 256 pipelines up to 32 sub-networks inside a wave
          # (two accumulator sets by parity of the tile: one, two and an odd number of tiles above
          # and here, the most sub-networks it takes, and one more: the register-staged kernel)
          (40, 1, 256, 2, 32), (130, 1, 256, 32, 32), (130, 1, 256, 33, 32)]


@pytest.mark.parametrize("N,H,dh,E,de", SHAPES)
def test_forward_small_shapes(N, H, dh, E, de):
    w = small_workload("hw_fwd", N, H, E, de, "bf16", dh=dh)
    d, Y = run_forward(w, seed=N + dh)
    assert relerr(Y, oracle_forward(d, w)) <= TOL["bf16"]


@pytest.mark.parametrize("N,H,dh,E,de", SHAPES)
def test_backward_small_shapes(N, H, dh, E, de):
    w = small_workload("hw_bwd", N, H, E, de, "bf16", dh=dh, backward=True)
    d, got = run_backward(w, seed=N + E + dh)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_all(got, ref, TOL["bf16"], single_subnetwork=(E == 1))


@pytest.mark.parametrize("N,H,E,de,route_weights", [
    # enough token tiles (48 x 8 heads) that a workgroup of the d_h = 256 forward walks the whole
    # intermediate dimension instead of a share of it (the small shapes above all run split):
    # ragged last tile, odd and even tile counts, one tile, more than 32 sub-networks, given
    # gating weights
    (6100, 8, 3, 64, False), (6200, 8, 32, 32, False), (6144, 8, 1, 32, False), (6100, 8, 2, 96, True),
    (6100, 8, 33, 32, False),
])
def test_dh256_forward_whole_depth_workgroups(N, H, E, de, route_weights):
    w = small_workload("hw_fwd_wide", N, H, E, de, "bf16", dh=256)
    d, Y = run_forward(w, seed=N + E, route_weights=route_weights)
    # the oracle on a sample of rows: first and last tile of 128, and a stride through the rest
    rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(N - 130, N), np.arange(0, N, 37)]))
    ref = oracle_forward(d, w, rows=rows, route_weights=route_weights)
    assert relerr(Y[rows], ref) <= TOL["bf16"]


@pytest.mark.parametrize("N,H,E,de", [
    # 54 groups of four 16-neuron blocks: 7 per XCD, less than a round, every group shares its
    # tokens out over four workgroups
    (2048, 9, 4, 96),
    # 300 groups (98 blocks per head: the last group of a head has two idle wave pairs): 38 per XCD
    # = 32 that take all tokens + 6 that share them out over two workgroups; ragged last block
    (1100, 12, 7, 224)])
def test_dh256_weight_major_rounds_and_token_shares(N, H, E, de):
    """d_h = 256 weight-major kernel on shapes whose neuron groups leave a partly filled last
    round per XCD: those groups write fp32 partials per token segment, summed in fixed order by
    a second kernel.  Every weight row against the oracle, bit-identical from run to run."""
    from tests.helpers import check_parity
    w = small_workload("hw_rounds", N, H, E, de, "bf16", dh=256, backward=True)
    desc = mhffn.Desc(N, H, 256, E, de, 0, 0, mhffn.BF16, mhffn.ROUTE_PARAMS, w.eps)
    a256 = lambda x: (x + 255) // 256 * 256
    assert mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD) > 2 * a256(N * H * E * 4) + a256(H * 64 * 256 * E * 4)
    d, got = run_backward(w, seed=N, want=("dW_gate", "dW_up", "dW_down"))
    _, again = run_backward(w, seed=N, want=("dW_gate", "dW_up", "dW_down"))
    for k in got:
        assert np.array_equal(got[k], again[k]), k
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_parity(got, {k: ref[k] for k in got}, TOL["bf16"], w.d_head, "rounds256")


@pytest.mark.parametrize("dh", [64, 256])
def test_strided_rows_and_partial_requests(dh):
    """X and dY as column slices of wider buffers with different row strides, a ragged token
    count, and a request for one weight gradient only (the weight-major kernels of these head
    widths stage their tiles from row-strided sources and skip the outputs not asked for)."""
    import torch
    w = small_workload("hw_strided", 333, 3, 5, 96, "bf16", dh=dh, backward=True)
    d = inputs.make_inputs(w, seed=21, with_dy=True)
    g = device_inputs(d, w.dtype)
    dm = w.d_model
    Xp = torch.zeros(w.n_tokens, dm + 64, dtype=g["X"].dtype, device="cuda")
    Xp[:, :dm] = g["X"]
    dYp = torch.zeros(w.n_tokens, dm + 192, dtype=g["X"].dtype, device="cuda")
    dYp[:, :dm] = g["dY"]
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    out = mhffn.backward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], dYp[:, :dm], w.eps)
    torch.cuda.synchronize()
    full = {k: to_host(v) for k, v in out.items()}
    check_all(full, ref, TOL["bf16"])
    only = mhffn.backward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], dYp[:, :dm], w.eps,
                          want=("dW_up",))
    torch.cuda.synchronize()
    assert set(only) == {"dW_up"}
    assert np.array_equal(to_host(only["dW_up"]), full["dW_up"])


@pytest.mark.parametrize("dh", [64, 256])
def test_very_large_row_stride_takes_the_generic_weight_major_kernel(dh):
    """Row strides of 2^24 elements and more do not fit the 32-bit row offsets of the kernels
    above; the backward then runs the register-staged kernel (1.3 GB buffers, 40 tokens)."""
    import torch
    w = small_workload("hw_wide", 40, 2, 3, 64, "bf16", dh=dh, backward=True)
    d = inputs.make_inputs(w, seed=22, with_dy=True)
    g = device_inputs(d, w.dtype)
    dm, ld = w.d_model, 1 << 24
    Xp = torch.zeros(w.n_tokens, ld, dtype=g["X"].dtype, device="cuda")
    Xp[:, :dm] = g["X"]
    dYp = torch.zeros(w.n_tokens, ld, dtype=g["X"].dtype, device="cuda")
    dYp[:, :dm] = g["dY"]
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    out = mhffn.backward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], dYp[:, :dm], w.eps,
                         want=("dW_gate", "dW_up", "dW_down", "d_route"))
    torch.cuda.synchronize()
    check_all({k: to_host(v) for k, v in out.items()}, {k: ref[k] for k in out}, TOL["bf16"])
    del Xp, dYp
    torch.cuda.empty_cache()


@pytest.mark.parametrize("dh", [64, 256])
def test_weights_mode(dh):
    w = small_workload("hw_weights", 333, 2, 6, 64, "bf16", dh=dh, backward=True)
    d, Y = run_forward(w, seed=5, route_weights=True)
    assert relerr(Y, oracle_forward(d, w, route_weights=True)) <= TOL["bf16"]
    d, got = run_backward(w, seed=5, route_weights=True)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["R"], d["dY"], w.eps,
                       orc.ROUTE_WEIGHTS)
    check_all(got, ref, TOL["bf16"])


@pytest.mark.parametrize("name,heads", [("paper_370m_dh64", (0, 9)), ("paper_370m_dh256", (1, 3))])
def test_full_size_on_whole_heads(name, heads):
    """The head-width ablation at full size: heads are independent, so the oracle evaluates
    whole heads (all tokens) and each is compared with its slice of the GPU result."""
    w = inputs.WORKLOADS[name]
    d, got = run_backward(w)
    _, Y = run_forward(w)
    for k in GRADS:
        assert np.all(np.isfinite(got[k])), k
    for h in heads:
        s = head_slice(d, w, h)
        cols = slice(h * w.d_head, (h + 1) * w.d_head)
        ref_y = orc.forward(s["X"], s["W_gate"], s["W_up"], s["W_down"], s["W_r"], w.eps)
        assert relerr(Y[:, cols], ref_y) <= TOL["bf16"]
        ref = orc.backward(s["X"], s["W_gate"], s["W_up"], s["W_down"], s["W_r"], s["dY"], w.eps)
        mine = {"dX": got["dX"][:, cols], "dW_gate": got["dW_gate"][h:h + 1],
                "dW_up": got["dW_up"][h:h + 1], "dW_down": got["dW_down"][h:h + 1],
                "d_route": got["d_route"][h:h + 1]}
        check_all(mine, ref, TOL["bf16"])
