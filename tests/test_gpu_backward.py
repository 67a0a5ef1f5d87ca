"""GPU parity of the fused backward against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import inputs, mhffn
from tests.helpers import TOL, device_inputs, relerr, small_workload, to_host

pytestmark = pytest.mark.gpu
GRADS = ("dX", "dW_gate", "dW_up", "dW_down", "d_route")


def run_backward(w, seed=0, route_weights=False, want=GRADS):
    import torch
    d = inputs.make_inputs(w, seed=seed, with_dy=True, route_weights=route_weights)
    g = device_inputs(d, w.dtype)
    route, mode = (g["R"], mhffn.ROUTE_WEIGHTS) if route_weights else (g["W_r"], mhffn.ROUTE_PARAMS)
    out = mhffn.backward(g["X"], g["W_gate"], g["W_up"], g["W_down"], route, g["dY"], w.eps, mode,
                         want=want)
    torch.cuda.synchronize()
    return d, {k: to_host(v) for k, v in out.items()}


def head_slice(d, w, h):
    """Inputs of one head as a self-contained H=1 problem (heads are independent)."""
    cols = slice(h * w.d_head, (h + 1) * w.d_head)
    return dict(X=d["X"][:, cols], W_gate=d["W_gate"][h:h + 1], W_up=d["W_up"][h:h + 1],
                W_down=d["W_down"][h:h + 1], W_r=d["W_r"][h:h + 1], dY=d["dY"][:, cols])


def check_all(got, ref, tol, single_subnetwork=False):
    errs = {k: relerr(got[k], ref[k]) for k in got}
    if single_subnetwork and "d_route" in errs:
        # Degenerate case E = 1: r = s/(s+eps) is constant up to O(eps), so dW_r is the
        # difference of two numbers that agree to ~6 digits.  Its value is O(eps) of the
        # other gradients and carries no information in fp32; only its size is checked.
        assert np.abs(got["d_route"]).max() <= 1e-3 * np.abs(ref["dW_down"]).max()
        del errs["d_route"]
    assert all(e <= tol for e in errs.values()), str(errs)
    return errs


@pytest.mark.parametrize("N,H,E,de", [(256, 2, 4, 128), (1, 1, 1, 32), (63, 2, 3, 64),
                                       (65, 1, 5, 32), (257, 3, 2, 96), (1000, 2, 33, 32),
                                       (700, 1, 7, 160),
                                       # many sub-networks (three 32-wide blocks of gating logits),
                                       # token counts that leave the last 32-token block ragged
                                       (300, 1, 80, 32), (97, 2, 96, 32),
                                       # two and three tiles per head (the staging ring's start and
                                       # tail), and both sides of the largest E that the directly
                                       # staged token-major kernel holds in LDS
                                       (40, 1, 2, 32), (40, 2, 1, 96), (70, 1, 88, 32), (70, 1, 89, 32)])
def test_bf16_small_shapes_params_mode(N, H, E, de):
    w = small_workload("bwd_small", N, H, E, de, "bf16", backward=True)
    d, got = run_backward(w, seed=N + E)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_all(got, ref, TOL["bf16"], single_subnetwork=(E == 1))


@pytest.mark.parametrize("N,H,E,de", [
    # 300 neuron groups: 38 per XCD (32 that take all tokens + 6 that share them out over four
    # workgroups each), 34 on the last XCD (32 + 2)
    (2048, 20, 5, 384),
    # 272 groups of which the last of every head has idle waves (126 blocks of 16 neurons), two
    # token segments, a ragged last block of tokens
    (1100, 17, 9, 224)])
def test_weight_major_last_round_shares_tokens_out(N, H, E, de):
    """Shapes whose neuron groups fill more than one round of workgroups per XCD with a partly
    filled last round: those groups leave fp32 partials per token segment that a second kernel
    adds up in fixed order; the others store their gradients directly.  Every weight row against
    the oracle, bit-identical from run to run."""
    from tests.helpers import check_parity
    w = small_workload("bwd_rounds", N, H, E, de, "bf16", backward=True)
    # the workspace holds more than R, dp and the dW_r partials: the token-segment partials
    desc = mhffn.Desc(N, H, 128, E, de, 0, 0, mhffn.BF16, mhffn.ROUTE_PARAMS, w.eps)
    a256 = lambda x: (x + 255) // 256 * 256
    assert mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD) > 2 * a256(N * H * E * 4) + a256(H * 64 * 128 * E * 4)
    d, got = run_backward(w, seed=N, want=("dW_gate", "dW_up", "dW_down"))
    _, again = run_backward(w, seed=N, want=("dW_gate", "dW_up", "dW_down"))
    for k in got:
        assert np.array_equal(got[k], again[k]), k
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_parity(got, {k: ref[k] for k in got}, TOL["bf16"], w.d_head, "rounds")


def test_bf16_weights_mode_returns_dr():
    w = small_workload("bwd_weights", 333, 2, 6, 64, "bf16", backward=True)
    d, got = run_backward(w, seed=4, route_weights=True)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["R"], d["dY"], w.eps,
                       orc.ROUTE_WEIGHTS)
    check_all(got, ref, TOL["bf16"])


def test_f32_tiny_config_backward():
    """fp32 companion kernels at the fp32 tolerance (the tiny configuration's shape)."""
    from dataclasses import replace
    w = replace(inputs.WORKLOADS["tiny_f32"], backward=True)
    d, got = run_backward(w)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_all(got, ref, TOL["f32"])


@pytest.mark.parametrize("N", [1, 31, 65, 300])
def test_f32_ragged_and_generic_shapes(N):
    w = inputs.Workload("f32_bwd_generic", N, 3, 72, 5, 40, "f32", w_std=0.1, route_scale=3.0,
                        backward=True)
    d, got = run_backward(w, seed=N)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_all(got, ref, TOL["f32"])


@pytest.mark.parametrize("dh,E,de", [(64, 6, 192), (256, 3, 704), (248, 5, 40), (232, 2, 96)])
def test_f32_other_head_widths(dh, E, de):
    """The paper's head-width variants (d_h = 64, 256 with d_e = 8/3 d_h rounded up to a
    multiple of 64) and two odd widths through the shape-generic fp32 kernels.  The fp32
    backward keeps whole d_h-wide tiles in LDS: weight chunks of 32 neurons up to d_h = 232,
    of 16 beyond (d_h = 248, 256 here), with a ragged last chunk (d_e = 40)."""
    import torch
    w = inputs.Workload("f32_head_width", 150, 2, dh, E, de, "f32", w_std=0.05, route_scale=2.0,
                        backward=True)
    d = inputs.make_inputs(w, seed=dh, with_dy=True)
    g = device_inputs(d, w.dtype)
    Y = mhffn.forward(g["X"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], w.eps)
    torch.cuda.synchronize()
    ref_y = orc.forward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], w.eps)
    assert relerr(to_host(Y), ref_y) <= TOL["f32"]
    _, got = run_backward(w, seed=dh)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    check_all(got, ref, TOL["f32"])


def test_f32_backward_refuses_what_does_not_fit_in_lds():
    """d_h = 256 with 200 sub-networks: the token tile, a 16-neuron weight chunk and the
    per-token gating rows exceed 160 KB of LDS; the call has to refuse rather than compute."""
    w = inputs.Workload("f32_too_wide", 40, 1, 256, 200, 16, "f32", backward=True)
    with pytest.raises(mhffn.MhffnError) as err:
        run_backward(w, seed=1)
    assert err.value.status == 3   # MHFFN_ERR_UNSUPPORTED


def test_f32_weights_mode_returns_dr():
    w = small_workload("bwd_weights_f32", 200, 2, 6, 64, "f32", backward=True)
    d, got = run_backward(w, seed=4, route_weights=True)
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["R"], d["dY"], w.eps,
                       orc.ROUTE_WEIGHTS)
    check_all(got, ref, TOL["f32"])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_strided_rows_dx_takes_the_stride_of_x(dtype):
    """X and dY are column slices of wider buffers (ld_x, ld_y > d_model, different from each
    other).  The binding allocates dX with X's row stride, the kernels write only the
    d_model columns of each row, and a caller-provided strided dX keeps its padding."""
    import torch
    w = small_workload("bwd_strided", 130, 2, 3, 64, dtype, backward=True)
    d = inputs.make_inputs(w, seed=9, with_dy=True)
    g = device_inputs(d, w.dtype)
    dm, td = w.d_model, g["X"].dtype
    Xp = torch.zeros(w.n_tokens, dm + 64, dtype=td, device="cuda")
    Xp[:, :dm] = g["X"]
    dYp = torch.zeros(w.n_tokens, dm + 128, dtype=td, device="cuda")
    dYp[:, :dm] = g["dY"]
    ref = orc.backward(d["X"], d["W_gate"], d["W_up"], d["W_down"], d["W_r"], d["dY"], w.eps)
    out = mhffn.backward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], dYp[:, :dm], w.eps)
    torch.cuda.synchronize()
    assert out["dX"].stride(0) == dm + 64 and out["dX"].shape == (w.n_tokens, dm)
    check_all({k: to_host(v) for k, v in out.items()}, ref, TOL[dtype])
    dXp = torch.full((w.n_tokens, dm + 64), 7.0, dtype=td, device="cuda")
    out = mhffn.backward(Xp[:, :dm], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], dYp[:, :dm], w.eps,
                         want=("dX",), out={"dX": dXp[:, :dm]})
    torch.cuda.synchronize()
    assert torch.all(dXp[:, dm:] == 7.0)
    assert relerr(to_host(dXp[:, :dm]), ref["dX"]) <= TOL[dtype]


def test_partial_gradient_requests():
    w = small_workload("bwd_partial", 300, 2, 3, 64, "bf16", backward=True)
    d, full = run_backward(w, seed=8)
    _, only_x = run_backward(w, seed=8, want=("dX",))
    _, only_w = run_backward(w, seed=8, want=("dW_up", "d_route"))
    assert np.array_equal(only_x["dX"], full["dX"])
    assert np.array_equal(only_w["dW_up"], full["dW_up"])
    assert np.array_equal(only_w["d_route"], full["d_route"])


def test_deterministic_run_to_run():
    w = small_workload("bwd_det", 900, 2, 4, 128, "bf16", backward=True)
    _, g1 = run_backward(w, seed=3)
    _, g2 = run_backward(w, seed=3)
    for k in GRADS:
        assert np.array_equal(g1[k], g2[k]), k


@pytest.mark.parametrize("name,heads", [("370m_fwdbwd", (0, 5)), ("1p3b_fwdbwd", (3, 15))])
def test_full_size_backward_on_whole_heads(name, heads):
    """Full-size configuration in the launch shape the bench times.  Heads are
    independent, so the oracle evaluates whole heads (all N tokens: the weight
    gradients sum over every token) and each is compared with its slice."""
    w = inputs.WORKLOADS[name]
    d, got = run_backward(w)
    for k in GRADS:
        assert np.all(np.isfinite(got[k])), k
    for h in heads:
        s = head_slice(d, w, h)
        ref = orc.backward(s["X"], s["W_gate"], s["W_up"], s["W_down"], s["W_r"], s["dY"], w.eps)
        cols = slice(h * w.d_head, (h + 1) * w.d_head)
        mine = {"dX": got["dX"][:, cols], "dW_gate": got["dW_gate"][h:h + 1],
                "dW_up": got["dW_up"][h:h + 1], "dW_down": got["dW_down"][h:h + 1],
                "d_route": got["d_route"][h:h + 1]}
        check_all(mine, ref, TOL["bf16"])


def test_empty_batch_zero_gradients_and_all_phase_events():
    """N = 0: the parameter gradients are zero, and every phase event is recorded so that the
    caller's elapsed-time queries between them succeed."""
    import torch
    from bench import HipEvents
    H, E, de, dh = 2, 3, 64, 128
    X = torch.empty(0, H * dh, dtype=torch.bfloat16, device="cuda")
    W = [torch.randn(H, E, de, dh, device="cuda").to(torch.bfloat16) for _ in range(3)]
    Wr = torch.randn(H, dh, E, device="cuda").to(torch.bfloat16)
    hip = HipEvents()
    ev = hip.create(4)
    out = {k: torch.full_like(t, 3.0) for k, t in zip(("dW_gate", "dW_up", "dW_down", "d_route"), W + [Wr])}
    out["dX"] = torch.empty_like(X)
    res = mhffn.backward(X, *W, Wr, X.clone(), out=out, phase_events=ev)
    torch.cuda.synchronize()
    for k in ("dW_gate", "dW_up", "dW_down", "d_route"):
        assert torch.count_nonzero(res[k]) == 0, k
    for i in range(3):
        assert hip.elapsed_ms(ev[i], ev[i + 1]) >= 0.0
