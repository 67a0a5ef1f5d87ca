"""Pins of the fp64 oracle against what the paper and the mathematics fix.

None of these tests calls the oracle to produce its own expected value: each
expected value comes from an independent numpy/scipy expression of a special
case, from pure-Python element loops, from a closed form, or from finite
differences."""
import itertools
import math

import numpy as np
import pytest
from scipy.special import expit

from oracle import mhffn_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def make(seed, N, H, dh, E, de, wscale=0.5):
    return dict(
        X=rnd(seed, N, H * dh),
        Wg=rnd(seed + 1, H, E, de, dh, scale=wscale),
        Wu=rnd(seed + 2, H, E, de, dh, scale=wscale),
        Wd=rnd(seed + 3, H, E, de, dh, scale=wscale),
        Wr=rnd(seed + 4, H, dh, E, scale=wscale),
    )


def relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ---------------------------------------------------------------- brute force
def brute_forward(X, Wg, Wu, Wd, Wr, eps):
    """Pure-Python element loops straight from the definitions (no numpy math)."""
    N = len(X)
    H, E, de, dh = len(Wg), len(Wg[0]), len(Wg[0][0]), len(Wg[0][0][0])
    Y = [[0.0] * (H * dh) for _ in range(N)]
    for l in range(N):
        for h in range(H):
            q = [X[l][h * dh + j] for j in range(dh)]
            sig = []
            for e in range(E):
                p = sum(q[j] * Wr[h][j][e] for j in range(dh))
                sig.append(1.0 / (1.0 + math.exp(-p)))
            Z = sum(sig)
            for j in range(dh):
                tot = 0.0
                for e in range(E):
                    r = sig[e] / (Z + eps)
                    ye = 0.0
                    for c in range(de):
                        g = sum(q[t] * Wg[h][e][c][t] for t in range(dh))
                        u = sum(q[t] * Wu[h][e][c][t] for t in range(dh))
                        silu = g / (1.0 + math.exp(-g))
                        ye += silu * u * Wd[h][e][c][j]
                    tot += r * ye
                Y[l][h * dh + j] = tot
    return Y


@pytest.mark.parametrize("shape", [(3, 2, 4, 3, 5), (1, 1, 2, 1, 1), (5, 3, 8, 2, 4)])
@pytest.mark.parametrize("eps", [0.0, 1e-6, 0.3])
def test_bruteforce_forward(shape, eps):
    d = make(10, *shape)
    Y = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], eps)
    Yb = np.array(brute_forward(d["X"].tolist(), d["Wg"].tolist(), d["Wu"].tolist(),
                                d["Wd"].tolist(), d["Wr"].tolist(), eps))
    assert relerr(Y, Yb) < 1e-13


# ------------------------------------------------------- special cases (numpy)
def test_swiglu_special_case():
    """H=1, E=1, eps=0 => R == 1 and the layer is a standard SwiGLU FFN."""
    N, dh, de = 17, 24, 40
    d = make(20, N, 1, dh, 1, de)
    Y = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], 0.0)
    W_gate, W_up, W_down = d["Wg"][0, 0].T, d["Wu"][0, 0].T, d["Wd"][0, 0]
    G = d["X"] @ W_gate
    ref = ((d["X"] @ W_up) * (G * expit(G))) @ W_down
    assert relerr(Y, ref) < 1e-13


def ffn_kv(Q, K, U, V):
    M = Q @ K.T
    return ((M * expit(M)) * (Q @ U.T)) @ V


def test_one_hot_weights_select_one_subnetwork():
    N, H, dh, E, de = 9, 3, 8, 4, 6
    d = make(30, N, H, dh, E, de)
    pick = np.random.default_rng(5).integers(0, E, size=(N, H))
    R = np.zeros((N, H, E))
    for l, h in itertools.product(range(N), range(H)):
        R[l, h, pick[l, h]] = 1.0
    Y = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], R, 0.0, orc.ROUTE_WEIGHTS)
    for l, h in itertools.product(range(N), range(H)):
        e = pick[l, h]
        q = d["X"][l:l + 1, h * dh:(h + 1) * dh]
        ref = ffn_kv(q, d["Wg"][h, e], d["Wu"][h, e], d["Wd"][h, e])[0]
        assert relerr(Y[l, h * dh:(h + 1) * dh], ref) < 1e-13


def test_saturated_logits_select_one_subnetwork():
    """Logits of +-40 through eq:routing: weight 1/(1+eps) on one sub-network."""
    N, H, dh, E, de = 6, 2, 8, 3, 5
    eps = 1e-3
    d = make(31, N, H, dh, E, de)
    X = d["X"].copy()
    Wr = np.zeros((H, dh, E))
    star = [2, 0]
    for h in range(H):
        X[:, h * dh] = 1.0
        Wr[h, 0, :] = -40.0
        Wr[h, 0, star[h]] = 40.0
    Y = orc.forward(X, d["Wg"], d["Wu"], d["Wd"], Wr, eps)
    for h in range(H):
        e = star[h]
        ref = ffn_kv(X[:, h * dh:(h + 1) * dh], d["Wg"][h, e], d["Wu"][h, e], d["Wd"][h, e])
        assert relerr(Y[:, h * dh:(h + 1) * dh], ref / (1.0 + eps)) < 1e-12


def test_uniform_gate_is_naive_mhffn():
    """W_r = 0 => r = 0.5/(0.5E+eps) for all e => constant x un-gated MH-FFN
    over the concatenated intermediate dimension."""
    N, H, dh, E, de = 11, 3, 8, 5, 7
    eps = 1e-2
    d = make(40, N, H, dh, E, de)
    Y = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], np.zeros((H, dh, E)), eps)
    c = 0.5 / (0.5 * E + eps)
    for h in range(H):
        q = d["X"][:, h * dh:(h + 1) * dh]
        ref = c * ffn_kv(q, d["Wg"][h].reshape(E * de, dh), d["Wu"][h].reshape(E * de, dh),
                         d["Wd"][h].reshape(E * de, dh))
        assert relerr(Y[:, h * dh:(h + 1) * dh], ref) < 1e-13


def test_identical_subnetworks():
    N, H, dh, E, de = 7, 2, 8, 4, 6
    eps = 0.05
    d = make(50, N, H, dh, E, de)
    for k in ("Wg", "Wu", "Wd"):
        d[k][:] = d[k][:, :1]
    Y, R = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], eps, return_weights=True)
    for h in range(H):
        q = d["X"][:, h * dh:(h + 1) * dh]
        Z = expit(q @ d["Wr"][h]).sum(axis=1, keepdims=True)
        ref = (Z / (Z + eps)) * ffn_kv(q, d["Wg"][h, 0], d["Wu"][h, 0], d["Wd"][h, 0])
        assert relerr(Y[:, h * dh:(h + 1) * dh], ref) < 1e-13


@pytest.mark.parametrize("b", [1, 7, 6, 24, 5])
def test_block_size_independence(b):
    """eq:flash-ffn-loop: accumulating blocks of b rows of K,U,V gives the same O."""
    N, H, dh, E, de = 8, 2, 8, 4, 6
    eps = 1e-6
    d = make(60, N, H, dh, E, de)
    Y = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], eps)
    dff = E * de
    for h in range(H):
        q = d["X"][:, h * dh:(h + 1) * dh]
        s = expit(q @ d["Wr"][h])
        R = s / (s.sum(axis=1, keepdims=True) + eps)
        Rcols = np.repeat(R, de, axis=1)  # weight of the sub-network owning column c
        K, U, V = (d[k][h].reshape(dff, dh) for k in ("Wg", "Wu", "Wd"))
        O = np.zeros((N, dh))
        for m in range(0, dff, b):
            M = q @ K[m:m + b].T
            A = (M * expit(M)) * (q @ U[m:m + b].T) * Rcols[:, m:m + b]
            O = O + A @ V[m:m + b]
        assert relerr(Y[:, h * dh:(h + 1) * dh], O) < 1e-12


def test_token_permutation_equivariance():
    N, H, dh, E, de = 13, 2, 8, 3, 5
    d = make(70, N, H, dh, E, de)
    dY = rnd(71, N, H * dh)
    perm = np.random.default_rng(3).permutation(N)
    args = (d["Wg"], d["Wu"], d["Wd"], d["Wr"])
    Y = orc.forward(d["X"], *args, 1e-6)
    Yp = orc.forward(d["X"][perm], *args, 1e-6)
    assert np.array_equal(Yp, Y[perm])
    g = orc.backward(d["X"], *args, dY, 1e-6)
    gp = orc.backward(d["X"][perm], *args, dY[perm], 1e-6)
    assert relerr(gp["dX"], g["dX"][perm]) < 1e-12
    for k in ("dW_gate", "dW_up", "dW_down", "d_route"):
        assert relerr(gp[k], g[k]) < 1e-12


def test_head_independence():
    N, H, dh, E, de = 6, 3, 8, 2, 4
    d = make(80, N, H, dh, E, de)
    base = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], 1e-6)
    for key in ("X", "Wg", "Wu", "Wd", "Wr"):
        m = {k: v.copy() for k, v in d.items()}
        if key == "X":
            m["X"][:, dh:2 * dh] += 1.0
        else:
            m[key][1] *= 1.5
        out = orc.forward(m["X"], m["Wg"], m["Wu"], m["Wd"], m["Wr"], 1e-6)
        changed = np.any(out != base, axis=0).reshape(H, dh).any(axis=1)
        assert changed.tolist() == [False, True, False], key


def test_linearity_in_down_projection_and_weights():
    N, H, dh, E, de = 6, 2, 8, 3, 4
    d = make(90, N, H, dh, E, de)
    R = np.abs(rnd(91, N, H, E))
    R2 = np.abs(rnd(92, N, H, E))
    f = lambda Wd, R_: orc.forward(d["X"], d["Wg"], d["Wu"], Wd, R_, 0.0, orc.ROUTE_WEIGHTS)
    assert relerr(f(3.5 * d["Wd"], R), 3.5 * f(d["Wd"], R)) < 1e-13
    assert relerr(f(d["Wd"], R + 2 * R2), f(d["Wd"], R) + 2 * f(d["Wd"], R2)) < 1e-13
    Wd2 = rnd(93, *d["Wd"].shape)
    assert relerr(f(d["Wd"] + Wd2, R), f(d["Wd"], R) + f(Wd2, R)) < 1e-13


@pytest.mark.parametrize("eps", [0.0, 1e-6, 0.5])
def test_gating_weights_row_sums(eps):
    N, H, dh, E, de = 20, 2, 8, 5, 2
    d = make(100, N, H, dh, E, de, wscale=2.0)
    _, R = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], eps, return_weights=True)
    assert np.all(R > 0) and np.all(R < 1)
    for h in range(H):
        Z = expit(d["X"][:, h * dh:(h + 1) * dh] @ d["Wr"][h]).sum(axis=1)
        assert np.allclose(R[:, h].sum(axis=1), Z / (Z + eps), rtol=0, atol=1e-15 * E)
    if eps == 0.0:
        assert np.allclose(R.sum(axis=2), 1.0, rtol=0, atol=1e-15 * E)


# ------------------------------------------------------------------- backward
def _fd(fun, x, h=1e-6):
    g = np.zeros_like(x)
    flat, gf = x.reshape(-1), g.reshape(-1)
    for i in range(flat.size):
        old = flat[i]
        flat[i] = old + h
        fp = fun()
        flat[i] = old - h
        fm = fun()
        flat[i] = old
        gf[i] = (fp - fm) / (2 * h)
    return g


@pytest.mark.parametrize("shape", [(3, 2, 4, 3, 5), (4, 1, 6, 2, 3)])
def test_backward_matches_finite_differences_params_mode(shape):
    d = make(110, *shape)
    G = rnd(111, shape[0], shape[1] * shape[2])
    eps = 1e-3
    loss = lambda: float((orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], eps) * G).sum())
    g = orc.backward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], G, eps)
    for key, name in (("X", "dX"), ("Wg", "dW_gate"), ("Wu", "dW_up"), ("Wd", "dW_down"),
                      ("Wr", "d_route")):
        fd = _fd(loss, d[key])
        assert relerr(g[name], fd) < 1e-7, name


def test_backward_matches_finite_differences_weights_mode():
    N, H, dh, E, de = 3, 2, 4, 3, 5
    d = make(120, N, H, dh, E, de)
    R = np.abs(rnd(121, N, H, E)) + 0.1
    G = rnd(122, N, H * dh)
    loss = lambda: float((orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], R, 0.0,
                                      orc.ROUTE_WEIGHTS) * G).sum())
    g = orc.backward(d["X"], d["Wg"], d["Wu"], d["Wd"], R, G, 0.0, orc.ROUTE_WEIGHTS)
    for arr, name in ((d["X"], "dX"), (d["Wg"], "dW_gate"), (d["Wu"], "dW_up"),
                      (d["Wd"], "dW_down"), (R, "d_route")):
        fd = _fd(loss, arr)
        assert relerr(g[name], fd) < 1e-7, name


def test_dr_is_inner_product_with_subnetwork_output():
    """dr[l,h,e] = <dy[l,h,:], y_e[l,h,:]>; the row accumulator restarts per e."""
    N, H, dh, E, de = 7, 2, 8, 4, 5
    d = make(130, N, H, dh, E, de)
    R = np.abs(rnd(131, N, H, E))
    dY = rnd(132, N, H * dh)
    g = orc.backward(d["X"], d["Wg"], d["Wu"], d["Wd"], R, dY, 0.0, orc.ROUTE_WEIGHTS)
    ref = np.zeros((N, H, E))
    for h, e in itertools.product(range(H), range(E)):
        ye = ffn_kv(d["X"][:, h * dh:(h + 1) * dh], d["Wg"][h, e], d["Wu"][h, e], d["Wd"][h, e])
        ref[:, h, e] = (dY[:, h * dh:(h + 1) * dh] * ye).sum(axis=1)
    assert relerr(g["d_route"], ref) < 1e-13
    Ysub = orc.subnet_outputs(d["X"], d["Wg"], d["Wu"], d["Wd"])
    assert relerr(np.einsum("lhej,lhj->lhe", Ysub, dY.reshape(N, H, dh)), ref) < 1e-13


def test_dlogits_sum_matches_row_sum_derivative():
    """With eps = 0 the weights sum to one, so a loss that reads only sum_e r[e]
    (every sub-network returning the same vector) has zero gradient w.r.t. W_r."""
    N, H, dh, E, de = 6, 2, 8, 4, 3
    d = make(140, N, H, dh, E, de)
    for k in ("Wg", "Wu", "Wd"):
        d[k][:] = d[k][:, :1]
    dY = rnd(141, N, H * dh)
    g = orc.backward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], dY, 0.0)
    assert np.abs(g["d_route"]).max() < 1e-13 * np.abs(g["dW_down"]).max()


def test_silu_derivative_forms_agree():
    """sigma(M) + M sigma(M)(1-sigma(M))  ==  A + sigma(M)(1-A),  A = SiLU(M)."""
    M = np.linspace(-30, 30, 2001)
    s = expit(M)
    A = M * s
    assert np.max(np.abs((s + M * s * (1 - s)) - (A + s * (1 - A)))) < 1e-14


def test_outputs_overwritten_and_partial_requests():
    N, H, dh, E, de = 4, 2, 4, 2, 3
    d = make(150, N, H, dh, E, de)
    dY = rnd(151, N, H * dh)
    full = orc.backward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], dY, 1e-6)
    only_x = orc.backward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], dY, 1e-6,
                          want_weights=False)
    assert np.array_equal(full["dX"], only_x["dX"])
    assert only_x["dW_gate"] is None


# ------------------------------------------------- module: projections around the path
def make_module(seed, N, H, dh, E, de):
    d = make(seed, N, H, dh, E, de)
    dm = H * dh
    d["Win"] = rnd(seed + 5, dm, dm, scale=1.0 / math.sqrt(dm))
    d["Wout"] = rnd(seed + 6, dm, dm, scale=1.0 / math.sqrt(dm))
    return d


@pytest.mark.parametrize("shape", [(3, 2, 3, 2, 4), (2, 1, 4, 3, 2)])
def test_module_forward_bruteforce(shape):
    """Q = X W_in and O = S W_out written as element loops around the element-loop forward:
    a transposed projection or a projection applied on the wrong side fails here (the
    matrices are not symmetric)."""
    N, H, dh, E, de = shape
    d = make_module(300, *shape)
    dm = H * dh
    X, Win, Wout = d["X"].tolist(), d["Win"].tolist(), d["Wout"].tolist()
    Q = [[sum(X[l][i] * Win[i][j] for i in range(dm)) for j in range(dm)] for l in range(N)]
    S = brute_forward(Q, d["Wg"].tolist(), d["Wu"].tolist(), d["Wd"].tolist(), d["Wr"].tolist(), 1e-6)
    O = [[sum(S[l][i] * Wout[i][j] for i in range(dm)) for j in range(dm)] for l in range(N)]
    got = orc.module_forward(d["X"], d["Win"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], d["Wout"], 1e-6)
    assert relerr(got, np.array(O)) < 1e-12


def test_module_with_identity_projections_is_the_path():
    d = make_module(310, 5, 2, 4, 3, 6)
    I = np.eye(8)
    O, Q, S = orc.module_forward(d["X"], I, d["Wg"], d["Wu"], d["Wd"], d["Wr"], I, 1e-6,
                                 return_saved=True)
    Y = orc.forward(d["X"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], 1e-6)
    assert np.array_equal(Q, d["X"]) and np.array_equal(O, S) and relerr(O, Y) == 0.0


@pytest.mark.parametrize("shape", [(3, 2, 4, 3, 5), (4, 1, 6, 2, 3)])
def test_module_backward_matches_finite_differences(shape):
    d = make_module(320, *shape)
    G = rnd(321, shape[0], shape[1] * shape[2])
    eps = 1e-3
    args = lambda: (d["X"], d["Win"], d["Wg"], d["Wu"], d["Wd"], d["Wr"], d["Wout"])
    loss = lambda: float((orc.module_forward(*args(), eps) * G).sum())
    g = orc.module_backward(*args(), G, eps)
    for key, name in (("X", "dX"), ("Win", "dW_in"), ("Wout", "dW_out"), ("Wg", "dW_gate"),
                      ("Wu", "dW_up"), ("Wd", "dW_down"), ("Wr", "d_route")):
        fd = _fd(loss, d[key])
        assert relerr(g[name], fd) < 1e-6, name
