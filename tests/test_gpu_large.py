"""More than 2^31 elements per activation tensor: byte and element offsets of X, Y, dY and dX
pass 32 bits.  The forward and dX are token-wise, so the oracle checks sampled tokens (taken
from both ends and from around the 2^31-element and 4 GiB marks); the weight gradients sum
over all tokens and are checked against the sum of the two halves of the batch run on their
own (a property that holds at any size)."""
import numpy as np
import pytest

from oracle import mhffn_oracle as orc
from paper_2512_06989_amd import mhffn
from tests.helpers import TOL, relerr, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dh", [128, 64, 256])
def test_more_than_2_to_31_activation_elements(dh):
    import torch
    E, de = 2, 64
    H = 256 // dh
    dm = H * dh
    N = (1 << 31) // dm + 4096 + 37          # 8.39 M tokens, ragged
    gen = torch.Generator(device="cuda").manual_seed(7)
    rnd = lambda *shape, std=1.0: (torch.randn(*shape, generator=gen, device="cuda") * std).to(torch.bfloat16)
    X, dY = rnd(N, dm), rnd(N, dm)
    W = [rnd(H, E, de, dh, std=0.05) for _ in range(3)]
    Wr = rnd(H, dh, E, std=0.2)
    Y = mhffn.forward(X, *W, Wr)
    g = mhffn.backward(X, *W, Wr, dY)
    torch.cuda.synchronize()
    edge = (1 << 31) // dm                    # first token past 2^31 elements (= 4 GiB in bf16)
    rows = np.array([0, 1, 255, edge // 2 - 1, edge // 2, edge - 1, edge, edge + 1, edge + 300,
                     N - 257, N - 38, N - 1])
    tr = torch.from_numpy(rows).cuda()
    host = lambda t: to_host(t)
    Wh = [host(w) for w in W]
    ref_y = orc.forward(host(X[tr]), *Wh, host(Wr), 1e-6)
    assert relerr(host(Y[tr]), ref_y) <= TOL["bf16"]
    ref = orc.backward(host(X[tr]), *Wh, host(Wr), host(dY[tr]), 1e-6, want_weights=False)
    assert relerr(host(g["dX"][tr]), ref["dX"]) <= TOL["bf16"]
    assert bool(torch.isfinite(Y[-4096:].float()).all()) and bool(torch.isfinite(g["dX"][-4096:].float()).all())
    del Y
    # weight gradients: whole batch = first half + second half
    half = N // 2
    g1 = mhffn.backward(X[:half], *W, Wr, dY[:half], want=("dW_gate", "dW_up", "dW_down", "d_route"))
    g2 = mhffn.backward(X[half:], *W, Wr, dY[half:], want=("dW_gate", "dW_up", "dW_down", "d_route"))
    torch.cuda.synchronize()
    for k in ("dW_gate", "dW_up", "dW_down", "d_route"):
        whole = g[k].float()
        parts = g1[k].float() + g2[k].float()
        err = float((whole - parts).norm() / parts.norm())
        assert err <= 2 * 2.0 ** -8, (k, err)     # three roundings to bf16 (whole, and each half)


def test_more_than_2_to_31_weight_elements():
    """Each weight tensor has 2.2e9 elements (4.4 GB): the last head starts past 2^31 elements.
    Heads are independent, so the oracle checks that head alone (forward and all gradients)."""
    import torch
    N, H, dh, E, de = 64, 16, 128, 96, 11264
    assert H * E * de * dh > (1 << 31) and (H - 1) * E * de * dh < (1 << 31) < H * E * de * dh
    gen = torch.Generator(device="cuda").manual_seed(11)

    def rnd(*shape, std=1.0):
        t = torch.empty(*shape, dtype=torch.bfloat16, device="cuda")
        flat = t.view(-1)
        step = 1 << 28                       # generate in pieces: no 9 GB fp32 temporary
        for i in range(0, flat.numel(), step):
            n = min(step, flat.numel() - i)
            flat[i:i + n] = (torch.randn(n, generator=gen, device="cuda") * std).to(torch.bfloat16)
        return t

    X, dY = rnd(N, H * dh), rnd(N, H * dh)
    W = [rnd(H, E, de, dh, std=0.003) for _ in range(3)]     # about 1 / sqrt(d_ff / E): outputs of order one
    Wr = rnd(H, dh, E, std=0.2)
    Y = mhffn.forward(X, *W, Wr)
    g = mhffn.backward(X, *W, Wr, dY)
    torch.cuda.synchronize()
    h = H - 1
    cols = slice(h * dh, (h + 1) * dh)
    Xh, dYh = to_host(X[:, cols]), to_host(dY[:, cols])
    Wh = [to_host(w[h:h + 1]) for w in W]
    Wrh = to_host(Wr[h:h + 1])
    assert relerr(to_host(Y[:, cols]), orc.forward(Xh, *Wh, Wrh, 1e-6)) <= TOL["bf16"]
    ref = orc.backward(Xh, *Wh, Wrh, dYh, 1e-6)
    got = {"dX": g["dX"][:, cols], "dW_gate": g["dW_gate"][h:h + 1], "dW_up": g["dW_up"][h:h + 1],
           "dW_down": g["dW_down"][h:h + 1], "d_route": g["d_route"][h:h + 1]}
    errs = {k: relerr(to_host(v), ref[k]) for k, v in got.items()}
    assert all(e <= TOL["bf16"] for e in errs.values()), str(errs)
