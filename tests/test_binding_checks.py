"""Argument checks of the Python binding (CPU only: every case must raise before the C ABI
is reached, so no device memory is touched)."""
import pytest
import torch

from paper_2512_06989_amd import mhffn

H, E, DE, DH, N = 2, 3, 64, 128, 10
DM = H * DH


def _args(dtype=torch.bfloat16):
    X = torch.zeros(N, DM, dtype=dtype)
    W = [torch.zeros(H, E, DE, DH, dtype=dtype) for _ in range(3)]
    Wr = torch.zeros(H, DH, E, dtype=dtype)
    return X, W, Wr


def test_descriptor_takes_each_stride_from_its_own_tensor():
    X, W, _ = _args()
    Xp = torch.zeros(N, DM + 64, dtype=torch.bfloat16)[:, :DM]
    Yp = torch.zeros(N, DM + 128, dtype=torch.bfloat16)[:, :DM]
    d = mhffn.make_desc(Xp, W[0], mhffn.ROUTE_PARAMS, 1e-6, Yp)
    assert (d.ld_x, d.ld_y) == (DM + 64, DM + 128)
    d = mhffn.make_desc(Xp, W[0], mhffn.ROUTE_PARAMS, 1e-6)
    assert (d.ld_x, d.ld_y) == (DM + 64, DM)
    # a gradient of X allocated by the binding has X's row stride, not a dense one
    assert mhffn._empty_rows_like(Xp).stride() == Xp.stride()


@pytest.mark.parametrize("what", ["weight_dtype", "weight_shape", "weight_strided", "route_dtype",
                                  "route_shape", "weights_mode_not_fp32", "x_columns"])
def test_forward_rejects_mismatched_arguments(what):
    X, W, Wr = _args()
    route, mode = Wr, mhffn.ROUTE_PARAMS
    if what == "weight_dtype":
        W[1] = W[1].float()
    elif what == "weight_shape":
        W[2] = torch.zeros(H, E, DE + 32, DH, dtype=torch.bfloat16)
    elif what == "weight_strided":
        W[0] = torch.zeros(H, E, DE, 2 * DH, dtype=torch.bfloat16)[..., :DH]
    elif what == "route_dtype":
        route = Wr.float()
    elif what == "route_shape":
        route = torch.zeros(H, E, DH, dtype=torch.bfloat16)
    elif what == "weights_mode_not_fp32":
        route, mode = torch.zeros(N, H, E, dtype=torch.bfloat16), mhffn.ROUTE_WEIGHTS
    elif what == "x_columns":
        X = torch.zeros(N, DM + 8, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        mhffn.forward(X, *W, route, 1e-6, mode)


@pytest.mark.parametrize("what", ["dy_dtype", "dy_rows", "dx_stride", "dw_strided", "dw_dtype"])
def test_backward_rejects_mismatched_arguments(what):
    X, W, Wr = _args()
    dY = torch.zeros(N, DM, dtype=torch.bfloat16)
    out = {}
    if what == "dy_dtype":
        dY = dY.float()
    elif what == "dy_rows":
        dY = torch.zeros(N + 1, DM, dtype=torch.bfloat16)
    elif what == "dx_stride":
        X = torch.zeros(N, DM + 64, dtype=torch.bfloat16)[:, :DM]
        out["dX"] = torch.zeros(N, DM, dtype=torch.bfloat16)      # dense, X is not
    elif what == "dw_strided":
        out["dW_up"] = torch.zeros(H, E, DE, 2 * DH, dtype=torch.bfloat16)[..., :DH]
    elif what == "dw_dtype":
        out["dW_down"] = torch.zeros(H, E, DE, DH, dtype=torch.float32)
    with pytest.raises(ValueError):
        mhffn.backward(X, *W, Wr, dY, out=out)


def test_unfused_rejects_y_and_dy_of_different_strides():
    X, W, Wr = _args()
    dY = torch.zeros(N, DM + 64, dtype=torch.bfloat16)[:, :DM]
    with pytest.raises(ValueError):
        mhffn.reference_unfused(X, *W, Wr, dY=dY, out={"Y": torch.zeros(N, DM, dtype=torch.bfloat16)})
