"""ctypes binding of the fp64 CPU oracle (oracle/mhffn_oracle.c).

Test infrastructure only.  Takes and returns numpy float64 arrays; inputs in a
narrower dtype must be widened by the caller *after* rounding, so the oracle
sees exactly the values the GPU sees."""
import ctypes
import os

import numpy as np

from . import build as _build

ROUTE_PARAMS = 0   # route = W_r [H][d_h][E]; weights from eq:routing
ROUTE_WEIGHTS = 1  # route = R [N][H][E]; used as given


class _Desc(ctypes.Structure):
    _fields_ = [("n_tokens", ctypes.c_int64), ("n_heads", ctypes.c_int32),
                ("d_head", ctypes.c_int32), ("n_sub", ctypes.c_int32),
                ("d_sub", ctypes.c_int32), ("ld_x", ctypes.c_int64),
                ("ld_y", ctypes.c_int64), ("route_mode", ctypes.c_int32),
                ("eps", ctypes.c_double)]


_lib = None


def load():
    global _lib
    if _lib is None:
        # The mutation test points the pins at a deliberately broken build of this same
        # source.  That needs both variables, and the second one names the only test file
        # that may run against such a build, so no other process can be redirected.
        path = None
        import sys
        if (os.environ.get("MHFFN_ORACLE_MUTATION_HARNESS") == "tests/test_oracle_pins.py"
                and any(a.endswith("test_oracle_pins.py") for a in sys.argv)):
            path = os.environ.get("MHFFN_ORACLE_LIB")
        path = path or _build.build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.c_void_p
        lib.mhffn_oracle_forward_f64.argtypes = [ctypes.POINTER(_Desc)] + [dp] * 7
        lib.mhffn_oracle_forward_f64.restype = ctypes.c_int
        lib.mhffn_oracle_subnet_outputs_f64.argtypes = [ctypes.POINTER(_Desc)] + [dp] * 5
        lib.mhffn_oracle_subnet_outputs_f64.restype = ctypes.c_int
        lib.mhffn_oracle_backward_f64.argtypes = [ctypes.POINTER(_Desc)] + [dp] * 11
        lib.mhffn_oracle_backward_f64.restype = ctypes.c_int
        lib.mhffn_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(load().mhffn_oracle_threads())


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _shapes(X, W_gate, route, route_mode):
    N, d_model = X.shape
    H, E, d_e, d_h = W_gate.shape
    if H * d_h != d_model:
        raise ValueError("X has %d columns, weights say H*d_h = %d" % (d_model, H * d_h))
    want = (H, d_h, E) if route_mode == ROUTE_PARAMS else (N, H, E)
    if tuple(route.shape) != want:
        raise ValueError("route has shape %s, expected %s" % (route.shape, want))
    return N, H, E, d_e, d_h


def forward(X, W_gate, W_up, W_down, route, eps, route_mode=ROUTE_PARAMS,
            return_weights=False):
    """Y [N, H*d_h] (and R [N, H, E] if return_weights)."""
    X, W_gate, W_up, W_down, route = map(_c, (X, W_gate, W_up, W_down, route))
    N, H, E, d_e, d_h = _shapes(X, W_gate, route, route_mode)
    assert W_up.shape == W_gate.shape == W_down.shape
    d = _Desc(N, H, d_h, E, d_e, 0, 0, route_mode, float(eps))
    Y = np.empty((N, H * d_h), dtype=np.float64)
    R = np.empty((N, H, E), dtype=np.float64) if return_weights else None
    rc = load().mhffn_oracle_forward_f64(ctypes.byref(d), _p(X), _p(W_gate), _p(W_up),
                                         _p(W_down), _p(route), _p(Y), _p(R))
    if rc:
        raise RuntimeError("oracle forward failed: %d" % rc)
    return (Y, R) if return_weights else Y


def subnet_outputs(X, W_gate, W_up, W_down):
    """Un-weighted sub-network outputs y_e: [N, H, E, d_h]."""
    X, W_gate, W_up, W_down = map(_c, (X, W_gate, W_up, W_down))
    N, d_model = X.shape
    H, E, d_e, d_h = W_gate.shape
    assert H * d_h == d_model
    d = _Desc(N, H, d_h, E, d_e, 0, 0, 0, 0.0)
    Ysub = np.empty((N, H, E, d_h), dtype=np.float64)
    rc = load().mhffn_oracle_subnet_outputs_f64(ctypes.byref(d), _p(X), _p(W_gate),
                                                _p(W_up), _p(W_down), _p(Ysub))
    if rc:
        raise RuntimeError("oracle subnet_outputs failed: %d" % rc)
    return Ysub


def backward(X, W_gate, W_up, W_down, route, dY, eps, route_mode=ROUTE_PARAMS,
             want_weights=True):
    """Returns dict with dX, d_route and (if want_weights) dW_gate, dW_up, dW_down."""
    X, W_gate, W_up, W_down, route, dY = map(_c, (X, W_gate, W_up, W_down, route, dY))
    N, H, E, d_e, d_h = _shapes(X, W_gate, route, route_mode)
    assert dY.shape == X.shape
    d = _Desc(N, H, d_h, E, d_e, 0, 0, route_mode, float(eps))
    dX = np.empty_like(X)
    dWg = np.empty_like(W_gate) if want_weights else None
    dWu = np.empty_like(W_gate) if want_weights else None
    dWd = np.empty_like(W_gate) if want_weights else None
    d_route = np.empty_like(route) if (want_weights or route_mode == ROUTE_WEIGHTS) else None
    rc = load().mhffn_oracle_backward_f64(ctypes.byref(d), _p(X), _p(W_gate), _p(W_up),
                                          _p(W_down), _p(route), _p(dY), _p(dX), _p(dWg),
                                          _p(dWu), _p(dWd), _p(d_route))
    if rc:
        raise RuntimeError("oracle backward failed: %d" % rc)
    return {"dX": dX, "dW_gate": dWg, "dW_up": dWu, "dW_down": dWd, "d_route": d_route}


# ---- the whole module: input and output projections around the path -------------------
# (Methodology, definition of Q = split_H(X W_in) and O = concat_H(S) W_out; no bias, no
# normalisation.)  W_in and W_out are [d_model][d_model], applied from the right.  The two
# projections are library matrix products in fp64; everything between them is the oracle above.

def module_forward(X, W_in, W_gate, W_up, W_down, W_r, W_out, eps, return_saved=False):
    """O [N, d_model] (and the saved Q, S if return_saved)."""
    X, W_in, W_out = (np.asarray(a, dtype=np.float64) for a in (X, W_in, W_out))
    Q = X @ W_in
    S = forward(Q, W_gate, W_up, W_down, W_r, eps)
    O = S @ W_out
    return (O, Q, S) if return_saved else O


def module_backward(X, W_in, W_gate, W_up, W_down, W_r, W_out, dO, eps):
    """Gradients of sum(O * dO) with respect to X and every parameter."""
    X, W_in, W_out, dO = (np.asarray(a, dtype=np.float64) for a in (X, W_in, W_out, dO))
    Q = X @ W_in
    S = forward(Q, W_gate, W_up, W_down, W_r, eps)
    dS = dO @ W_out.T
    g = backward(Q, W_gate, W_up, W_down, W_r, dS, eps)
    return {"dX": g["dX"] @ W_in.T, "dW_in": X.T @ g["dX"], "dW_out": S.T @ dO,
            "dW_gate": g["dW_gate"], "dW_up": g["dW_up"], "dW_down": g["dW_down"],
            "d_route": g["d_route"]}
