"""Thin binding over the C ABI in include/mhffn.h (libmhffn.so, built from csrc/).

Argument marshalling only: every step of the operation runs in the HIP kernels
of the library.  PyTorch is used for device memory and the current stream.
There is no fallback: if the library is missing or a call fails, this raises."""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmhffn.so")

OK = 0
F32, BF16 = 0, 1
ROUTE_PARAMS, ROUTE_WEIGHTS = 0, 1
OP_FORWARD, OP_BACKWARD, OP_UNFUSED_FORWARD, OP_UNFUSED_BACKWARD = 0, 1, 2, 3
OP_MODULE_FORWARD, OP_MODULE_BACKWARD = 4, 5
EXPORTS = ("mhffn_workspace_bytes", "mhffn_forward", "mhffn_backward", "mhffn_backward_phases",
           "mhffn_reference_unfused", "mhffn_module_forward", "mhffn_module_backward",
           "mhffn_status_string", "mhffn_version", "mhffn_init", "mhffn_forward_static")


class Desc(ctypes.Structure):
    """Mirror of `mhffn_desc`."""
    _fields_ = [("n_tokens", ctypes.c_int64), ("n_heads", ctypes.c_int32),
                ("d_head", ctypes.c_int32), ("n_sub", ctypes.c_int32),
                ("d_sub", ctypes.c_int32), ("ld_x", ctypes.c_int64),
                ("ld_y", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("route_mode", ctypes.c_int32), ("eps", ctypes.c_float)]


class MhffnError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: status %d (%s)" % (where, status, status_string(status)))


_lib = None


def load():
    """Load libmhffn.so (building it first only if it was never built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(Desc)
    lib.mhffn_workspace_bytes.argtypes = [dp, ctypes.c_int]
    lib.mhffn_workspace_bytes.restype = sz
    lib.mhffn_forward.argtypes = [dp] + [vp] * 6 + [vp, sz, vp]
    lib.mhffn_forward.restype = ctypes.c_int
    lib.mhffn_forward_static.argtypes = [dp] + [vp] * 6 + [vp]
    lib.mhffn_forward_static.restype = ctypes.c_int
    lib.mhffn_backward.argtypes = [dp] + [vp] * 11 + [vp, sz, vp]
    lib.mhffn_backward.restype = ctypes.c_int
    lib.mhffn_backward_phases.argtypes = [dp] + [vp] * 11 + [vp, sz, vp, ctypes.POINTER(vp),
                                          ctypes.c_int]
    lib.mhffn_backward_phases.restype = ctypes.c_int
    lib.mhffn_reference_unfused.argtypes = [dp] + [vp] * 12 + [vp, sz, vp]
    lib.mhffn_reference_unfused.restype = ctypes.c_int
    lib.mhffn_module_forward.argtypes = [dp] + [vp] * 10 + [vp, sz, vp]
    lib.mhffn_module_forward.restype = ctypes.c_int
    lib.mhffn_module_backward.argtypes = [dp] + [vp] * 17 + [vp, sz, vp]
    lib.mhffn_module_backward.restype = ctypes.c_int
    lib.mhffn_status_string.argtypes = [ctypes.c_int]
    lib.mhffn_status_string.restype = ctypes.c_char_p
    lib.mhffn_version.restype = ctypes.c_char_p
    lib.mhffn_init.argtypes = []
    lib.mhffn_init.restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status):
    return load().mhffn_status_string(int(status)).decode()


def version():
    return load().mhffn_version().decode()


def init():
    """Raise every kernel's LDS limit on the current device (see mhffn_init)."""
    rc = load().mhffn_init()
    if rc != OK:
        raise MhffnError(rc, "mhffn_init")


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _require(cond, msg):
    if not cond:
        raise ValueError(msg)


def _rows(name, t, like, n_tokens=None):
    """Check a row tensor ([N, d_model], unit column stride, dtype and device of `like`);
    returns its row stride in elements (d_model for fewer than two rows)."""
    _require(t.dim() == 2 and t.shape[1] == like.shape[1], "%s must be [N, %d], got %s"
             % (name, like.shape[1], tuple(t.shape)))
    _require(t.shape[0] == (like.shape[0] if n_tokens is None else n_tokens),
             "%s has %d rows, expected %d" % (name, t.shape[0], like.shape[0]))
    _require(t.dtype == like.dtype, "%s has dtype %s, expected %s" % (name, t.dtype, like.dtype))
    _require(t.device == like.device, "%s is on %s, expected %s" % (name, t.device, like.device))
    if t.shape[0] < 2:
        _require(t.shape[0] == 0 or t.stride(1) == 1, "%s rows must be contiguous" % name)
        return t.shape[1]
    _require(t.stride(1) == 1, "%s rows must be contiguous" % name)
    _require(t.stride(0) >= t.shape[1], "%s rows overlap (row stride %d)" % (name, t.stride(0)))
    return t.stride(0)


def _dense(name, t, shape, dtype, device):
    """Check a dense tensor the kernels index without strides (weights, gating, their gradients)."""
    _require(tuple(t.shape) == tuple(shape), "%s must have shape %s, got %s"
             % (name, tuple(shape), tuple(t.shape)))
    _require(t.dtype == dtype, "%s has dtype %s, expected %s" % (name, t.dtype, dtype))
    _require(t.device == device, "%s is on %s, expected %s" % (name, t.device, device))
    _require(t.is_contiguous(), "%s must be contiguous" % name)


def _check_params(X, W_gate, W_up, W_down, route, route_mode):
    _require(W_gate.dim() == 4, "W_gate must be [H, E, d_e, d_h]")
    H, E, d_e, d_h = W_gate.shape
    _require(X.dim() == 2 and X.shape[1] == H * d_h,
             "X must be [N, H*d_h] = [N, %d], got %s" % (H * d_h, tuple(X.shape)))
    for name, w in (("W_gate", W_gate), ("W_up", W_up), ("W_down", W_down)):
        _dense(name, w, (H, E, d_e, d_h), X.dtype, X.device)
    if int(route_mode) == ROUTE_PARAMS:
        _dense("route (W_r)", route, (H, d_h, E), X.dtype, X.device)
    else:
        _dense("route (R)", route, (X.shape[0], H, E), torch.float32, X.device)


def make_desc(X, W_gate, route_mode, eps, Y=None):
    """Descriptor for X (row stride ld_x) and, where given, the Y-side row tensor (Y, dY, O
    or dO: row stride ld_y; dense otherwise)."""
    H, E, d_e, d_h = W_gate.shape
    if X.dim() != 2 or X.shape[1] != H * d_h:
        raise ValueError("X must be [N, H*d_h] = [N, %d], got %s" % (H * d_h, tuple(X.shape)))
    ld_x = _rows("X", X, X)
    ld_y = H * d_h if Y is None else _rows("the output-side row tensor", Y, X)
    return Desc(X.shape[0], H, d_h, E, d_e, ld_x, ld_y, _dtype_code(X), int(route_mode), float(eps))


def _empty_rows_like(X):
    """Uninitialised [N, d_model] tensor with X's row stride (the kernels index dX with ld_x)."""
    if X.shape[0] < 2 or X.is_contiguous():
        return torch.empty_like(X)
    return torch.empty_strided(tuple(X.shape), tuple(X.stride()), dtype=X.dtype, device=X.device)


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def workspace_bytes(desc, op):
    return int(load().mhffn_workspace_bytes(ctypes.byref(desc), int(op)))


def _workspace(desc, op, device, workspace):
    need = workspace_bytes(desc, op)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    have = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return workspace, have


def forward(X, W_gate, W_up, W_down, route, eps=1e-6, route_mode=ROUTE_PARAMS, out=None,
            stream=None, workspace=None):
    """Fused forward.  Returns Y [N, H*d_h] (dtype of X).  Scratch is needed only
    for small token counts (see mhffn_workspace_bytes); allocated here if not given."""
    _check_params(X, W_gate, W_up, W_down, route, route_mode)
    Y = torch.empty(X.shape, dtype=X.dtype, device=X.device) if out is None else out
    d = make_desc(X, W_gate, route_mode, eps, Y)
    workspace, have = _workspace(d, OP_FORWARD, X.device, workspace)
    rc = load().mhffn_forward(ctypes.byref(d), _p(X), _p(W_gate), _p(W_up), _p(W_down),
                              _p(route), _p(Y), _p(workspace), have, _stream(stream))
    if rc != OK:
        raise MhffnError(rc, "mhffn_forward")
    return Y


def forward_static(X, W_gate, W_up, W_down, route, out, eps=1e-6, route_mode=ROUTE_PARAMS,
                   stream=None):
    """mhffn_forward_static: the fused forward into the caller's `out`, with the scratch in the
    library's static device buffer.  Nothing is allocated here either."""
    _check_params(X, W_gate, W_up, W_down, route, route_mode)
    d = make_desc(X, W_gate, route_mode, eps, out)
    rc = load().mhffn_forward_static(ctypes.byref(d), _p(X), _p(W_gate), _p(W_up), _p(W_down),
                                     _p(route), _p(out), _stream(stream))
    if rc != OK:
        raise MhffnError(rc, "mhffn_forward_static")
    return out


def _grad_outputs(X, W_gate, W_up, W_down, route, want, out, ld_x):
    """The gradient tensors of a backward call: those the caller passed, checked against what
    the kernels assume (dX: X's row stride; the rest dense, shaped like their parameter), and
    fresh ones for the rest of `want`."""
    out = dict(out or {})
    like = {"dW_gate": W_gate, "dW_up": W_up, "dW_down": W_down, "d_route": route}
    for k in want:
        if k not in out:
            out[k] = _empty_rows_like(X) if k == "dX" else torch.empty_like(like[k])
    if out.get("dX") is not None:
        _require(_rows("dX", out["dX"], X) == ld_x or X.shape[0] < 2,
                 "dX must have X's row stride (%d), got %d" % (ld_x, out["dX"].stride(0)))
    for k, ref in like.items():
        if out.get(k) is not None:
            _dense(k, out[k], ref.shape, ref.dtype, ref.device)
    return out


def backward(X, W_gate, W_up, W_down, route, dY, eps=1e-6, route_mode=ROUTE_PARAMS,
             want=("dX", "dW_gate", "dW_up", "dW_down", "d_route"), workspace=None, out=None,
             stream=None, phase_events=None):
    """Fused recompute-based backward.  Returns a dict of the requested gradients.
    `phase_events`: optional list of raw hipEvent_t handles (ints) recorded between
    the phases of the backward (see mhffn_backward_phases)."""
    _check_params(X, W_gate, W_up, W_down, route, route_mode)
    d = make_desc(X, W_gate, route_mode, eps, dY)
    out = _grad_outputs(X, W_gate, W_up, W_down, route, want, out, d.ld_x)
    workspace, have = _workspace(d, OP_BACKWARD, X.device, workspace)
    args = (ctypes.byref(d), _p(X), _p(W_gate), _p(W_up), _p(W_down), _p(route), _p(dY),
            _p(out.get("dX")), _p(out.get("dW_gate")), _p(out.get("dW_up")),
            _p(out.get("dW_down")), _p(out.get("d_route")), _p(workspace), have, _stream(stream))
    if phase_events:
        ev = (ctypes.c_void_p * len(phase_events))(*phase_events)
        rc = load().mhffn_backward_phases(*args, ev, len(phase_events))
    else:
        rc = load().mhffn_backward(*args)
    if rc != OK:
        raise MhffnError(rc, "mhffn_backward")
    return out


def reference_unfused(X, W_gate, W_up, W_down, route, eps=1e-6, route_mode=ROUTE_PARAMS,
                      dY=None, want=("dX", "dW_gate", "dW_up", "dW_down", "d_route"),
                      workspace=None, out=None, stream=None):
    """Unfused GPU baseline (materialises the intermediates in `workspace`).
    Returns Y, or (Y, grads) when dY is given."""
    _check_params(X, W_gate, W_up, W_down, route, route_mode)
    out = dict(out or {})
    Y = out.get("Y")
    if Y is None:
        # Y and dY share the descriptor's ld_y: a fresh Y takes dY's row stride
        Y = _empty_rows_like(dY) if dY is not None else torch.empty(X.shape, dtype=X.dtype,
                                                                    device=X.device)
    d = make_desc(X, W_gate, route_mode, eps, Y)
    if dY is not None:
        _require(_rows("dY", dY, X) == d.ld_y or X.shape[0] < 2,
                 "Y and dY must have the same row stride (%d and %d)" % (d.ld_y, dY.stride(0)))
        grads = _grad_outputs(X, W_gate, W_up, W_down, route, want,
                              {k: v for k, v in out.items() if k != "Y"}, d.ld_x)
        out.update(grads)
    op = OP_UNFUSED_FORWARD if dY is None else OP_UNFUSED_BACKWARD
    workspace, have = _workspace(d, op, X.device, workspace)
    rc = load().mhffn_reference_unfused(
        ctypes.byref(d), _p(X), _p(W_gate), _p(W_up), _p(W_down), _p(route), _p(Y), _p(dY),
        _p(out.get("dX")), _p(out.get("dW_gate")), _p(out.get("dW_up")), _p(out.get("dW_down")),
        _p(out.get("d_route")), _p(workspace), have, _stream(stream))
    if rc != OK:
        raise MhffnError(rc, "mhffn_reference_unfused")
    if dY is None:
        return Y
    return Y, {k: out[k] for k in want}


MODULE_GRADS = ("dX", "dW_in", "dW_gate", "dW_up", "dW_down", "dW_r", "dW_out")


def module_forward(X, W_in, W_gate, W_up, W_down, W_r, W_out, eps=1e-6, out=None, stream=None,
                   workspace=None):
    """The whole module: O = fused(X W_in) W_out.  Returns (O, Q, S); Q and S are the two
    d_model-wide activations that module_backward needs."""
    _check_params(X, W_gate, W_up, W_down, W_r, ROUTE_PARAMS)
    out = dict(out or {})
    N, dm = X.shape
    for k in ("O", "Q", "S"):
        if k not in out:
            out[k] = torch.empty((N, dm), dtype=X.dtype, device=X.device)
    for k, w in (("W_in", W_in), ("W_out", W_out)):
        _dense(k, w, (dm, dm), X.dtype, X.device)
    for k in ("Q", "S"):
        _dense(k, out[k], (N, dm), X.dtype, X.device)
    d = make_desc(X, W_gate, ROUTE_PARAMS, eps, out["O"])
    workspace, have = _workspace(d, OP_MODULE_FORWARD, X.device, workspace)
    rc = load().mhffn_module_forward(ctypes.byref(d), _p(X), _p(W_in), _p(W_gate), _p(W_up),
                                     _p(W_down), _p(W_r), _p(W_out), _p(out["O"]), _p(out["Q"]),
                                     _p(out["S"]), _p(workspace), have, _stream(stream))
    if rc != OK:
        raise MhffnError(rc, "mhffn_module_forward")
    return out["O"], out["Q"], out["S"]


def module_backward(X, W_in, W_gate, W_up, W_down, W_r, W_out, Q, S, dO, eps=1e-6,
                    want=MODULE_GRADS, out=None, stream=None, workspace=None):
    """Backward of module_forward from the saved Q and S.  Returns a dict of gradients."""
    _check_params(X, W_gate, W_up, W_down, W_r, ROUTE_PARAMS)
    out = dict(out or {})
    N, dm = X.shape
    like = {"dW_in": W_in, "dW_gate": W_gate, "dW_up": W_up, "dW_down": W_down,
            "dW_r": W_r, "dW_out": W_out}
    for k, w in (("W_in", W_in), ("W_out", W_out)):
        _dense(k, w, (dm, dm), X.dtype, X.device)
    for k, t in (("Q", Q), ("S", S)):
        _dense(k, t, (N, dm), X.dtype, X.device)
    d = make_desc(X, W_gate, ROUTE_PARAMS, eps, dO)
    for k in want:
        if k not in out:
            out[k] = _empty_rows_like(X) if k == "dX" else torch.empty_like(like[k])
    if out.get("dX") is not None:
        _require(_rows("dX", out["dX"], X) == d.ld_x or N < 2,
                 "dX must have X's row stride (%d), got %d" % (d.ld_x, out["dX"].stride(0)))
    for k, ref in like.items():
        if out.get(k) is not None:
            _dense(k, out[k], ref.shape, ref.dtype, ref.device)
    workspace, have = _workspace(d, OP_MODULE_BACKWARD, X.device, workspace)
    rc = load().mhffn_module_backward(
        ctypes.byref(d), _p(X), _p(W_in), _p(W_gate), _p(W_up), _p(W_down), _p(W_r), _p(W_out),
        _p(Q), _p(S), _p(dO), *[_p(out.get(k)) for k in MODULE_GRADS], _p(workspace), have,
        _stream(stream))
    if rc != OK:
        raise MhffnError(rc, "mhffn_module_backward")
    return {k: out[k] for k in want}
