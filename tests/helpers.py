"""Shared plumbing of the GPU parity tests: moving the seeded inputs to the
device in their storage dtype, widening them for the oracle, error norms."""
import numpy as np

from paper_2512_06989_amd import inputs
from paper_2512_06989_amd.device import device_inputs, to_device, to_host  # noqa: F401

TOL = {"f32": 1e-5, "bf16": 5e-3}   # relative Frobenius error bounds of the parity bar


# Per-row companion of the Frobenius bound: no single row (a token's head slice of Y or dX, a
# neuron's row of a weight gradient, a sub-network's column of dW_r) may be off by more than
# ROW_FACTOR x the tolerance relative to its own norm.  The rounding errors of a row of n
# elements are independent, so its relative error scatters around the whole-tensor figure by
# about 1/sqrt(2n), and the smallest row norm among 10^5..10^6 rows of 64..256 Gaussian
# elements is about 0.6 of the typical one: the worst row is expected below 2x the whole-tensor
# error (measured at the full sizes: whole tensor 2.35e-3, worst row 2.6e-3..3.0e-3), while one
# wrong row, or a tile edge that is 10 % off, is 10x..100x the bound.  Rows whose reference norm is below a tenth of the root-mean-square row norm are
# measured against that floor (a row of exact zeros has no relative error).
ROW_FACTOR = 2.0
ROW_FLOOR = 0.1


def row_relerr(got, want, row_len):
    """max over rows of ||got_row - want_row|| / (||want_row|| + ROW_FLOOR * rms row norm);
    rows = consecutive runs of `row_len` elements of the last axis."""
    g = np.asarray(got, dtype=np.float64).reshape(-1, row_len)
    w = np.asarray(want, dtype=np.float64).reshape(-1, row_len)
    num = np.linalg.norm(g - w, axis=1)
    den = np.linalg.norm(w, axis=1)
    floor = ROW_FLOOR * np.sqrt(np.mean(den * den)) if den.size else 0.0
    return float(np.max(num / np.maximum(den + floor, 1e-300))) if den.size else 0.0


def dwr_columns(a):
    """dW_r [H, d_h, E] -> one row per (head, sub-network): [H*E, d_h]."""
    a = np.asarray(a, dtype=np.float64)
    return np.ascontiguousarray(np.swapaxes(a, -1, -2))


def check_parity(got, want, tol, d_head, what="", route_weights=False, skip=()):
    """Frobenius and per-row bounds for a dict of results (Y, dX: rows of d_head per token and
    head; dW_*: rows of d_head per neuron; d_route: columns of dW_r, or rows of dR per token
    and head).  Returns the measured figures."""
    out = {}
    for k in got:
        if k in skip or want.get(k) is None:
            continue
        g, w = np.asarray(got[k], dtype=np.float64), np.asarray(want[k], dtype=np.float64)
        assert g.shape == w.shape, (k, g.shape, w.shape)
        assert np.all(np.isfinite(g)), "%s %s: non-finite values" % (what, k)
        if k == "d_route":
            if route_weights:
                rows_g, rows_w, n = g, w, g.shape[-1]
            else:
                rows_g, rows_w, n = dwr_columns(g), dwr_columns(w), g.shape[-2]
        else:
            rows_g, rows_w, n = g, w, d_head
        fro, row = relerr(g, w), row_relerr(rows_g, rows_w, n)
        out[k] = (fro, row)
        assert fro <= tol, "%s %s: Frobenius error %.3e > %.1e" % (what, k, fro, tol)
        assert row <= ROW_FACTOR * tol, "%s %s: worst row %.3e > %.1e" % (what, k, row, ROW_FACTOR * tol)
    return out


def relerr(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def small_workload(name, N, H, E, de, dtype, dh=128, w_std=0.05, route_scale=4.0,
                   backward=False):
    return inputs.Workload(name, N, H, dh, E, de, dtype, w_std=w_std,
                           route_scale=route_scale, backward=backward)
