"""Shared plumbing of the GPU parity tests: moving the seeded inputs to the
device in their storage dtype, widening them for the oracle, error norms."""
import numpy as np

from paper_2512_06989_amd import inputs
from paper_2512_06989_amd.device import device_inputs, to_device, to_host  # noqa: F401

TOL = {"f32": 1e-5, "bf16": 5e-3}   # relative Frobenius error bounds of the parity bar


def relerr(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def small_workload(name, N, H, E, de, dtype, dh=128, w_std=0.05, route_scale=4.0,
                   backward=False):
    return inputs.Workload(name, N, H, dh, E, de, dtype, w_std=w_std,
                           route_scale=route_scale, backward=backward)
