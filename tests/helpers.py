"""Shared plumbing of the GPU parity tests: moving the seeded inputs to the
device in their storage dtype, widening them for the oracle, error norms."""
import numpy as np

from paper_2512_06989_amd import inputs

TOL = {"f32": 1e-5, "bf16": 5e-3}   # relative Frobenius error bounds of the parity bar


def relerr(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def to_device(a, dtype, device="cuda"):
    """float32 numpy array (already rounded to `dtype`) -> torch tensor on the device."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)   # exact: the values are bf16-representable
    return t.to(device)


def to_host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def device_inputs(d, dtype, route_weights=False):
    out = {k: to_device(v, dtype) for k, v in d.items() if k != "R"}
    if "R" in d:
        out["R"] = to_device(d["R"], "f32")
    return out


def small_workload(name, N, H, E, de, dtype, dh=128, w_std=0.05, route_scale=4.0,
                   backward=False):
    return inputs.Workload(name, N, H, dh, E, de, dtype, w_std=w_std,
                           route_scale=route_scale, backward=backward)
