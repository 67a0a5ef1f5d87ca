"""Moving the seeded inputs between numpy and the device: storage-dtype tensors on
the GPU from float32 arrays that are already rounded to that dtype, and results back
as float64 arrays.  No arithmetic of the method lives here."""
import numpy as np


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


def device_inputs(d, dtype):
    """Every tensor of an input dict in the storage dtype; the gating weights R, where
    present, stay fp32 (the boundary takes them in fp32 whatever the storage dtype)."""
    out = {k: to_device(v, dtype) for k, v in d.items() if k != "R"}
    if "R" in d:
        out["R"] = to_device(d["R"], "f32")
    return out
