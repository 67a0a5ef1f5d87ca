"""Seeded synthetic inputs for the gated Multi-Head FFN, shared by the tests,
the bench and the smoke check.  Holds none of the method's arithmetic: it only
draws random tensors of the workload shapes and rounds them to the storage
dtype, so that the GPU library and the CPU oracle consume identical values.

Shapes and distributions follow the paper's model table (d_model, H, d_h = 128,
`initializer_range` 0.02) with the sub-network width fixed at 128:
X ~ N(0,1) stands in for normalised hidden states, every weight ~ N(0, std).
All tensors come from a Philox stream keyed by (seed, tensor id), so any tensor
can be regenerated alone and the result is bit-reproducible across machines."""
from dataclasses import dataclass, replace
import math

import numpy as np

STREAM_X, STREAM_WG, STREAM_WU, STREAM_WD, STREAM_WR, STREAM_DY, STREAM_R = range(7)
STREAM_WIN, STREAM_WOUT = 7, 8


@dataclass(frozen=True)
class Workload:
    name: str
    n_tokens: int
    n_heads: int
    d_head: int
    n_sub: int
    d_sub: int
    dtype: str            # "f32" or "bf16"
    w_std: float = 0.02
    route_scale: float = 1.0
    backward: bool = False
    eps: float = 1e-6

    @property
    def d_model(self):
        return self.n_heads * self.d_head

    @property
    def d_ff(self):
        return self.n_sub * self.d_sub

    def unit_flops(self):
        """Flops of one full-size contraction over all heads: 2*N*d_model*d_ff."""
        return 2.0 * self.n_tokens * self.d_model * self.d_ff

    def with_tokens(self, n):
        return replace(self, n_tokens=int(n), name="%s@N=%d" % (self.name.split("@")[0], n))


WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", 256, 6, 128, 4, 128, "f32"),
    "128m_fwd": Workload("128m_fwd", 16384, 6, 128, 16, 128, "bf16"),
    "370m_fwdbwd": Workload("370m_fwdbwd", 16384, 8, 128, 22, 128, "bf16", backward=True),
    "1p3b_fwdbwd": Workload("1p3b_fwdbwd", 16384, 16, 128, 44, 128, "bf16",
                            w_std=0.02 / math.sqrt(24.0), backward=True),
    "1p3b_sweep": Workload("1p3b_sweep", 1024, 16, 128, 44, 128, "bf16", route_scale=8.0),
    # The paper's own shapes (model table: E sub-networks of width intermediate/E; sub-network
    # width 8/3 d_h rounded up to a multiple of 64 = 384 for d_h = 128) and the shape of its
    # efficiency benchmark (batch 8 x sequence L, H = 16, E = 22, d_e = 384; tokens = 8 L).
    "paper_128m": Workload("paper_128m", 16384, 6, 128, 8, 256, "bf16", backward=True),
    "paper_370m": Workload("paper_370m", 16384, 8, 128, 7, 384, "bf16", backward=True),
    "paper_1p3b": Workload("paper_1p3b", 16384, 16, 128, 15, 384, "bf16", backward=True),
    "paper_bench": Workload("paper_bench", 8 * 1920, 16, 128, 22, 384, "bf16", backward=True),
    # Head-width ablation of the paper (d_h = 64 and 256; sub-network width 8/3 d_h rounded up to
    # a multiple of 64 = 192 and 704), on the 370M model's d_model = 1024 and intermediate size
    # of about 2688, and on the 1.3B model's d_model = 2048 / about 5632.
    "paper_370m_dh64": Workload("paper_370m_dh64", 16384, 16, 64, 14, 192, "bf16", backward=True),
    "paper_370m_dh256": Workload("paper_370m_dh256", 16384, 4, 256, 4, 704, "bf16", backward=True),
    "paper_1p3b_dh64": Workload("paper_1p3b_dh64", 16384, 32, 64, 29, 192, "bf16", backward=True),
    "paper_1p3b_dh256": Workload("paper_1p3b_dh256", 16384, 8, 256, 8, 704, "bf16", backward=True),
}
SWEEP_TOKENS = (64, 1024, 32768)
PAPER_BENCH_SEQ_LENS = (192, 384, 768, 1536, 1920, 2880, 4032, 8064, 16128)   # batch 8 each


def _normal(seed, stream, shape, std):
    g = np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def f32_to_bf16_bits(a):
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(a, dtype):
    """Value of `a` after one rounding to the storage dtype, as float32."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    raise ValueError(dtype)


def make_inputs(w: Workload, seed: int = 0, with_dy=None, route_weights: bool = False):
    """Dict of float32 arrays already rounded to w.dtype:
    X [N, d_model], W_gate/W_up/W_down [H, E, d_e, d_h], W_r [H, d_h, E],
    optionally dY [N, d_model] ~ N(0,1) and R [N, H, E] (float32, uniform(0,1)
    rows scaled to sum to one; only for the weights-as-input mode)."""
    if with_dy is None:
        with_dy = w.backward
    wshape = (w.n_heads, w.n_sub, w.d_sub, w.d_head)
    out = {
        "X": round_to(_normal(seed, STREAM_X, (w.n_tokens, w.d_model), 1.0), w.dtype),
        "W_gate": round_to(_normal(seed, STREAM_WG, wshape, w.w_std), w.dtype),
        "W_up": round_to(_normal(seed, STREAM_WU, wshape, w.w_std), w.dtype),
        "W_down": round_to(_normal(seed, STREAM_WD, wshape, w.w_std), w.dtype),
        "W_r": round_to(_normal(seed, STREAM_WR, (w.n_heads, w.d_head, w.n_sub),
                                w.w_std) * np.float32(w.route_scale), w.dtype),
    }
    if with_dy:
        out["dY"] = round_to(_normal(seed, STREAM_DY, (w.n_tokens, w.d_model), 1.0), w.dtype)
    if route_weights:
        g = np.random.Generator(np.random.Philox(key=[int(seed), STREAM_R]))
        r = g.random(size=(w.n_tokens, w.n_heads, w.n_sub), dtype=np.float32) + np.float32(0.05)
        out["R"] = (r / r.sum(axis=-1, keepdims=True)).astype(np.float32)
    return out


def make_module_inputs(w: Workload, seed: int = 0, with_dy=None):
    """make_inputs plus the module's projections W_in, W_out [d_model, d_model] ~ N(0, 1/d_model)
    (so that Q = X W_in has the unit scale the path's own inputs have), rounded to w.dtype.
    X is then the module's input and dY the gradient of its output O."""
    out = make_inputs(w, seed=seed, with_dy=with_dy)
    std = 1.0 / math.sqrt(w.d_model)
    out["W_in"] = round_to(_normal(seed, STREAM_WIN, (w.d_model, w.d_model), std), w.dtype)
    out["W_out"] = round_to(_normal(seed, STREAM_WOUT, (w.d_model, w.d_model), std), w.dtype)
    return out
