"""Host-only tests of the C-ABI library: it loads without a GPU, exports every
symbol the header declares, and rejects bad arguments before launching."""
import ctypes
import os
import re

import pytest

from paper_2512_06989_amd import mhffn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mhffn.h")).read()
    declared = set(re.findall(r"\b(mhffn_[a-z_]+)\s*\(", header))
    assert declared == set(mhffn.EXPORTS)
    lib = mhffn.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert mhffn.version().startswith("mhffn-gfx950")


def test_desc_struct_matches_header_field_order():
    header = open(os.path.join(ROOT, "include", "mhffn.h")).read()
    body = header[header.index("typedef struct {"):header.index("} mhffn_desc;")]
    names = re.findall(r"\b(?:int64_t|int32_t|float)\s+(\w+);", body)
    assert names == [f[0] for f in mhffn.Desc._fields_]


def desc(**kw):
    base = dict(n_tokens=64, n_heads=2, d_head=128, n_sub=3, d_sub=128, ld_x=0, ld_y=0,
                dtype=mhffn.BF16, route_mode=mhffn.ROUTE_PARAMS, eps=1e-6)
    base.update(kw)
    return mhffn.Desc(*[base[f[0]] for f in mhffn.Desc._fields_])


FAKE = ctypes.c_void_p(0x10000)   # aligned, never dereferenced: validation fails first


def fwd(d, ptrs=None):
    ptrs = ptrs or [FAKE] * 6
    return mhffn.load().mhffn_forward(ctypes.byref(d), *ptrs, None, 0, None)


@pytest.mark.parametrize("kw,status", [
    (dict(n_tokens=-1), 2), (dict(n_heads=0), 2), (dict(d_sub=0), 2), (dict(ld_x=100), 2),
    (dict(eps=-1.0), 2), (dict(eps=float("nan")), 2), (dict(dtype=7), 3), (dict(route_mode=2), 3),
    (dict(d_head=96), 3), (dict(d_head=512), 3), (dict(d_sub=48), 3), (dict(n_sub=1000), 3),
    (dict(ld_x=260), 4),
    (dict(dtype=mhffn.F32, d_head=130), 3), (dict(dtype=mhffn.F32, d_head=512), 3),
])
def test_forward_rejects_bad_descriptors(kw, status):
    assert fwd(desc(**kw)) == status


def test_bf16_head_widths_64_and_256_pass_validation():
    """The fused bf16 kernels exist for d_h in {64, 128, 256}: these descriptors get as far as
    the workspace check (64 tokens: the intermediate dimension is split)."""
    lib = mhffn.load()
    for dh, de in ((64, 192), (256, 704)):
        d = desc(d_head=dh, d_sub=de)
        assert fwd(d) == 5
        assert lib.mhffn_backward(ctypes.byref(d), *([FAKE] * 11), None, 0, None) == 5
        assert mhffn.workspace_bytes(d, mhffn.OP_BACKWARD) > 0
    # d_h = 256: the backward takes at most 64 sub-networks, the forward 96
    d = desc(d_head=256, d_sub=64, n_sub=96)
    assert fwd(d) == 5
    assert lib.mhffn_backward(ctypes.byref(d), *([FAKE] * 11), FAKE, 1 << 40, None) == 3


def test_forward_rejects_null_and_misaligned_pointers():
    d = desc()
    for i in range(6):
        ptrs = [FAKE] * 6
        ptrs[i] = None
        assert fwd(d, ptrs) == 1
        ptrs[i] = ctypes.c_void_p(0x10004)
        assert fwd(d, ptrs) == 4
    assert mhffn.load().mhffn_forward(None, *([FAKE] * 6), None, 0, None) == 1


def test_empty_input_is_ok_and_launches_nothing():
    assert fwd(desc(n_tokens=0)) == 0


def test_status_strings():
    seen = {mhffn.status_string(i) for i in range(7)}
    assert len(seen) == 7 and mhffn.status_string(99) == "unknown status"


def test_forward_needs_no_workspace_when_token_tiles_fill_the_chip():
    for n_heads, n_sub in ((6, 16), (8, 22), (16, 44)):
        d = desc(n_tokens=16384, n_heads=n_heads, n_sub=n_sub)
        assert mhffn.workspace_bytes(d, mhffn.OP_FORWARD) == 0
    assert mhffn.workspace_bytes(desc(n_tokens=32768, n_heads=16, n_sub=44), mhffn.OP_FORWARD) == 0
    assert mhffn.workspace_bytes(desc(n_heads=0), mhffn.OP_FORWARD) == 0


def test_small_token_counts_split_the_intermediate_dimension():
    """Decode-sized inputs: fp32 partial outputs, a few times the output, never d_ff-sized."""
    for n in (1, 64, 1024):
        d = desc(n_tokens=n, n_heads=16, n_sub=44)
        ws = mhffn.workspace_bytes(d, mhffn.OP_FORWARD)
        out_f32 = n * 16 * 128 * 4
        assert ws > 0 and ws % out_f32 == 0
        assert ws // out_f32 <= 88                       # at most one split per two tiles
        assert ws < n * 16 * 44 * 128 * 2 * 3            # far below the materialised intermediate
    # the fused forward refuses a missing workspace before launching anything
    rc = mhffn.load().mhffn_forward(ctypes.byref(desc(n_tokens=64, n_heads=16, n_sub=44)),
                                    *([FAKE] * 6), None, 0, None)
    assert rc == 5


def test_backward_and_unfused_workspace_sizes():
    d = desc(n_tokens=16384, n_heads=16, n_sub=44)
    inter = 16384 * 16 * 44 * 128 * 2
    bwd = mhffn.workspace_bytes(d, mhffn.OP_BACKWARD)
    # R and dp [H][E][N] fp32, partial sums of dW_r, and fp32 partial weight gradients of the
    # neuron groups of the last round (24 of 88 per XCD, four token segments): 266 MB, a
    # multiple of the parameter count and not of the token count -- not the intermediate
    n_weights = 3 * 16 * 44 * 128 * 128
    assert 2 * 16384 * 16 * 44 * 4 <= bwd < inter // 8
    assert bwd <= 2 * 16384 * 16 * 44 * 4 + 4 * (24 * n_weights // 88) * 4 + (32 << 20)
    assert mhffn.workspace_bytes(d, mhffn.OP_UNFUSED_FORWARD) >= 3 * inter
    assert mhffn.workspace_bytes(d, mhffn.OP_UNFUSED_BACKWARD) >= 4 * inter
    assert mhffn.workspace_bytes(d, 99) == 0


def test_backward_rejects_bad_arguments():
    lib = mhffn.load()
    d = desc(n_tokens=256)
    args = [FAKE] * 11
    assert lib.mhffn_backward(ctypes.byref(d), *args, None, 0, None) == 5      # no workspace
    # fp32 backward: supported shapes pass validation up to the workspace check, others do not
    assert lib.mhffn_backward(ctypes.byref(desc(dtype=mhffn.F32)), *args, None, 0, None) == 5
    assert lib.mhffn_backward(ctypes.byref(desc(dtype=mhffn.F32, d_head=512)), *args, FAKE, 1 << 30, None) == 3
    assert lib.mhffn_backward(ctypes.byref(desc(dtype=mhffn.F32, d_head=256, n_sub=200)), *args, FAKE, 1 << 30, None) == 3
    bad = list(args)
    bad[5] = None                                                               # dY missing
    assert lib.mhffn_backward(ctypes.byref(d), *bad, FAKE, 1 << 30, None) == 1
    assert lib.mhffn_backward_phases(ctypes.byref(d), *args, FAKE, 1 << 30, None, None, 3) == 1


def test_unfused_rejects_bad_arguments():
    lib = mhffn.load()
    args = [FAKE] * 12
    assert lib.mhffn_reference_unfused(ctypes.byref(desc()), *args, None, 0, None) == 5
    assert lib.mhffn_reference_unfused(ctypes.byref(desc(d_head=12)), *args, FAKE, 1 << 40, None) == 3


def test_module_entry_points_validate_before_launching():
    lib = mhffn.load()
    d = desc(n_tokens=16384, n_heads=16, n_sub=44)
    fwd_args, bwd_args = [FAKE] * 10, [FAKE] * 17
    # big batch: the forward needs no scratch, the backward needs dS, dQ and the fused scratch
    assert mhffn.workspace_bytes(d, mhffn.OP_MODULE_FORWARD) == 0
    act = 16384 * 2048 * 2
    need = mhffn.workspace_bytes(d, mhffn.OP_MODULE_BACKWARD)
    # dS, dQ, the fused scratch, and fp32 partial tiles of the two d_model x d_model weight
    # gradients (their contraction over the tokens is split over a few workgroups)
    partials = need - 2 * act - mhffn.workspace_bytes(d, mhffn.OP_BACKWARD)
    assert 0 <= partials <= 16 * 2048 * 2048 * 4 and partials % (2048 * 2048 * 4) == 0
    assert lib.mhffn_module_backward(ctypes.byref(d), *bwd_args, None, 0, None) == 5
    assert lib.mhffn_module_backward(ctypes.byref(d), *bwd_args, FAKE, need - 1, None) == 5
    # the module computes its gating weights itself
    dw = desc(route_mode=mhffn.ROUTE_WEIGHTS)
    assert lib.mhffn_module_forward(ctypes.byref(dw), *fwd_args, None, 0, None) == 3
    assert lib.mhffn_module_backward(ctypes.byref(dw), *bwd_args, FAKE, 1 << 40, None) == 3
    assert mhffn.workspace_bytes(dw, mhffn.OP_MODULE_BACKWARD) == 0
    # required pointers: X, the seven weights, O, Q, S
    for i in range(10):
        a = list(fwd_args)
        a[i] = None
        assert lib.mhffn_module_forward(ctypes.byref(d), *a, None, 0, None) == 1
        a[i] = ctypes.c_void_p(0x10008)
        assert lib.mhffn_module_forward(ctypes.byref(d), *a, None, 0, None) == 4
    for i in range(10):   # X .. dO are required, the gradient pointers are optional
        a = list(bwd_args)
        a[i] = None
        assert lib.mhffn_module_backward(ctypes.byref(d), *a, FAKE, 1 << 40, None) == 1
    # shapes the fused kernels do not take
    assert lib.mhffn_module_forward(ctypes.byref(desc(d_head=96)), *fwd_args, None, 0, None) == 3
    # empty batch: nothing to launch in the forward
    assert lib.mhffn_module_forward(ctypes.byref(desc(n_tokens=0)), *fwd_args, None, 0, None) == 0
