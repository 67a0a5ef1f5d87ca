#!/usr/bin/env python3
"""Benchmark of the fused Multi-Head FFN hot path on one MI355X.

One step = one fused forward plus one fused backward (all gradients) over one
batch of seeded synthetic input that is already resident in device memory.
Default workload: the 1.3B-scale shape (N = 16384 tokens, d_model = 2048,
H = 16, d_h = 128, E = 44 sub-networks of width 128, bf16 with fp32 accumulate).

Prints ONE JSON line.  `value` is algorithmic TFLOP/s of the whole step: 3
contraction units forward + 8 backward (recompute counted once), one unit being
2*N*d_model*d_ff flops.  Per-kernel durations are taken live with HIP events on
the stream the kernels run on; `roofline` describes the kernel that takes the
largest share of the step.  `cpu_baseline` is the fp64 oracle timed on this
machine's host cores on a bounded sample of the same workload.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


class HipEvents:
    """Raw hipEvent_t handles (the library records them between its kernels)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self, n):
        out = []
        for _ in range(n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError("hipEventCreate failed: %d" % rc)
            out.append(e.value)
        return out

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ctypes.c_void_p(ev), ctypes.c_void_p(stream))
        if rc != 0:
            raise RuntimeError("hipEventRecord failed: %d" % rc)

    def elapsed_ms(self, e0, e1):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(e0), ctypes.c_void_p(e1))
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)


def load_traffic(workload, forward_only):
    """{kernel key: HBM bytes per launch} for `workload` from profiles/hbm_traffic.txt
    (lines: workload step kernel-key read-bytes written-bytes source-file)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    out = {}
    if not os.path.exists(path):
        return out
    step = "fwd" if forward_only else "fwdbwd"
    for line in open(path):
        f = line.split()
        if len(f) >= 5 and not line.startswith("#") and f[0] == workload and f[1] == step:
            out[f[2]] = float(f[3]) + float(f[4])
    return out


def cpu_baseline(w, d, budget_heads=16, budget_tokens=6144):
    """The fp64 oracle, as it stands, on a bounded sample of the workload:
    `budget_heads` whole heads x the first `budget_tokens` tokens, forward + backward."""
    import numpy as np
    from oracle import mhffn_oracle as orc
    hs = min(budget_heads, w.n_heads)
    n = min(budget_tokens, w.n_tokens)
    cols = slice(0, hs * w.d_head)
    X = np.ascontiguousarray(d["X"][:n, cols], dtype=np.float64)
    dY = np.ascontiguousarray(d["dY"][:n, cols], dtype=np.float64)
    Wg, Wu, Wd = (d[k][:hs].astype(np.float64) for k in ("W_gate", "W_up", "W_down"))
    Wr = d["W_r"][:hs].astype(np.float64)
    orc.forward(X[:64], Wg, Wu, Wd, Wr, w.eps)  # load the library, warm the pages
    t0 = time.perf_counter()
    orc.forward(X, Wg, Wu, Wd, Wr, w.eps)
    t1 = time.perf_counter()
    orc.backward(X, Wg, Wu, Wd, Wr, dY, w.eps)
    t2 = time.perf_counter()
    unit = 2.0 * n * hs * w.d_head * w.d_ff
    return {
        "value": round(11.0 * unit / (t2 - t0) / 1e12, 5), "unit": "TFLOP/s",
        "cores": orc.threads(), "kind": "oracle",
        "sample": "fp64 oracle forward+backward on %d heads x first %d tokens of the workload "
                  "(%.1f s; 11 algorithmic units counted, 14 executed)" % (hs, n, t2 - t0),
        "fwd_s": round(t1 - t0, 3), "bwd_s": round(t2 - t1, 3),
    }


def time_config(hip, name, tokens=0, forward_only=True, steps=10, warmup=2):
    """One compact row for a configuration other than the headline one: average kernel
    durations over `steps` runs (HIP events on the launch stream), outside the headline's
    timed region."""
    import torch
    from paper_2512_06989_amd import inputs, mhffn
    from paper_2512_06989_amd.device import device_inputs
    w = inputs.WORKLOADS[name]
    if tokens:
        w = w.with_tokens(tokens)
    d = inputs.make_inputs(w, seed=0, with_dy=not forward_only)
    g = device_inputs(d, w.dtype)
    a = [g[k] for k in ("X", "W_gate", "W_up", "W_down", "W_r")]
    desc = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_PARAMS, w.eps)
    fws_b = mhffn.workspace_bytes(desc, mhffn.OP_FORWARD)
    bws_b = 0 if forward_only else mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD)
    fws = torch.empty(max(fws_b, 256), dtype=torch.uint8, device="cuda")
    bws = torch.empty(max(bws_b, 256), dtype=torch.uint8, device="cuda")
    Y = torch.empty_like(g["X"])
    grads = None if forward_only else {k: torch.empty_like(v) for k, v in zip(
        ("dX", "dW_gate", "dW_up", "dW_down", "d_route"), a)}
    hbm_bound = w.n_tokens <= 128
    # a weight-streaming shape must not be served from the 256 MB Infinity Cache
    wsets = [a[1:4]] + ([[t.clone() for t in a[1:4]] for _ in range(7)] if hbm_bound else [])
    stream = torch.cuda.current_stream().cuda_stream
    timing = "HIP events around every call"
    if forward_only and w.n_tokens <= 2048:
        # A forward of a few tens of microseconds is shorter than the host needs to enqueue it:
        # events around single calls would time the host.  Sixteen calls (twice round the weight
        # copies) are recorded into a HIP graph, as a serving loop would do, and replays are timed.
        per_graph = 16
        mhffn.init()
        mhffn.forward(a[0], *wsets[0], a[4], w.eps, out=Y, workspace=fws)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(per_graph):
                    mhffn.forward(a[0], *wsets[i % len(wsets)], a[4], w.eps, out=Y, workspace=fws)
        torch.cuda.current_stream().wait_stream(side)
        evs = [hip.create(2) for _ in range(warmup + steps)]
        for ev in evs:
            hip.record(ev[0], stream)
            graph.replay()
            hip.record(ev[1], stream)
        torch.cuda.synchronize()
        t_f = [hip.elapsed_ms(ev[0], ev[1]) / per_graph for ev in evs[warmup:]]
        f_ms, b_ms = sum(t_f) / len(t_f), 0.0
        timing = "replays of a HIP graph of %d calls" % per_graph
    else:
        evs = [hip.create(3) for _ in range(warmup + steps)]
        for i, ev in enumerate(evs):     # back to back, as in a serving or training loop
            ws_i = wsets[i % len(wsets)]
            hip.record(ev[0], stream)
            mhffn.forward(a[0], *ws_i, a[4], w.eps, out=Y, workspace=fws)
            hip.record(ev[1], stream)
            if not forward_only:
                mhffn.backward(*a, g["dY"], w.eps, workspace=bws, out=grads)
            hip.record(ev[2], stream)
        torch.cuda.synchronize()
        t_f = [hip.elapsed_ms(ev[0], ev[1]) for ev in evs[warmup:]]
        t_b = [hip.elapsed_ms(ev[1], ev[2]) for ev in evs[warmup:]]
        f_ms, b_ms = sum(t_f) / len(t_f), sum(t_b) / len(t_b)
    unit = w.unit_flops()
    row = {"workload": w.name, "n_tokens": w.n_tokens, "d_model": w.d_model, "n_sub": w.n_sub,
           "step": "forward" if forward_only else "forward + backward",
           "forward_ms": round(f_ms, 5), "timing": timing,
           "forward_workspace_bytes": fws_b}
    if hbm_bound:
        nbytes = (3 * w.d_model * w.d_ff + w.d_model * w.n_sub + 2 * w.n_tokens * w.d_model) * 2
        gbs = nbytes / (f_ms * 1e-3) / 1e9
        row.update({"bound": "hbm", "forward_GBps": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4),
                    "algorithmic_bytes": nbytes})
    else:
        tf = 3.0 * unit / (f_ms * 1e-3) / 1e12
        row.update({"bound": "mfma", "forward_TFLOPs": round(tf, 1), "frac": round(tf / PEAK_BF16_TFLOPS, 4)})
    if not forward_only:
        tb = 8.0 * unit / (b_ms * 1e-3) / 1e12
        ts = 11.0 * unit / ((f_ms + b_ms) * 1e-3) / 1e12
        row.update({"backward_ms": round(b_ms, 5), "backward_TFLOPs": round(tb, 1),
                    "backward_frac": round(tb / PEAK_BF16_TFLOPS, 4),
                    "step_TFLOPs": round(ts, 1), "step_frac": round(ts / PEAK_BF16_TFLOPS, 4),
                    "backward_workspace_bytes": bws_b})
    row["tokens_per_s"] = round(w.n_tokens / ((f_ms + (0 if forward_only else b_ms)) * 1e-3), 1)
    return row


def mfma_calibration(hip, launches=40, iters=2000):
    """Sustained rate of bare bf16 MFMA loops on this machine (calibration kernels of
    libmhffn_calib.so, about 0.15 s of back-to-back launches per mode after as much warm-up):
    with constant operands and with fresh pseudo-random operands for every product.  The
    second is what power management leaves of the published peak for data like the workload's."""
    import torch
    from paper_2512_06989_amd import build as lib_build
    if not os.path.exists(lib_build.CALIB_LIB):
        return None
    lib = ctypes.CDLL(lib_build.CALIB_LIB)
    lib.mhffn_calib_mfma_launch.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_void_p]
    lib.mhffn_calib_mfma_flops.restype = ctypes.c_double
    lib.mhffn_calib_mfma_flops.argtypes = [ctypes.c_int, ctypes.c_int]
    n_wg = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(n_wg * 512, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(n_wg * 16, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    out = {}
    for mode, key in ((0, "constant_operands"), (1, "random_operands")):
        def launch():
            rc = lib.mhffn_calib_mfma_launch(mode, n_wg, iters, sink.data_ptr(), clocks.data_ptr(), stream)
            if rc != 0:
                raise RuntimeError("calibration launch failed: %d" % rc)
        for _ in range(launches):
            launch()
        ev = hip.create(2)
        hip.record(ev[0], stream)
        for _ in range(launches):
            launch()
        hip.record(ev[1], stream)
        torch.cuda.synchronize()
        ms = hip.elapsed_ms(ev[0], ev[1])
        c = clocks.cpu().numpy().reshape(-1, 2)
        tf = lib.mhffn_calib_mfma_flops(n_wg, iters) * launches / (ms * 1e-3) / 1e12
        out[key] = {"TFLOPs": round(tf, 1), "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                    "clock_GHz": round(float(c[:, 0].sum()) / (float(c[:, 1].sum()) * 10.0), 3)}
    out["kernel"] = "v_mfma_f32_32x32x16_bf16 back to back, 2 waves per SIMD on %d CUs, no memory traffic" % n_wg
    return out


def allocator_high_water(fn):
    """Peak of torch's device allocator above its level before `fn` (buffers that fn allocates
    itself: the binding's workspace and outputs)."""
    import torch
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    before = torch.cuda.memory_allocated()
    fn()
    torch.cuda.synchronize()
    return int(torch.cuda.max_memory_allocated() - before)


def module_bench(args, w):
    """Step = forward + backward of the whole module: Q = X W_in, the fused path, O = S W_out
    and the four products of the backward around the fused backward.  The fused path alone is
    timed in the same run; the difference is the time of the six d_model x d_model products."""
    import torch
    from paper_2512_06989_amd import inputs, mhffn
    from paper_2512_06989_amd.device import device_inputs
    d = inputs.make_module_inputs(w, seed=0, with_dy=True)
    g = device_inputs(d, w.dtype)
    names = ("X", "W_in", "W_gate", "W_up", "W_down", "W_r", "W_out")
    a = [g[k] for k in names]
    core = [g[k] for k in ("X", "W_gate", "W_up", "W_down", "W_r")]
    desc = mhffn.make_desc(g["X"], g["W_gate"], mhffn.ROUTE_PARAMS, w.eps)
    ws = torch.empty(max(mhffn.workspace_bytes(desc, mhffn.OP_MODULE_BACKWARD), 256),
                     dtype=torch.uint8, device="cuda")
    fws = torch.empty(max(mhffn.workspace_bytes(desc, mhffn.OP_MODULE_FORWARD), 256),
                      dtype=torch.uint8, device="cuda")
    acts = {k: torch.empty_like(g["X"]) for k in ("O", "Q", "S")}
    grads = {k: torch.empty_like(v) for k, v in zip(mhffn.MODULE_GRADS, (
        g["X"], g["W_in"], g["W_gate"], g["W_up"], g["W_down"], g["W_r"], g["W_out"]))}
    cgrads = {"dX": grads["dX"], "dW_gate": grads["dW_gate"], "dW_up": grads["dW_up"],
              "dW_down": grads["dW_down"], "d_route": grads["dW_r"]}
    stream = torch.cuda.current_stream().cuda_stream
    hip = HipEvents()
    K = args.steps

    def mod_fwd():
        mhffn.module_forward(*a, w.eps, out=acts, workspace=fws)

    def mod_bwd():
        mhffn.module_backward(*a, acts["Q"], acts["S"], g["dY"], w.eps, out=grads, workspace=ws)

    def core_fwd():
        mhffn.forward(*core, w.eps, out=acts["S"], workspace=fws)

    def core_bwd():
        mhffn.backward(*core, g["dY"], w.eps, workspace=ws, out=cgrads)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        ev = hip.create(2)
        hip.record(ev[0], stream)
        for _ in range(K):
            fn()
        hip.record(ev[1], stream)
        torch.cuda.synchronize()
        return hip.elapsed_ms(ev[0], ev[1]) / K

    t = {"core_fwd": timed(core_fwd), "core_bwd": timed(core_bwd)}
    # the module step itself, timed as the contract says: K steps between synchronisations
    for _ in range(args.warmup):
        mod_fwd(); mod_bwd()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        mod_fwd(); mod_bwd()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K
    t["module_fwd"], t["module_bwd"] = timed(mod_fwd), timed(mod_bwd)
    # A dense SwiGLU FFN of the same d_model and d_ff (the layer the module replaces; same
    # 3 + 6 units of contraction work, no projections, no recompute): the unfused path with
    # one head, one sub-network and unit weights, which runs on the same product kernel and
    # keeps G, U' and A in device memory.
    dff = w.d_ff
    sw = [(torch.randn(1, 1, dff, w.d_model, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(3)]
    ones = torch.ones(w.n_tokens, 1, 1, device="cuda", dtype=torch.float32)
    sdesc = mhffn.make_desc(g["X"], sw[0], mhffn.ROUTE_WEIGHTS, w.eps)
    s_ws_f = mhffn.workspace_bytes(sdesc, mhffn.OP_UNFUSED_FORWARD)
    s_ws_b = mhffn.workspace_bytes(sdesc, mhffn.OP_UNFUSED_BACKWARD)
    sws = torch.empty(max(s_ws_b, 256), dtype=torch.uint8, device="cuda")
    sout = {"Y": torch.empty_like(g["X"]), "dX": torch.empty_like(g["X"]), "d_route": torch.empty_like(ones),
            "dW_gate": torch.empty_like(sw[0]), "dW_up": torch.empty_like(sw[0]), "dW_down": torch.empty_like(sw[0])}

    def swiglu_fwd():
        mhffn.reference_unfused(g["X"], *sw, ones, w.eps, mhffn.ROUTE_WEIGHTS, workspace=sws, out=sout)

    def swiglu_all():
        mhffn.reference_unfused(g["X"], *sw, ones, w.eps, mhffn.ROUTE_WEIGHTS, dY=g["dY"], workspace=sws, out=sout)

    t["swiglu_fwd"], t["swiglu_fwd_bwd"] = timed(swiglu_fwd), timed(swiglu_all)
    act_bytes = g["X"].numel() * 2
    unit = w.unit_flops()
    proj = 2.0 * w.n_tokens * w.d_model * w.d_model          # one projection-sized product
    flops = 11.0 * unit + 6.0 * proj
    gemm_ms = (t["module_fwd"] - t["core_fwd"]) + (t["module_bwd"] - t["core_bwd"])
    value = flops / (ms_per_step * 1e-3) / 1e12
    return {
        "metric": "FlashMHF module fwd/bwd TFLOP/s (projections W_in, W_out around the fused path)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + " (module)", "n_tokens": w.n_tokens, "d_model": w.d_model,
                   "n_heads": w.n_heads, "d_head": w.d_head, "n_sub": w.n_sub, "d_sub": w.d_sub,
                   "step": "module forward + module backward"},
        "frac_of_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "phase_ms": {k: round(v, 4) for k, v in t.items()},
        "dense_swiglu_same_size": {
            "forward_ms": round(t["swiglu_fwd"], 4), "forward_backward_ms": round(t["swiglu_fwd_bwd"], 4),
            "module_forward_speedup": round(t["swiglu_fwd"] / t["module_fwd"], 3),
            "module_step_speedup": round(t["swiglu_fwd_bwd"] / (t["module_fwd"] + t["module_bwd"]), 3),
            "saved_activation_bytes": {"module (Q, S)": 2 * act_bytes, "swiglu (G, U', A)": 3 * w.n_tokens * dff * 2},
            "forward_workspace_bytes": {"module": mhffn.workspace_bytes(desc, mhffn.OP_MODULE_FORWARD), "swiglu": s_ws_f},
        },
        "projections": {"count": 6, "ms": round(gemm_ms, 4),
                        "tflops": round(6.0 * proj / (gemm_ms * 1e-3) / 1e12, 1) if gemm_ms > 0 else None,
                        "frac_of_bf16_peak": round(6.0 * proj / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
                        if gemm_ms > 0 else None},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="1p3b_fwdbwd")
    ap.add_argument("--tokens", type=int, default=0, help="override the token count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the HBM byte "
                         "counters of a profiler run)")
    ap.add_argument("--rotate-weights", type=int, default=-1,
                    help="number of distinct weight copies to rotate over (default: 8 for the "
                         "HBM-bound small-N forward, else 1)")
    ap.add_argument("--no-unfused", dest="unfused", action="store_false",
                    help="skip the unfused GPU baseline comparison")
    ap.add_argument("--forward-only", action="store_true",
                    help="time the forward alone (step = forward); for profiling")
    ap.add_argument("--no-configs", dest="configs", action="store_false",
                    help="skip the MFMA calibration and the compact rows for the other configurations "
                         "(128M forward, 370M forward + backward, inference sweep)")
    ap.add_argument("--module", action="store_true",
                    help="time the whole module (W_in and W_out projections around the path) "
                         "instead; prints its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_06989_amd import inputs, mhffn
    from paper_2512_06989_amd.device import device_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    mhffn.load()
    w = inputs.WORKLOADS[args.workload]
    if args.tokens:
        w = w.with_tokens(args.tokens)
    if args.module:
        print(json.dumps(module_bench(args, w)))
        return
    d = inputs.make_inputs(w, seed=0, with_dy=True)
    g = device_inputs(d, w.dtype)
    X, Wg, Wu, Wd, Wr, dY = (g[k] for k in ("X", "W_gate", "W_up", "W_down", "W_r", "dY"))
    desc = mhffn.make_desc(X, Wg, mhffn.ROUTE_PARAMS, w.eps)
    ws_bytes = mhffn.workspace_bytes(desc, mhffn.OP_BACKWARD)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    Y = torch.empty_like(X)
    grads = {"dX": torch.empty_like(X), "dW_gate": torch.empty_like(Wg),
             "dW_up": torch.empty_like(Wu), "dW_down": torch.empty_like(Wd),
             "d_route": torch.empty_like(Wr)}
    stream = torch.cuda.current_stream().cuda_stream
    hip = HipEvents()
    K = args.steps
    ev = [hip.create(6) for _ in range(K)]   # per step: fwd start, fwd end/bwd start.. (4 bwd marks)
    fwd_ws_bytes = mhffn.workspace_bytes(desc, mhffn.OP_FORWARD)
    fwd_ws = torch.empty(max(fwd_ws_bytes, 256), dtype=torch.uint8, device="cuda")
    # A weight-streaming (HBM-bound) shape must not be served from the 256 MB
    # Infinity Cache: rotate over distinct copies of the weights (> 256 MB in total).
    hbm_bound = args.forward_only and w.n_tokens <= 128
    n_rot = args.rotate_weights if args.rotate_weights >= 0 else (8 if hbm_bound else 1)
    wsets = [(Wg, Wu, Wd)] + [(Wg.clone(), Wu.clone(), Wd.clone()) for _ in range(max(n_rot, 1) - 1)]
    counter = [0]

    def step(events=None):
        Wg_, Wu_, Wd_ = wsets[counter[0] % len(wsets)]
        counter[0] += 1
        if events is not None:
            hip.record(events[0], stream)
        mhffn.forward(X, Wg_, Wu_, Wd_, Wr, w.eps, out=Y, workspace=fwd_ws)
        if events is not None:
            hip.record(events[1], stream)
        if not args.forward_only:
            mhffn.backward(X, Wg, Wu, Wd, Wr, dY, w.eps, workspace=ws, out=grads,
                           phase_events=None if events is None else events[2:6])

    for _ in range(args.warmup):
        step()
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    unit = w.unit_flops()
    kern = {"fwd": [], "bwd_tok": [], "bwd_wgt": [], "bwd_route": []}
    for e in ev:
        kern["fwd"].append(hip.elapsed_ms(e[0], e[1]))
        if not args.forward_only:
            kern["bwd_tok"].append(hip.elapsed_ms(e[2], e[3]))
            kern["bwd_wgt"].append(hip.elapsed_ms(e[3], e[4]))
            kern["bwd_route"].append(hip.elapsed_ms(e[4], e[5]))
    avg = {k: (sum(v) / len(v) if v else 0.0) for k, v in kern.items()}
    # algorithmic contraction units per launch: recompute inside the weight-major
    # kernel is not credited (forward 3; token-major M,N,dA,dX,dX = 5; weight-major dK,dU,dV = 3)
    units = {"fwd": 3.0, "bwd_tok": 5.0, "bwd_wgt": 3.0, "bwd_route": 0.0}
    # up to 64 sub-networks the forward runs the pipelined kernel
    # (d_h = 128; the other head widths run the plainer kernels)
    fwd_pipelined = w.d_head == 128 and w.n_sub <= 64
    kernel_names = {"fwd": "fwd_bf16_flow_kernel" if fwd_pipelined else "fwd_bf16_kernel",
                    "bwd_tok": "bwd_tok_kernel",
                    "bwd_wgt": "bwd_wgt16_kernel" if w.d_head == 128 else "bwd_wgt_dh_kernel",
                    "bwd_route": "bwd_route_*"}

    # HBM bytes per launch measured with rocprofv3 (FETCH_SIZE + WRITE_SIZE, each scaled by
    # what the counter reads for a 256 MiB copy): read from profiles/hbm_traffic.txt, which is
    # written together with the profile summaries.  Only valid for the workload and step they
    # were taken on; null where there is no measurement.
    measured_traffic = load_traffic(w.name, args.forward_only)

    def roof(k):
        if k == "fwd" and hbm_bound:
            # compulsory bytes of one forward: weights + W_r + X + Y
            nbytes = (3 * w.d_model * w.d_ff + w.d_model * w.n_sub + 2 * w.n_tokens * w.d_model) * 2
            ach = nbytes / (avg[k] * 1e-3) / 1e9 if avg[k] > 0 else 0.0
            return {"bound": "hbm", "kernel": kernel_names[k], "achieved": round(ach, 1),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4),
                    "traffic": None, "avg_ms": round(avg[k], 5), "algorithmic_bytes": nbytes,
                    "weight_copies_rotated": len(wsets)}
        ach = units[k] * unit / (avg[k] * 1e-3) / 1e12 if avg[k] > 0 else 0.0
        # what the kernel actually runs on the MFMA (the weight-major kernel recomputes M, N, dA)
        executed = {"fwd": 3.0, "bwd_tok": 5.0, "bwd_wgt": 6.0, "bwd_route": 0.0}[k]
        return {"bound": "mfma", "kernel": kernel_names[k], "achieved": round(ach, 1),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                "traffic": measured_traffic.get(k), "avg_ms": round(avg[k], 4),
                "algorithmic_units": units[k], "executed_units": executed,
                "executed_frac": round(ach / PEAK_BF16_TFLOPS * executed / units[k], 4) if units[k] else None}

    dominant = max(avg, key=lambda k: avg[k])
    step_units = 3.0 if args.forward_only else 11.0
    value = step_units * unit / (ms_per_step * 1e-3) / 1e12

    # activation footprint: what the op needs beyond inputs, weights and gradients
    act_fused = Y.numel() * Y.element_size()
    unfused_ws = mhffn.workspace_bytes(desc, mhffn.OP_UNFUSED_FORWARD)
    unfused_ws_bwd = mhffn.workspace_bytes(desc, mhffn.OP_UNFUSED_BACKWARD)
    out = {
        "metric": "fused MH-FFN fwd/bwd TFLOP/s, % bf16 MFMA peak; peak activation bytes",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + (" (forward only)" if args.forward_only else ""),
                   "n_tokens": w.n_tokens, "d_model": w.d_model, "n_heads": w.n_heads,
                   "d_head": w.d_head, "n_sub": w.n_sub, "d_sub": w.d_sub, "d_ff": w.d_ff,
                   "step": "fused forward" if args.forward_only else "fused forward + fused backward"},
        "frac_of_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "tokens_per_s": round(w.n_tokens / (ms_per_step * 1e-3), 1),
        "kernel_ms": {k: round(v, 4) for k, v in avg.items()},
        "roofline": roof(dominant),
        "roofline_fwd": roof("fwd"),
        "peak_activation_bytes": {
            "fused_forward": act_fused,
            "fused_forward_workspace": fwd_ws_bytes,
            "fused_backward_workspace": ws_bytes,
            "unfused_forward_workspace": unfused_ws or None,
            "unfused_backward_workspace": unfused_ws_bwd or None,
            "intermediate_if_materialised": 3 * w.n_tokens * w.n_heads * w.d_ff * 2,
        },
    }
    if args.unfused:
        # the unfused GPU baseline on the same inputs (outside the timed region)
        uws = torch.empty(unfused_ws_bwd, dtype=torch.uint8, device="cuda")
        uout = {"Y": torch.empty_like(X), **{k: torch.empty_like(v) for k, v in grads.items()}}

        def time_unfused(with_bwd, reps=3):
            mhffn.reference_unfused(X, Wg, Wu, Wd, Wr, w.eps, dY=dY if with_bwd else None,
                                    workspace=uws, out=uout)
            e0, e1 = hip.create(2)
            hip.record(e0, stream)
            for _ in range(reps):
                mhffn.reference_unfused(X, Wg, Wu, Wd, Wr, w.eps, dY=dY if with_bwd else None,
                                        workspace=uws, out=uout)
            hip.record(e1, stream)
            torch.cuda.synchronize()
            return hip.elapsed_ms(e0, e1) / reps

        u_fwd = time_unfused(False)
        u_all = time_unfused(True)
        out["unfused_baseline"] = {
            "forward_ms": round(u_fwd, 3), "forward_backward_ms": round(u_all, 3),
            "fused_forward_speedup": round(u_fwd / avg["fwd"], 2) if avg["fwd"] else None,
            "fused_step_speedup": None if args.forward_only else round(u_all / ms_per_step, 2),
            "activation_bytes_ratio_forward": round((act_fused + unfused_ws) / act_fused, 1),
        }
        del uws, uout
    if not args.forward_only:
        out["roofline_bwd_tok"] = roof("bwd_tok")
        out["roofline_bwd_wgt"] = roof("bwd_wgt")
    if args.unfused and not args.forward_only:
        # allocator high-water marks of one call each, outputs and scratch allocated by the
        # binding (what a caller without buffers of its own pays)
        out["peak_activation_bytes"]["allocator_high_water"] = {
            "fused_forward": allocator_high_water(lambda: mhffn.forward(X, Wg, Wu, Wd, Wr, w.eps)),
            "unfused_forward": allocator_high_water(lambda: mhffn.reference_unfused(X, Wg, Wu, Wd, Wr, w.eps)),
            "fused_forward_backward": allocator_high_water(
                lambda: (mhffn.forward(X, Wg, Wu, Wd, Wr, w.eps), mhffn.backward(X, Wg, Wu, Wd, Wr, dY, w.eps))),
            "unfused_forward_backward": allocator_high_water(
                lambda: mhffn.reference_unfused(X, Wg, Wu, Wd, Wr, w.eps, dY=dY)),
        }
    if args.configs and not hbm_bound:
        # Context for the roofline fractions: the same launches on operands that hardly toggle
        # the multipliers (X = dY = 1, weights 0.01: every product is the same number).  The
        # instruction streams are identical; what differs is the clock that power management
        # grants, so these times are what the kernels' schedules take when power is no limit.
        cX, cdY = torch.ones_like(X), torch.ones_like(dY)
        cW = [torch.full_like(t, 0.01) for t in (Wg, Wu, Wd)]
        cev = [hip.create(6) for _ in range(8)]
        for i in range(3 + len(cev)):
            e = cev[i - 3] if i >= 3 else None
            if e is not None:
                hip.record(e[0], stream)
            mhffn.forward(cX, *cW, Wr, w.eps, out=Y, workspace=fwd_ws)
            if e is not None:
                hip.record(e[1], stream)
            if not args.forward_only:
                mhffn.backward(cX, *cW, Wr, cdY, w.eps, workspace=ws, out=grads,
                               phase_events=None if e is None else e[2:6])
        torch.cuda.synchronize()
        cavg = {"fwd": sum(hip.elapsed_ms(e[0], e[1]) for e in cev) / len(cev)}
        if not args.forward_only:
            cavg["bwd_tok"] = sum(hip.elapsed_ms(e[2], e[3]) for e in cev) / len(cev)
            cavg["bwd_wgt"] = sum(hip.elapsed_ms(e[3], e[4]) for e in cev) / len(cev)
        executed = {"fwd": 3.0, "bwd_tok": 5.0, "bwd_wgt": 6.0}
        out["constant_operands"] = {
            "what": "same kernels and launches, X = dY = 1 and weights = 0.01 (power management "
                    "grants a higher clock when the operands do not toggle the multipliers)",
            "kernel_ms": {k: round(v, 4) for k, v in cavg.items()},
            "executed_frac_of_peak": {k: round(executed[k] * unit / (v * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
                                      for k, v in cavg.items() if v > 0},
        }
        del cX, cdY, cW
    if args.configs:
        # context for the roofline fractions: what bare MFMA loops sustain on this machine
        cal = mfma_calibration(hip)
        if cal:
            out["mfma_sustained"] = cal
            # the same rates against what a bare MFMA loop with data like the workload's sustains
            # here (context only: `frac` stays the fraction of the published peak)
            sus = cal["random_operands"]["TFLOPs"]
            for key in ("roofline", "roofline_fwd", "roofline_bwd_tok", "roofline_bwd_wgt"):
                r = out.get(key)
                if r and r.get("bound") == "mfma" and sus > 0:
                    r["frac_of_sustained_mfma"] = round(r["achieved"] / sus, 4)
                    if "executed_frac" in r:
                        r["executed_frac_of_sustained_mfma"] = round(r["executed_frac"] * PEAK_BF16_TFLOPS / sus, 4)
    if args.configs and w.name == "1p3b_fwdbwd" and not args.forward_only and not args.tokens:
        # the other configurations, a few seconds in all, outside the timed region above
        del g, X, Y, dY, grads, ws, fwd_ws
        torch.cuda.empty_cache()
        out["configs"] = [
            time_config(hip, "128m_fwd"),
            time_config(hip, "370m_fwdbwd", forward_only=False),
            time_config(hip, "1p3b_sweep", tokens=64, steps=40, warmup=8),
            time_config(hip, "1p3b_sweep", tokens=1024, steps=20, warmup=4),
            time_config(hip, "1p3b_sweep", tokens=32768),
        ]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, d)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
