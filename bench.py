#!/usr/bin/env python3
"""Benchmark of the in-hindsight quantized layer path on one MI355X.

A step is one pass of the whole hot path over one batch of the ResNet-style 3x3 conv
64->64 at 56x56, batch 128 (M=401408, K=576, N=64): forward GEMM with the fused
in-hindsight epilogue, input-gradient GEMM with the same epilogue, the FP32 weight-gradient
GEMM, and the range update (eq. (2)-(3)) of both quantizers in one launch.  Inputs are seeded synthetic tensors that
are resident in HBM before the timed region.  The dynamic two-pass baseline, the depthwise
stencil and the other layer shapes are timed next to it and reported in the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--calibrate-copy]

One GPU only: this build has no multi-GPU path.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0        # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-extras", action="store_true", help="time only the headline step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch plain device copies of known size (counter calibration under rocprofv3 --pmc)")
    ap.add_argument("--stack-only", choices=["fused", "dynamic"],
                    help="run nothing but the ResNet-18-shaped stack: range initialisation, one warm-up step and "
                         "--steps steps of the chosen kind (for counter collection under rocprofv3 --pmc: the "
                         "last `launches_per_step` dispatches of the run are one step)")
    return ap.parse_args()


class Layer:
    """Device-side operands and state of one layer (torch holds the memory, nothing else)."""

    def __init__(self, hq, torch, wl, L, X, W, dY, state=None):
        self.hq, self.torch, self.L = hq, torch, L
        self.p = hq.problem(L.kind, L.B, L.H, L.W, L.C, L.R, L.S, L.stride, L.pad, L.Cout)
        dev = lambda a: a if torch.is_tensor(a) else torch.from_numpy(np.ascontiguousarray(a)).cuda()
        self.X, self.xq = dev(X.codes), hq.new_qparams(X.scale, X.zero_point)
        self.dY, self.gq = dev(dY.codes), hq.new_qparams(dY.scale, dY.zero_point)
        self.W, self.wq = dev(W.codes), hq.new_qparams(W.scale, 0)
        self.wsum = torch.empty(L.Cout, dtype=torch.int32, device="cuda")
        self.wdsum = torch.empty(L.C, dtype=torch.int32, device="cuda")
        if L.kind == wl.DEPTHWISE:
            self.Wd = self.W
            hq.hq_weight_prepare(self.p, self.W, None, self.wsum, self.wdsum)
        else:
            self.Wd = torch.empty(self.W.numel(), dtype=torch.int8, device="cuda")
            hq.hq_weight_prepare(self.p, self.W, self.Wd, self.wsum, self.wdsum)
        self.Y = torch.empty(wl.out_shape(L), dtype=torch.int8, device="cuda")
        self.dX = torch.empty(wl.in_shape(L), dtype=torch.int8, device="cuda")
        self.dW = torch.empty(wl.w_shape(L), dtype=torch.float32, device="cuda")
        self.yq, self.dxq = hq.new_qparams(0, 0), hq.new_qparams(0, 0)
        if state is None:
            # range states and statistics of the layer's two quantizers as arrays of two records, so that
            # both are updated by one launch
            self.ranges, self.stats = hq.new_ranges([False, True]), hq.new_stats(2)
            rs, ss = hq.RANGE.itemsize, hq.STATS.itemsize
            state = (self.ranges[:rs], self.ranges[rs:], self.stats[:ss], self.stats[ss:])
        self.yr, self.gr, self.yst, self.gst = state
        self.ws_w = hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, self.p)
        self.ws_f = hq.hq_workspace_bytes(hq.HQ_ENTRY_DYNAMIC_FWD, self.p)
        self.ws_d = hq.hq_workspace_bytes(hq.HQ_ENTRY_DYNAMIC_DGRAD, self.p) if L.C != 3 else 0
        self.ws = torch.empty(max(self.ws_w, self.ws_f, self.ws_d, 16), dtype=torch.uint8, device="cuda")

    # the five entry points ------------------------------------------------------------
    def fwd(self):
        self.hq.hq_gemm_fwd(self.p, self.X, self.xq, self.W, self.wq, self.wsum, self.yr, self.Y, self.yq, self.yst)

    def dgrad(self):
        self.hq.hq_gemm_dgrad(self.p, self.dY, self.gq, self.Wd, self.wq, self.wdsum, self.gr, self.dX, self.dxq, self.gst)

    def dgrad_sr(self):
        """The input gradient with stochastic rounding (what the paper uses for gradients, Sec. 5)."""
        self.sr_step = getattr(self, "sr_step", 0) + 1
        self.hq.hq_gemm_dgrad_sr(self.p, self.dY, self.gq, self.Wd, self.wq, self.wdsum, self.gr,
                                 (0x9e3779b97f4a7c15 * self.sr_step) % 2 ** 64, self.dX, self.dxq, self.gst)

    def wgrad(self):
        self.hq.hq_gemm_wgrad(self.p, self.X, self.xq, self.dY, self.gq, self.dW, None, self.ws, self.ws_w)

    def upd_y(self):
        self.hq.hq_range_update(self.yr, self.yst)

    def upd_g(self):
        self.hq.hq_range_update(self.gr, self.gst)

    def dyn_fwd(self):
        hq = self.hq
        hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_FWD, hq.HQ_DYN_CURRENT, self.p, self.X, self.xq, self.W, self.wq,
                           self.wsum, self.yr, self.Y, self.yq, self.yst, self.ws, self.ws_f)

    def dyn_dgrad(self):
        hq = self.hq
        hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_DGRAD, hq.HQ_DYN_CURRENT, self.p, self.dY, self.gq, self.Wd, self.wq,
                           self.wdsum, self.gr, self.dX, self.dxq, self.gst, self.ws, self.ws_d)

    def init_ranges(self):
        """Iteration 0: the first batch sets q^0 through the dynamic path (Sec. 4.1)."""
        self.dyn_fwd(); self.upd_y()
        if self.L.C != 3:                      # a 3-channel first layer has no input gradient
            self.dyn_dgrad(); self.upd_g()

    def upd_both(self):
        self.hq.hq_range_update_batch(self.ranges, self.stats, 2)

    def wgrad_upd(self):
        """The weight gradient with both range updates (eq. (2)-(3) for Q_Y and Q_G) riding in its last launch."""
        self.hq.hq_gemm_wgrad_update(self.p, self.X, self.xq, self.dY, self.gq, self.dW, None, self.ws, self.ws_w,
                                     self.ranges, self.stats, 2)

    def fused_step(self):
        # a tensor's range is read next by the following iteration: both updates ride in the step's last launch
        self.fwd(); self.dgrad(); self.wgrad_upd()

    def fused_step_separate_update(self):
        self.fwd(); self.dgrad(); self.wgrad(); self.upd_both()

    def dynamic_step(self):
        self.dyn_fwd(); self.dyn_dgrad(); self.wgrad_upd()


class DeviceLayer(Layer):
    """Layer whose synthetic operands are drawn on the device (same recipe as workloads.py:
    post-ReLU activations on the unsigned grid, He-normal symmetric weights, Laplace gradients),
    used where host generation of a whole network's tensors would dominate the run."""

    def __init__(self, hq, torch, wl, L, seed, state=None):
        from collections import namedtuple
        Q = namedtuple("Q", "codes scale zero_point")
        g = torch.Generator(device="cuda").manual_seed(seed)
        x = torch.randn(wl.in_shape(L), generator=g, device="cuda").clamp_(min=0)
        sx = float(x.max()) / 255.0
        xc = (torch.round(x / sx).clamp_(0, 255) - 128).to(torch.int8)
        fan_in = L.R * L.S * (1 if L.kind == wl.DEPTHWISE else L.C)
        w = torch.randn(wl.w_shape(L), generator=g, device="cuda") * (2.0 / fan_in) ** 0.5
        sw = float(w.abs().max()) / 127.0
        wc = torch.round(w / sw).clamp_(-127, 127).to(torch.int8)
        u = torch.rand(wl.out_shape(L), generator=g, device="cuda") - 0.5
        gr = -1e-3 * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.4999999))
        sg = float(gr.abs().max()) / 127.0
        gc = torch.round(gr / sg).clamp_(-127, 127).to(torch.int8)
        del x, w, u, gr
        as_q = lambda t, s, z: Q(t, np.float32(s), z)
        Layer.__init__(self, hq, torch, wl, L, as_q(xc, sx, -128), as_q(wc, sw, 0), as_q(gc, sg, 0), state)


def kernel_family(wl, L, op):
    """Name of the kernel the library's dispatch picks for one launch (mirrors the rules of hq_api.hip / the launchers)."""
    k3 = L.kind == wl.CONV and L.R == 3 and L.S == 3 and L.stride == 1 and L.pad == 1
    first = L.kind == wl.CONV and L.C in (3, 4)
    staged = first and L.stride % 2 == 0 and L.W % 4 == 0 and L.S <= 8        # input rows staged in LDS
    if op == "wgrad":
        if k3 and L.C % 64 == 0 and L.Cout % 64 == 0:
            return "hq_wgrad_band_kernel + wband_finalize_kernel"
        if staged and L.R <= 8 and L.Cout <= 64 and L.Cout % 16 == 0:
            return "hq_wgrad_stem_kernel + wgrad_finalize_kernel"
        return "hq_wgrad_kernel + wgrad_finalize_kernel"
    cin = L.Cout if op == "dgrad" else L.C
    cout = L.C if op == "dgrad" else L.Cout
    if op == "fwd" and first:
        return "hq_stem_kernel" if staged else "hq_direct_kernel"
    if k3 and cin % 64 == 0 and cin >= 128 and cout >= 128:
        return "hq_bandw_kernel"
    if k3 and cin == 64:
        return "hq_band_kernel"
    return "hq_gemm_kernel"


def stack_step(hq, torch, wl, specs, label, reps=20, warmup=3, config=None, only=None):
    """One quantized training step over a stack of layers at batch 256: a forward and a wgrad launch
    per layer and a dgrad launch for all but the first, with in-hindsight ranges, against the same
    step with the dynamic two-pass path.  With `config` the operands are the host-generated tensors of
    workloads.layer_inputs(L, config, 1, index) -- the generator the parity tests use -- otherwise they
    are drawn on the device with the same recipe."""
    # all range states of the step in one array ([activations of every layer], [gradients of every
    # layer]) and their statistics in another: one update launch after each sweep
    n = len(specs)
    ranges, stats = hq.new_ranges([False] * n + [True] * n), hq.new_stats(2 * n)
    rs, ss = hq.RANGE.itemsize, hq.STATS.itemsize
    state = lambda i: (ranges[i * rs:(i + 1) * rs], ranges[(n + i) * rs:(n + i + 1) * rs],
                       stats[i * ss:(i + 1) * ss], stats[(n + i) * ss:(n + i + 1) * ss])
    layers = []
    for i, L in enumerate(specs):
        if config is None:
            layers.append(DeviceLayer(hq, torch, wl, L, 1000 + i, state(i)))
        else:
            X, W, dY = wl.layer_inputs(L, config, 1, i, image_input=(i == 0))
            layers.append(Layer(hq, torch, wl, L, X, W, dY, state(i)))
    for ly in layers:
        ly.init_ranges()

    def sweep(fwd, dgrad):
        for ly in layers:
            fwd(ly)
        hq.hq_range_update_batch(ranges, stats, n)                       # Q_Y of every layer
        for i, ly in reversed(list(enumerate(layers))):
            if i > 0:
                dgrad(ly)
            ly.wgrad()
        hq.hq_range_update_batch(ranges[n * rs:], stats[n * ss:], n)      # Q_G of every layer (the stem's saw no data)

    fused = lambda: sweep(lambda ly: ly.fwd(), lambda ly: ly.dgrad())
    dynamic = lambda: sweep(lambda ly: ly.dyn_fwd(), lambda ly: ly.dyn_dgrad())
    # kernel launches of one step: 1 per fused GEMM, 3 per dynamic one (two passes and the range between
    # them), 2 per weight gradient (3 where the integer sums start from zero), 2 range updates
    if only is not None:
        # counter collection: a stats_fold_kernel launch (used nowhere else in a step) brackets every step
        step = fused if only == "fused" else dynamic
        mark = hq.new_stats(1)
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            hq.hq_stats_fold(mark, 1)
            step()
        hq.hq_stats_fold(mark, 1)
        torch.cuda.synchronize()
        return {"workload": label, "kind": only, "steps": reps, "ms_per_step_wall": (time.perf_counter() - t0) * 1e3 / reps}

    fused_sr = lambda: sweep(lambda ly: ly.fwd(), lambda ly: ly.dgrad_sr())       # the paper's gradient rounding (Sec. 5)
    f_ms, d_ms = time_calls(torch, fused, reps, warmup), time_calls(torch, dynamic, reps, warmup)
    sr_ms = time_calls(torch, fused_sr, reps, warmup)
    # every layer's three launches on their own (five repetitions each, back to back)
    per_layer, fam = [], {}
    for i, (L, ly) in enumerate(zip(specs, layers)):
        gop = 2 * wl.macs(L) / 1e9
        row = {"layer": L.name, "gop": gop, "fwd_ms": time_calls(torch, ly.fwd, 5, 1),
               "dgrad_ms": time_calls(torch, ly.dgrad, 5, 1) if i > 0 else None, "wgrad_ms": time_calls(torch, ly.wgrad, 5, 1)}
        row["fwd_tops"] = gop / row["fwd_ms"]
        per_layer.append(row)
        for op in ("fwd", "dgrad", "wgrad"):
            if row[op + "_ms"] is None:
                continue
            f = fam.setdefault(kernel_family(wl, L, op), {"launches": 0, "ms": 0.0, "gop": 0.0, "alg_bytes": 0})
            f["launches"] += 1; f["ms"] += row[op + "_ms"]; f["gop"] += gop; f["alg_bytes"] += wl.fused_bytes(L, op)
    hq.hq_stats_reset(stats, 2 * n)
    ops = sum(2 * wl.macs(L) * (3 if i > 0 else 2) for i, L in enumerate(specs))
    fb = sum(wl.fused_bytes(L, o) for i, L in enumerate(specs) for o in (("fwd", "dgrad", "wgrad") if i > 0 else ("fwd", "wgrad")))
    db = sum(wl.dynamic_bytes(L, o) for i, L in enumerate(specs) for o in (("fwd", "dgrad", "wgrad") if i > 0 else ("fwd", "wgrad")))
    # the kernel that takes the largest share of the fused step, against the int8 MFMA peak
    dom = max(fam, key=lambda k: fam[k]["ms"])
    d = fam[dom]
    roofline = {"kernel": dom, "bound": "mfma", "launches_per_step": d["launches"], "ms_per_step": d["ms"],
                "achieved": d["gop"] / d["ms"], "peak": PEAK_INT8_TOPS, "unit": "TOP/s",        # GOP / ms = TOP/s
                "frac": d["gop"] / d["ms"] / PEAK_INT8_TOPS,
                "hbm_frac_of_8TBs": d["alg_bytes"] / (d["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "how": "sum over the step's launches of this kernel, each timed alone (5 back-to-back repetitions, HIP events)"}
    return {"workload": "%s: %d fwd + %d dgrad + %d wgrad" % (label, n, n - 1, n), "ops": ops,
            "inputs": "workloads.layer_inputs (host-generated, the parity tests' generator)" if config is not None
                      else "drawn on the device with the recipe of workloads.py (not the parity tests' tensors)",
            "timed_steps": reps, "warmup_steps": warmup,
            "fused_ms_per_step": f_ms, "dynamic_ms_per_step": d_ms, "fused_tops": ops / (f_ms * 1e-3) / 1e12,
            "speedup_vs_dynamic": d_ms / f_ms,
            "fused_ms_per_step_stochastic_dgrad": sr_ms, "per_layer": per_layer,
            "time_by_kernel_ms": {k: v["ms"] for k, v in fam.items()}, "roofline": roofline,
            "algorithmic_hbm_bytes_per_step": {"fused": fb, "dynamic": db, "ratio": db / fb}}


def range_tracking(hq, torch, lay, op, scales, report):
    """How the in-hindsight range follows a tensor whose magnitude changes from one iteration to the
    next (Sec. 4, eq. (2)-(3)): `op` ("fwd" or "dgrad") runs once per entry of `scales` with the
    quantization scale of its data operand set to that entry (same codes, so the real-valued output
    grows or shrinks by exactly that factor).  Iteration 0 sets the range from its own statistics;
    every later one quantizes with the range it was handed and then updates it.  Reported for the
    iterations in `report`: the share of outputs clipped, and the width of the range that was used
    over the width of the tensor's own min / max."""
    sym = op == "dgrad"
    rng_, st = hq.new_range(0.9, sym), hq.new_stats(1)
    keep = (lay.yr, lay.yst, lay.gr, lay.gst)
    qp, run, dyn = (lay.gq, lay.dgrad, lay.dyn_dgrad) if sym else (lay.xq, lay.fwd, lay.dyn_fwd)
    qp0 = qp.clone()
    zp = int(hq.from_device(qp0, hq.QPARAMS)[0]["zero_point"])
    if sym:
        lay.gr, lay.gst = rng_, st
    else:
        lay.yr, lay.yst = rng_, st
    rows = []
    for t, sc in enumerate(scales):
        qp.copy_(hq.new_qparams(sc, zp))
        (dyn if t == 0 else run)()
        hq.hq_stats_fold(st, 1)
        s, r = hq.from_device(st, hq.STATS)[0], hq.from_device(rng_, hq.RANGE)[0]
        if t in report:
            true_w = (float(s["acc_max"]) - float(s["acc_min"])) * float(s["acc_scale"])
            rows.append({"t": t, "clip_rate": float(s["clip_lo"] + s["clip_hi"]) / float(s["count"]),
                         "range_over_minmax": (float(r["qmax"]) - float(r["qmin"])) / true_w if t else 1.0})
        hq.hq_range_update(rng_, st)
    qp.copy_(qp0)
    lay.yr, lay.yst, lay.gr, lay.gst = keep
    return rows


def tensor_quantizer(hq, torch, wl):
    """Element-wise quantizer of an FP32 tensor the size of the headline layer's output (a
    normalisation / activation output): the in-hindsight single pass against the dynamic two-pass
    one, each as GB/s of its own algorithmic traffic (5 and 9 bytes per element)."""
    n = wl.nelem(wl.out_shape(wl.c2_layer()))
    x = torch.from_numpy(wl.real_activation(wl.rng(2, 0, 77), n)).cuda()
    q = torch.empty(n, dtype=torch.int8, device="cuda")
    r, st, qp = hq.new_range(0.9, False), hq.new_stats(1), hq.new_qparams(1.0, 0)
    hq.hq_tensor_quantize_dynamic(hq.HQ_DYN_CURRENT, x, n, r, q, qp, st)
    hq.hq_range_update(r, st)

    def static():
        hq.hq_tensor_quantize(x, n, r, q, qp, st)
        hq.hq_range_update(r, st)

    def dynamic():
        hq.hq_tensor_quantize_dynamic(hq.HQ_DYN_CURRENT, x, n, r, q, qp, st)
        hq.hq_range_update(r, st)

    s_ms, d_ms = time_calls(torch, static, 20), time_calls(torch, dynamic, 20)
    return {"elements": n, "in_hindsight_ms": s_ms, "dynamic_ms": d_ms, "speedup": d_ms / s_ms,
            "in_hindsight_alg_GBs": 5 * n / (s_ms * 1e-3) / 1e9, "dynamic_alg_GBs": 9 * n / (d_ms * 1e-3) / 1e9}


def time_calls(torch, fn, reps, warmup=2):
    """Average milliseconds of fn() over `reps` back-to-back launches, HIP events on the launch stream."""
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def cpu_baseline(wl, sample_B, min_seconds=10.0):
    """The oracle as it stands, timed on the host cores on a slice of the same workload:
    whole passes of the layer step until at least `min_seconds` of CPU work are done."""
    import oracle
    L, X, W = wl.c2_inputs(1, B=sample_B)
    dY = wl.laplace_gradient(wl.rng(2, 1, 2), wl.out_shape(L), 1e-3)
    p = oracle.Problem(L.kind, L.B, L.H, L.W, L.C, L.R, L.S, L.stride, L.pad, L.Cout)
    ry, rg = oracle.Range.new(0.9, False), oracle.Range.new(0.9, True)
    passes, t0 = 0, time.perf_counter()
    while passes == 0 or time.perf_counter() - t0 < min_seconds:
        c = oracle.fwd(p, X.codes, X.zero_point, W.codes)
        oracle.in_hindsight_step(c, oracle.acc_scale(X.scale, W.scale), ry)
        c = oracle.dgrad(p, dY.codes, dY.zero_point, W.codes)
        oracle.in_hindsight_step(c, oracle.acc_scale(dY.scale, W.scale), rg)
        c = oracle.wgrad(p, X.codes, X.zero_point, dY.codes, dY.zero_point)
        oracle.wgrad_scale(c, X.scale, dY.scale)
        passes += 1
    dt = time.perf_counter() - t0
    ops = passes * 3 * 2 * wl.macs(L)
    return {"value": ops / dt / 1e12, "unit": "TOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "the headline layer and step at batch %d of 128 (the same seeded inputs), %d whole passes (%.1f GOP) in %.1f s"
                      % (sample_B, passes, ops / 1e9, dt)}


def stored_traffic(kernel):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        return json.load(open(path)).get(kernel)
    except (OSError, ValueError):
        return None


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no multi-GPU path exists); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    import paper_2105_04246_amd as hq
    import workloads as wl

    torch.cuda.set_device(0)
    if args.stack_only:
        out = stack_step(hq, torch, wl, wl.resnet18_layers(B=256), "ResNet-18-shaped stack, batch 256 @224x224",
                         reps=args.steps, only=args.stack_only)
        if args.calibrate_copy:
            a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
            b = torch.empty_like(a)
            b.copy_(a)
            torch.cuda.synchronize()
            out["calibration_copy_bytes"] = {"read": a.numel(), "write": a.numel()}
        print(json.dumps(out))
        return
    L, X, W = wl.c2_inputs(1)
    dY = wl.laplace_gradient(wl.rng(2, 1, 2), wl.out_shape(L), 1e-3)
    lay = Layer(hq, torch, wl, L, X, W, dY)
    lay.init_ranges()
    torch.cuda.synchronize()

    # ---- headline: W warm-up steps, then exactly K timed steps -----------------------------
    K, Wm = args.steps, args.warmup
    calls = [("fwd", lay.fwd), ("dgrad", lay.dgrad), ("wgrad", lay.wgrad_upd)]       # wgrad carries both range updates
    # warm-up steps, with an event after every call: they name the slowest GEMM launch
    wev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(max(Wm, 1))]
    for k in range(max(Wm, 1)):
        wev[k][0].record()
        for i, (_, fn) in enumerate(calls):
            fn()
            wev[k][i + 1].record()
    torch.cuda.synchronize()
    per_call = {name: min(wev[k][i].elapsed_time(wev[k][i + 1]) for k in range(len(wev))) for i, (name, _) in enumerate(calls)}
    dom = max(("fwd", "dgrad", "wgrad"), key=lambda n: per_call[n])
    # timed region: exactly K steps.  The dominant launch is bracketed by events on every EV-th step only:
    # an event between two kernels keeps the second from starting while the first drains, which costs
    # the step about as much as the range update does
    EV = 10
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range((K + EV - 1) // EV)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        for name, fn in calls:
            if name == dom and k % EV == 0:
                ev[k // EV][0].record(); fn(); ev[k // EV][1].record()
            else:
                fn()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / K
    dom_ms = sum(a.elapsed_time(b) for a, b in ev) / len(ev)
    # what a pair of events with nothing between them reads on the same busy stream (after the timed
    # region): the part of dom_ms that is the events' own, reported next to it and not subtracted
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for a, b in pairs:
        calls[0][1]()
        a.record(); b.record()
    torch.cuda.synchronize()
    pair_ms = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)

    ops_gemm = 2 * wl.macs(L)
    step_ops = 3 * ops_gemm
    value = step_ops / (wall_ms * 1e-3) / 1e12

    # ---- roofline of the dominant kernel: the slowest of the three GEMM launches ------------
    names = {"fwd": "hq_band_kernel<64,3,2,8,1,fused> (forward)", "dgrad": "hq_band_kernel<64,3,2,8,1,fused> (dgrad)",
             "wgrad": "hq_wgrad_band_kernel + wband_finalize_kernel (one hq_gemm_wgrad_update call)"}
    achieved = ops_gemm / (dom_ms * 1e-3) / 1e12
    # the int8 MFMA rate this device sustains in a register-only loop, next to the published peak
    sink = torch.empty(2048 * 256, dtype=torch.int32, device="cuda")
    probe_ops = hq.hq_probe_mfma_rate(2048, 512, sink)
    probe_ms = time_calls(torch, lambda: hq.hq_probe_mfma_rate(2048, 4096, sink), 3, 1)
    peak_measured = probe_ops * 8 / (probe_ms * 1e-3) / 1e12
    del sink
    roofline = {"kernel": names[dom], "bound": "mfma", "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": achieved / PEAK_INT8_TOPS, "peak_measured": peak_measured,
                "frac_of_measured": achieved / peak_measured, "traffic": stored_traffic(dom),
                "traffic_source": "stored: profiles/hbm_traffic.json, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs "
                                  "summarised in profiles/ (not measured in this run; all of this layer's tensors fit "
                                  "the 256 MB last-level cache, so these are bytes between L2 and the fabric)",
                "algorithmic_bytes": wl.fused_bytes(L, dom), "avg_launch_ms": dom_ms, "empty_event_pair_ms": pair_ms,
                "launches_timed": "every %dth of the %d timed steps" % (EV, K),
                "hbm_frac_of_8TBs": wl.fused_bytes(L, dom) / (dom_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}

    out = {"metric": "int8 GEMM TOPS + HBM bytes/step, in-hindsight fused vs dynamic 2-pass", "value": value,
           "unit": "TOP/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": wall_ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
           "config": {"workload": "ResNet-style conv3x3 64->64 @56x56, batch 128 (M=401408,K=576,N=64): "
                                  "fwd + dgrad + wgrad with in-hindsight ranges (eta 0.9, both range updates in the last launch), one layer step",
                      "global_batch": 128, "parallelism": "single GPU"},
           "roofline": roofline,
           "per_call_ms_warmup": per_call,
           "per_call_tops_warmup": {n: ops_gemm / (per_call[n] * 1e-3) / 1e12 for n in ("fwd", "dgrad", "wgrad")}}

    # ---- the dynamic two-pass baseline on the same layer -----------------------------------
    if not args.no_extras:
        reps = max(5, min(K, 20))
        dyn_ms = time_calls(torch, lay.dynamic_step, reps)
        fus_ms = time_calls(torch, lay.fused_step, reps)
        fb = sum(wl.fused_bytes(L, o) for o in ("fwd", "dgrad", "wgrad"))
        db = sum(wl.dynamic_bytes(L, o) for o in ("fwd", "dgrad", "wgrad"))
        out["fused_vs_dynamic"] = {
            "fused_ms_per_step_separate_range_update": time_calls(torch, lay.fused_step_separate_update, reps),
            "fused_ms_per_step": fus_ms, "dynamic_ms_per_step": dyn_ms, "speedup": dyn_ms / fus_ms,
            "fwd_fused_ms": time_calls(torch, lay.fwd, reps), "fwd_dynamic_ms": time_calls(torch, lay.dyn_fwd, reps),
            "dgrad_fused_ms": time_calls(torch, lay.dgrad, reps), "dgrad_dynamic_ms": time_calls(torch, lay.dyn_dgrad, reps),
            "algorithmic_hbm_bytes_per_step": {"fused": fb, "dynamic": db, "ratio": db / fb},
            "measured_hbm_bytes_per_step": stored_traffic("step"), "traffic_source": "stored: profiles/hbm_traffic.json"}
        # the same input-gradient GEMM with stochastic rounding in the epilogue
        out["stochastic_rounding"] = {"dgrad_sr_ms": time_calls(torch, lay.dgrad_sr, reps),
                                      "dgrad_nearest_even_ms": out["fused_vs_dynamic"]["dgrad_fused_ms"]}
        lay.upd_y(); lay.upd_g()
        # activations that grow 5 % per iteration (the range lags; eq. (2)-(3) settle at
        # (1 - eta) / (1.05 - eta) = 2/3 of the tensor's width)
        out["range_tracking"] = {"c2_fwd_growth_1.05_per_iter": range_tracking(
            hq, torch, lay, "fwd", [float(X.scale) * 1.05 ** t for t in range(11)], range(11))}

        # ---- other layer shapes of the configurations (same kernels, single launches) ------
        extra = {}
        del lay
        torch.cuda.empty_cache()
        shapes = [("c3_conv3x3_128_b128", wl.c3_layer())] + [(l.name + "_b128", l) for l in wl.c4_layers()]
        for name, Ls in shapes:
            g = wl.rng(9, 0, len(extra))
            Xs = wl.relu6_activation(g, wl.in_shape(Ls)) if name.startswith("c4") else wl.relu_activation(g, wl.in_shape(Ls))
            ly = Layer(hq, torch, wl, Ls, Xs, wl.he_weight(g, Ls), wl.laplace_gradient(g, wl.out_shape(Ls), 1e-3))
            ly.init_ranges()
            row = {}
            for op, f, fd in (("fwd", ly.fwd, ly.dyn_fwd), ("dgrad", ly.dgrad, ly.dyn_dgrad), ("wgrad", ly.wgrad, None)):
                ms = time_calls(torch, f, 10)
                row[op] = {"ms": ms, "tops": 2 * wl.macs(Ls) / (ms * 1e-3) / 1e12,
                           "alg_GBs": wl.fused_bytes(Ls, op) / (ms * 1e-3) / 1e9}
                if fd is not None:
                    dms = time_calls(torch, fd, 10)
                    row[op]["dynamic_ms"] = dms
                    row[op]["dynamic_alg_GBs"] = wl.dynamic_bytes(Ls, op) / (dms * 1e-3) / 1e9
            extra[name] = row
            if name.startswith("c3"):
                # gradients that decay 1 -> 1e-3 over 50 iterations: the range shrinks slower than the tensor
                out["range_tracking"]["c3_dgrad_decay_1e-3_over_50_iters"] = range_tracking(
                    hq, torch, ly, "dgrad", [1e-3 / 127.0 * wl.c3_grad_scale(t) for t in range(50)],
                    (0, 1, 2, 5, 10, 20, 30, 40, 49))
            del ly
            torch.cuda.empty_cache()
        out["other_layers"] = extra
        out["resnet18_step"] = stack_step(hq, torch, wl, wl.resnet18_layers(B=256), "ResNet-18-shaped stack, batch 256 @224x224",
                                          config=5)
        out["resnet18_step"]["measured_hbm_bytes_per_step"] = stored_traffic("resnet18_step")
        out["resnet18_step"]["traffic_source"] = "stored: profiles/hbm_traffic.json (rocprofv3 --pmc over bench.py --stack-only)"
        torch.cuda.empty_cache()
        out["vgg16_step"] = stack_step(hq, torch, wl, wl.vgg16_layers(B=256), "VGG16-shaped stack, batch 256 @64x64", reps=5, warmup=1)
        torch.cuda.empty_cache()
        out["real_tensor_quantizer"] = tensor_quantizer(hq, torch, wl)
        torch.cuda.empty_cache()
        # every launch measured above against both ceilings (single launches, back to back): the
        # larger fraction names the bound; the depthwise stencil is bound by neither (vector ALU)
        rl = []
        fd = out["fused_vs_dynamic"]
        for op in ("fwd", "dgrad"):
            ms = fd[op + "_fused_ms"]
            rl.append({"launch": "config 2 " + op, "ms": ms, "mfma_frac": ops_gemm / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS,
                       "hbm_frac": wl.fused_bytes(L, op) / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
            dms = fd[op + "_dynamic_ms"]
            rl.append({"launch": "config 2 " + op + " (dynamic two-pass)", "ms": dms,
                       "mfma_frac": ops_gemm / (dms * 1e-3) / 1e12 / PEAK_INT8_TOPS,
                       "hbm_frac": wl.dynamic_bytes(L, op) / (dms * 1e-3) / 1e9 / PEAK_HBM_GBS})
        rl.append({"launch": "config 2 wgrad", "ms": dom_ms if dom == "wgrad" else per_call["wgrad"],
                   "mfma_frac": roofline["frac"] if dom == "wgrad" else None,
                   "hbm_frac": roofline["hbm_frac_of_8TBs"] if dom == "wgrad" else None})
        for name, row in extra.items():
            for op, r in row.items():
                rl.append({"launch": name + " " + op, "ms": r["ms"], "mfma_frac": r["tops"] / PEAK_INT8_TOPS,
                           "hbm_frac": r["alg_GBs"] / PEAK_HBM_GBS})
        tq = out["real_tensor_quantizer"]
        rl.append({"launch": "FP32 tensor quantizer, in hindsight", "ms": tq["in_hindsight_ms"], "mfma_frac": None,
                   "hbm_frac": tq["in_hindsight_alg_GBs"] / PEAK_HBM_GBS})
        rl.append({"launch": "FP32 tensor quantizer, dynamic", "ms": tq["dynamic_ms"], "mfma_frac": None,
                   "hbm_frac": tq["dynamic_alg_GBs"] / PEAK_HBM_GBS})
        out["rooflines_all_launches"] = rl

    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = {"read": a.numel(), "write": a.numel()}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, 128)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
