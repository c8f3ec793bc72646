"""Test harness: runs one layer operation through the HIP library (via its C-ABI binding) and
through the CPU oracle on the same seeded inputs.  The two sides meet only here."""
import numpy as np
import torch

import oracle
import paper_2105_04246_amd as hq
import workloads as wl


def hq_problem(L):
    return hq.problem(L.kind, L.B, L.H, L.W, L.C, L.R, L.S, L.stride, L.pad, L.Cout)


def oracle_problem(L):
    return oracle.Problem(L.kind, L.B, L.H, L.W, L.C, L.R, L.S, L.stride, L.pad, L.Cout)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class DevTensor:
    """Quantized tensor on the device: codes + hq_qparams buffer."""
    def __init__(self, qt):
        self.codes = dev(qt.codes)
        self.qp = hq.new_qparams(qt.scale, qt.zero_point)


class DevWeights:
    """Weight-side buffers of one layer, prepared on the device by hq_weight_prepare."""
    def __init__(self, L, W):
        p = hq_problem(L)
        self.W = dev(W.codes)
        self.qp = hq.new_qparams(W.scale, 0)
        self.wsum = torch.empty(L.Cout, dtype=torch.int32, device="cuda")
        self.wdsum = torch.empty(L.C, dtype=torch.int32, device="cuda")
        if L.kind == wl.DEPTHWISE:
            self.Wd = self.W
            hq.hq_weight_prepare(p, self.W, None, self.wsum, self.wdsum)
        else:
            self.Wd = torch.empty(L.C * L.R * L.S * L.Cout, dtype=torch.int8, device="cuda")
            hq.hq_weight_prepare(p, self.W, self.Wd, self.wsum, self.wdsum)


def read_range(r):
    return hq.from_device(r, hq.RANGE)[0]


def read_stats(st):
    """The statistics record with its partial records folded into the leading fields."""
    hq.hq_stats_fold(st)
    rec = hq.from_device(st, hq.STATS)[0]
    assert (rec["part"]["clip_lo"] == 0).all() and (rec["part"]["acc_min"] == np.iinfo(np.int32).max).all()
    return rec


def read_qparams(q):
    return hq.from_device(q, hq.QPARAMS)[0]


def gpu_quantized_op(L, op, A, Wdev, r, st, mode="fused", dyn_mode=hq.HQ_DYN_CURRENT, seed=None):
    """op in {'fwd','dgrad'}; mode 'fused' (in-hindsight static; with a seed: stochastic rounding,
    dgrad only) or 'dynamic' (with a seed: stochastic rounding in its second pass).
    Returns (codes ndarray, qparams record).  Range state / stats stay on the device."""
    p = hq_problem(L)
    shape = wl.out_shape(L) if op == "fwd" else wl.in_shape(L)
    out = torch.empty(shape, dtype=torch.int8, device="cuda")
    outq = hq.new_qparams(0.0, 0)
    Bw, bsum = (Wdev.W, Wdev.wsum) if op == "fwd" else (Wdev.Wd, Wdev.wdsum)
    if mode == "fused" and seed is not None:
        assert op == "dgrad"
        hq.hq_gemm_dgrad_sr(p, A.codes, A.qp, Bw, Wdev.qp, bsum, r, seed, out, outq, st)
    elif mode == "fused":
        f = hq.hq_gemm_fwd if op == "fwd" else hq.hq_gemm_dgrad
        f(p, A.codes, A.qp, Bw, Wdev.qp, bsum, r, out, outq, st)
    else:
        entry = hq.HQ_ENTRY_DYNAMIC_FWD if op == "fwd" else hq.HQ_ENTRY_DYNAMIC_DGRAD
        nbytes = hq.hq_workspace_bytes(entry, p)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        if seed is not None:
            hq.hq_gemm_dynamic_sr(entry, dyn_mode, p, A.codes, A.qp, Bw, Wdev.qp, bsum, r, seed, out, outq, st, ws, nbytes)
        else:
            hq.hq_gemm_dynamic(entry, dyn_mode, p, A.codes, A.qp, Bw, Wdev.qp, bsum, r, out, outq, st, ws, nbytes)
    torch.cuda.synchronize()
    return out.cpu().numpy(), read_qparams(outq)


def gpu_wgrad(L, X, dY):
    p = hq_problem(L)
    nbytes = hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, p)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    dW = torch.empty(wl.w_shape(L), dtype=torch.float32, device="cuda")
    dWa = torch.empty(wl.w_shape(L), dtype=torch.int32, device="cuda")
    hq.hq_gemm_wgrad(p, X.codes, X.qp, dY.codes, dY.qp, dW, dWa, ws, nbytes)
    torch.cuda.synchronize()
    return dW.cpu().numpy(), dWa.cpu().numpy()


def oracle_acc(L, op, A, W):
    p = oracle_problem(L)
    if op == "fwd":
        return oracle.fwd(p, A.codes, A.zero_point, W.codes)
    return oracle.dgrad(p, A.codes, A.zero_point, W.codes)


def assert_stats_equal(gpu_st, ref, a_scale):
    assert int(gpu_st["acc_min"]) == ref["acc_min"] and int(gpu_st["acc_max"]) == ref["acc_max"], \
        (gpu_st, ref["acc_min"], ref["acc_max"])
    assert int(gpu_st["clip_lo"]) == ref["clip_lo"] and int(gpu_st["clip_hi"]) == ref["clip_hi"], \
        (gpu_st, ref["clip_lo"], ref["clip_hi"])
    assert int(gpu_st["count"]) == ref["count"]
    assert np.float32(gpu_st["acc_scale"]) == np.float32(a_scale)


def assert_range_close(gpu_r, ref_r, rel=1e-6):
    """fp32 range state: within `rel` relative (the tolerance the benchmark spec fixes)."""
    for f in ("qmin", "qmax"):
        a, b = float(gpu_r[f]), float(getattr(ref_r, f))
        assert abs(a - b) <= rel * max(abs(a), abs(b)), (f, a, b)
    a, b = float(gpu_r["scale"]), float(ref_r.scale)
    assert abs(a - b) <= rel * abs(b), ("scale", a, b)
    assert int(gpu_r["zero_point"]) == ref_r.zero_point
    assert int(gpu_r["initialized"]) == ref_r.initialized


class TensorTrack:
    """One quantized output tensor followed over iterations on both sides: device range
    state + stats, and the oracle's Range."""
    def __init__(self, eta=0.9, symmetric=False, state=None, bits=8):
        """state: (range record, statistics record) views into caller-owned arrays, for the batched update."""
        self.r, self.st = state if state is not None else (hq.new_range(eta, symmetric, bits=bits), hq.new_stats(1))
        self.ref = oracle.Range.new(eta, symmetric, bits)

    def step(self, L, op, A_q, W_q, A_dev, W_dev, check=True, update=True, seed=None):
        """Runs iteration t on both sides (dynamic init at t=0, fused afterwards), compares
        codes, quantizer, statistics and the updated range.  Returns (gpu codes, oracle dict)."""
        a_scale = oracle.acc_scale(A_q.scale, W_q.scale)
        c = oracle_acc(L, op, A_q, W_q)
        first = not self.ref.initialized
        ref = oracle.in_hindsight_step(c, a_scale, self.ref, seed)
        codes, qp = gpu_quantized_op(L, op, A_dev, W_dev, self.r, self.st, "dynamic" if first else "fused",
                                     seed=None if first else seed)
        st = read_stats(self.st)
        if update:
            hq.hq_range_update(self.r, self.st)
        torch.cuda.synchronize()
        if check:
            assert_stats_equal(st, ref, a_scale)
            assert np.float32(qp["scale"]) == ref["scale"] and int(qp["zero_point"]) == ref["zero_point"], (qp, ref["scale"], ref["zero_point"])
            assert np.array_equal(codes, ref["codes"]), "int8 outputs differ in %d places" % int((codes != ref["codes"]).sum())
        if check and update:
            assert_range_close(read_range(self.r), self.ref)
            st2 = read_stats(self.st)
            assert int(st2["count"]) == 0 and int(st2["acc_min"]) == 2**31 - 1 and int(st2["acc_max"]) == -2**31
        return codes, ref
