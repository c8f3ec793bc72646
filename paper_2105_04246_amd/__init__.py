"""Python binding of the hq C-ABI library (include/hq.h): argument marshalling only.

Every function below has the name and argument order of its C counterpart and passes
device pointers of torch tensors straight through; all arithmetic of the layer path runs
in the HIP kernels of ``libhq.so``.  PyTorch is used for device memory and streams only.
There is no CPU fallback: if the library cannot be loaded, importing the symbols fails.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

HQ_OK, HQ_E_BADARG, HQ_E_BADSHAPE, HQ_E_WORKSPACE, HQ_E_HIP = 0, -1, -2, -3, -4
HQ_LINEAR, HQ_CONV2D, HQ_DEPTHWISE = 0, 1, 2
HQ_ENTRY_FWD, HQ_ENTRY_DGRAD, HQ_ENTRY_WGRAD, HQ_ENTRY_DYNAMIC_FWD, HQ_ENTRY_DYNAMIC_DGRAD = 0, 1, 2, 3, 4
HQ_DYN_CURRENT, HQ_DYN_RUNNING = 0, 1
HQ_STATIC_SCRATCH_BYTES = 64 << 20

# Host views of the device structs (little-endian, same field order as include/hq.h).
QPARAMS = np.dtype([("scale", "<f4"), ("zero_point", "<i4")])
RANGE = np.dtype([("qmin", "<f4"), ("qmax", "<f4"), ("eta", "<f4"), ("qlo", "<i4"), ("qhi", "<i4"),
                  ("symmetric", "<i4"), ("initialized", "<i4"), ("scale", "<f4"), ("zero_point", "<i4")])
STATS_PARTS = 64
STATS_PART = np.dtype([("acc_min", "<i4"), ("acc_max", "<i4"), ("clip_lo", "<u8"), ("clip_hi", "<u8"),
                       ("pad", "u1", (104,))])
STATS = np.dtype([("acc_min", "<i4"), ("acc_max", "<i4"), ("acc_scale", "<f4"), ("fp32_keys", "<u4"),
                  ("clip_lo", "<u8"), ("clip_hi", "<u8"), ("count", "<u8"), ("pad", "u1", (88,)),
                  ("part", STATS_PART, (STATS_PARTS,))])
SATURATION = np.dtype([("alpha_min", "<f4"), ("alpha_max", "<f4"), ("alpha_target", "<f4"), ("tau", "<i4"), ("streak", "<i4")])
assert QPARAMS.itemsize == 8 and RANGE.itemsize == 36 and STATS_PART.itemsize == 128
assert STATS.itemsize == 128 * (1 + STATS_PARTS)


class hq_problem(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "B", "H", "W", "C", "R", "S", "stride", "pad", "Cout")]

    def out_hw(self):
        return ((self.H + 2 * self.pad - self.R) // self.stride + 1,
                (self.W + 2 * self.pad - self.S) // self.stride + 1)


class HqError(RuntimeError):
    def __init__(self, fn, code):
        self.code = code
        super().__init__("%s: %s (%d)" % (fn, lib().hq_error_string(code).decode(), code))


_lib = None
EXPORTS = ("hq_workspace_bytes", "hq_gemm_fwd", "hq_gemm_dgrad", "hq_gemm_dgrad_sr", "hq_gemm_wgrad", "hq_gemm_wgrad_static", "hq_gemm_wgrad_update", "hq_range_update",
           "hq_range_update_batch", "hq_range_update_saturation",
           "hq_gemm_dynamic", "hq_gemm_dynamic_sr", "hq_stats_reset", "hq_stats_fold", "hq_weight_prepare", "hq_weight_quantize", "hq_tensor_quantize", "hq_tensor_quantize_sr", "hq_tensor_quantize_dynamic",
           "hq_probe_mfma_rate",
           "hq_error_string")


def lib():
    """Loads libhq.so (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        vp, PP = C.c_void_p, C.POINTER(hq_problem)
        L.hq_error_string.restype = C.c_char_p
        L.hq_error_string.argtypes = [C.c_int]
        L.hq_workspace_bytes.restype = C.c_size_t
        L.hq_workspace_bytes.argtypes = [C.c_int32, PP]
        L.hq_gemm_fwd.argtypes = [PP] + [vp] * 10
        L.hq_gemm_dgrad.argtypes = [PP] + [vp] * 10
        L.hq_gemm_dgrad_sr.argtypes = [PP] + [vp] * 6 + [C.c_uint64] + [vp] * 4
        L.hq_gemm_wgrad.argtypes = [PP, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.hq_gemm_wgrad_static.argtypes = [PP, vp, vp, vp, vp, vp, vp, vp]
        L.hq_gemm_wgrad_update.argtypes = [PP, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, vp, C.c_int32, vp]
        L.hq_range_update.argtypes = [vp, vp, vp]
        L.hq_range_update_batch.argtypes = [vp, vp, C.c_int32, vp]
        L.hq_range_update_saturation.argtypes = [vp, vp, vp, C.c_int32, vp]
        L.hq_gemm_dynamic.argtypes = [C.c_int32, C.c_int32, PP] + [vp] * 10 + [C.c_size_t, vp]
        L.hq_gemm_dynamic_sr.argtypes = [C.c_int32, C.c_int32, PP] + [vp] * 6 + [C.c_uint64] + [vp] * 4 + [C.c_size_t, vp]
        L.hq_stats_reset.argtypes = [vp, C.c_int32, vp]
        L.hq_stats_fold.argtypes = [vp, C.c_int32, vp]
        L.hq_weight_prepare.argtypes = [PP, vp, vp, vp, vp, vp]
        L.hq_probe_mfma_rate.argtypes = [C.c_int32, C.c_int32, vp, vp]
        L.hq_weight_quantize.argtypes = [vp, C.c_size_t, vp, vp, vp]
        L.hq_tensor_quantize.argtypes = [vp, C.c_size_t, vp, vp, vp, vp, vp]
        L.hq_tensor_quantize_sr.argtypes = [vp, C.c_size_t, vp, C.c_uint64, vp, vp, vp, vp]
        L.hq_tensor_quantize_dynamic.argtypes = [C.c_int32, vp, C.c_size_t, vp, vp, vp, vp, vp]
        for f in EXPORTS[1:-1]:
            getattr(L, f).restype = C.c_int
        _lib = L
    return _lib


def _ptr(t):
    """Device pointer of a torch tensor (None -> NULL).  A raw int is passed through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(fn, rc):
    if rc != HQ_OK:
        raise HqError(fn, rc)


def hq_workspace_bytes(entry, p):
    return int(lib().hq_workspace_bytes(entry, C.byref(p)))


def hq_gemm_fwd(p, X, xq, W, wq, wsum, yr, Y, yq, st, stream=None):
    _check("hq_gemm_fwd", lib().hq_gemm_fwd(C.byref(p), _ptr(X), _ptr(xq), _ptr(W), _ptr(wq), _ptr(wsum),
                                            _ptr(yr), _ptr(Y), _ptr(yq), _ptr(st), _stream(stream)))


def hq_gemm_dgrad(p, dY, gq, Wd, wq, wdsum, gr, dX, dxq, st, stream=None):
    _check("hq_gemm_dgrad", lib().hq_gemm_dgrad(C.byref(p), _ptr(dY), _ptr(gq), _ptr(Wd), _ptr(wq), _ptr(wdsum),
                                                _ptr(gr), _ptr(dX), _ptr(dxq), _ptr(st), _stream(stream)))


def hq_gemm_dgrad_sr(p, dY, gq, Wd, wq, wdsum, gr, seed, dX, dxq, st, stream=None):
    _check("hq_gemm_dgrad_sr", lib().hq_gemm_dgrad_sr(C.byref(p), _ptr(dY), _ptr(gq), _ptr(Wd), _ptr(wq), _ptr(wdsum),
                                                    _ptr(gr), int(seed), _ptr(dX), _ptr(dxq), _ptr(st), _stream(stream)))


def hq_gemm_wgrad(p, X, xq, dY, gq, dW, dW_acc, ws, ws_bytes, stream=None):
    _check("hq_gemm_wgrad", lib().hq_gemm_wgrad(C.byref(p), _ptr(X), _ptr(xq), _ptr(dY), _ptr(gq), _ptr(dW),
                                                _ptr(dW_acc), _ptr(ws), ws_bytes, _stream(stream)))


def hq_gemm_wgrad_static(p, X, xq, dY, gq, dW, dW_acc, stream=None):
    _check("hq_gemm_wgrad_static", lib().hq_gemm_wgrad_static(C.byref(p), _ptr(X), _ptr(xq), _ptr(dY), _ptr(gq), _ptr(dW),
                                                              _ptr(dW_acc), _stream(stream)))


def hq_gemm_wgrad_update(p, X, xq, dY, gq, dW, dW_acc, ws, ws_bytes, r, st, n, stream=None):
    _check("hq_gemm_wgrad_update", lib().hq_gemm_wgrad_update(C.byref(p), _ptr(X), _ptr(xq), _ptr(dY), _ptr(gq), _ptr(dW),
                                                              _ptr(dW_acc), _ptr(ws), ws_bytes, _ptr(r), _ptr(st), n,
                                                              _stream(stream)))


def hq_range_update(r, st, stream=None):
    _check("hq_range_update", lib().hq_range_update(_ptr(r), _ptr(st), _stream(stream)))


def hq_range_update_batch(r, st, n, stream=None):
    _check("hq_range_update_batch", lib().hq_range_update_batch(_ptr(r), _ptr(st), n, _stream(stream)))


def hq_range_update_saturation(r, st, sat, n=1, stream=None):
    _check("hq_range_update_saturation", lib().hq_range_update_saturation(_ptr(r), _ptr(st), _ptr(sat), n, _stream(stream)))


def hq_gemm_dynamic(op, mode, p, A, aq, Bw, bq, bsum, r, out, outq, st, ws, ws_bytes, stream=None):
    _check("hq_gemm_dynamic", lib().hq_gemm_dynamic(op, mode, C.byref(p), _ptr(A), _ptr(aq), _ptr(Bw), _ptr(bq),
                                                    _ptr(bsum), _ptr(r), _ptr(out), _ptr(outq), _ptr(st),
                                                    _ptr(ws), ws_bytes, _stream(stream)))


def hq_gemm_dynamic_sr(op, mode, p, A, aq, Bw, bq, bsum, r, seed, out, outq, st, ws, ws_bytes, stream=None):
    _check("hq_gemm_dynamic_sr", lib().hq_gemm_dynamic_sr(op, mode, C.byref(p), _ptr(A), _ptr(aq), _ptr(Bw), _ptr(bq),
                                                          _ptr(bsum), _ptr(r), int(seed), _ptr(out), _ptr(outq), _ptr(st),
                                                          _ptr(ws), ws_bytes, _stream(stream)))


def hq_stats_reset(st, n=1, stream=None):
    _check("hq_stats_reset", lib().hq_stats_reset(_ptr(st), n, _stream(stream)))


def hq_stats_fold(st, n=1, stream=None):
    _check("hq_stats_fold", lib().hq_stats_fold(_ptr(st), n, _stream(stream)))


def hq_weight_prepare(p, W, Wd, wsum, wdsum, stream=None):
    _check("hq_weight_prepare", lib().hq_weight_prepare(C.byref(p), _ptr(W), _ptr(Wd), _ptr(wsum), _ptr(wdsum),
                                                        _stream(stream)))


def hq_weight_quantize(Wf, n, Wq, wq, stream=None):
    _check("hq_weight_quantize", lib().hq_weight_quantize(_ptr(Wf), n, _ptr(Wq), _ptr(wq), _stream(stream)))


def hq_tensor_quantize(X, n, r, Q, q_out, st, stream=None):
    _check("hq_tensor_quantize", lib().hq_tensor_quantize(_ptr(X), n, _ptr(r), _ptr(Q), _ptr(q_out), _ptr(st),
                                                          _stream(stream)))


def hq_tensor_quantize_sr(X, n, r, seed, Q, q_out, st, stream=None):
    _check("hq_tensor_quantize_sr", lib().hq_tensor_quantize_sr(_ptr(X), n, _ptr(r), int(seed), _ptr(Q), _ptr(q_out),
                                                                _ptr(st), _stream(stream)))


def hq_tensor_quantize_dynamic(mode, X, n, r, Q, q_out, st, stream=None):
    _check("hq_tensor_quantize_dynamic", lib().hq_tensor_quantize_dynamic(mode, _ptr(X), n, _ptr(r), _ptr(Q),
                                                                          _ptr(q_out), _ptr(st), _stream(stream)))


def hq_probe_mfma_rate(blocks, iters, sink, stream=None):
    """Launches the register-only MFMA loop; returns the int8 operations it issues."""
    _check("hq_probe_mfma_rate", lib().hq_probe_mfma_rate(blocks, iters, _ptr(sink), _stream(stream)))
    return blocks * 4 * iters * 8 * 2 * 32 ** 3


# ---------------------------------------------------------------------------
# Marshalling helpers: host records <-> device bytes.  No arithmetic.
# ---------------------------------------------------------------------------

def problem(kind, B, H, W, Cin, R, S, stride, pad, Cout):
    return hq_problem(kind, B, H, W, Cin, R, S, stride, pad, Cout)


def to_device(rec, device="cuda"):
    """Copies a NumPy record (QPARAMS / RANGE / STATS, scalar or array) into a new device byte buffer."""
    import torch
    host = torch.from_numpy(np.ascontiguousarray(rec).reshape(-1).view(np.uint8).copy())
    return host.to(device)


def from_device(t, dtype):
    """Copies a device byte buffer back and views it as records of `dtype` (synchronises)."""
    return t.cpu().numpy().view(dtype)


def new_qparams(scale, zero_point, device="cuda"):
    rec = np.zeros((), QPARAMS)
    rec["scale"], rec["zero_point"] = scale, zero_point
    return to_device(rec, device)


def new_range(eta=0.9, symmetric=False, device="cuda", bits=8):
    """Uninitialised range state on a b-bit grid in 8-bit storage (8 bits: asymmetric -128..127,
    symmetric -127..127; fewer bits: -2^(b-1)..2^(b-1)-1, symmetric without the lowest code)."""
    if not 2 <= bits <= 8:
        raise ValueError("bits must be 2..8")
    top = 2 ** (bits - 1) - 1
    rec = np.zeros((), RANGE)
    rec["eta"], rec["symmetric"] = eta, int(symmetric)
    rec["qlo"], rec["qhi"] = (-top, top) if symmetric else (-top - 1, top)
    rec["scale"] = 1.0
    return to_device(rec, device)


def new_saturation(alpha_min=1e-5, alpha_max=1e-3, alpha_target=1e-4, tau=2, n=1, device="cuda"):
    """n saturation-estimator states (hq_saturation) with the same settings, streak 0."""
    rec = np.zeros(n, SATURATION)
    rec["alpha_min"], rec["alpha_max"], rec["alpha_target"], rec["tau"] = alpha_min, alpha_max, alpha_target, tau
    return to_device(rec, device)


def new_ranges(symmetric_flags, eta=0.9, device="cuda"):
    """An array of uninitialised range states (one per flag) in one device buffer, for
    hq_range_update_batch; record i starts at byte i * RANGE.itemsize."""
    rec = np.zeros(len(symmetric_flags), RANGE)
    for i, sym in enumerate(symmetric_flags):
        rec[i]["eta"], rec[i]["symmetric"] = eta, int(sym)
        rec[i]["qlo"], rec[i]["qhi"] = (-127, 127) if sym else (-128, 127)
        rec[i]["scale"] = 1.0
    return to_device(rec, device)


def new_stats(n=1, device="cuda"):
    import torch
    st = torch.empty(n * STATS.itemsize, dtype=torch.uint8, device=device)
    hq_stats_reset(st, n)
    return st
