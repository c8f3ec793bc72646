"""CPU oracle of the in-hindsight quantized-training layer path (test infrastructure).

Thin ctypes front of ``hq_oracle.c`` plus the few lines that string its steps
together in the order the paper gives them (Sec. 3.2 static / dynamic
quantization, Sec. 4.1 in-hindsight min-max).  Only tests, the smoke check and
the benchmark's CPU-baseline leg may import this package; the HIP library never
does, and this package imports nothing from it.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class Problem(C.Structure):
    """Layer shape.  kind: 0 linear, 1 conv2d, 2 depthwise conv2d."""
    _fields_ = [(n, C.c_int32) for n in
                ("kind", "B", "H", "W", "C", "R", "S", "stride", "pad", "Cout")]

    @staticmethod
    def linear(M, K, N):
        return Problem(0, M, 1, 1, K, 1, 1, 1, 0, N)

    @staticmethod
    def conv(B, H, W, Cin, Cout, R, S, stride, pad):
        return Problem(1, B, H, W, Cin, R, S, stride, pad, Cout)

    @staticmethod
    def depthwise(B, H, W, Ch, R, S, stride, pad):
        return Problem(2, B, H, W, Ch, R, S, stride, pad, Ch)

    def out_hw(self):
        oh, ow = C.c_int32(), C.c_int32()
        lib().hqo_out_hw(C.byref(self), C.byref(oh), C.byref(ow))
        return oh.value, ow.value

    def out_shape(self):
        oh, ow = self.out_hw()
        return (self.B, oh, ow, self.Cout)

    def in_shape(self):
        return (self.B, self.H, self.W, self.C)

    def w_shape(self):
        if self.kind == 2:
            return (self.R, self.S, self.C)
        return (self.Cout, self.R, self.S, self.C)


class Range(C.Structure):
    """State of one quantizer: eq. (2)-(3) range, momentum, grid, derived (scale, zero point)."""
    _fields_ = [("qmin", C.c_float), ("qmax", C.c_float), ("eta", C.c_float),
                ("qlo", C.c_int32), ("qhi", C.c_int32), ("symmetric", C.c_int32),
                ("initialized", C.c_int32), ("scale", C.c_float), ("zero_point", C.c_int32)]

    @staticmethod
    def new(eta=0.9, symmetric=False, bits=8):
        """b-bit grid held in 8-bit storage: -2^(b-1)..2^(b-1)-1, symmetric without its lowest code."""
        assert 2 <= bits <= 8
        top = 2 ** (bits - 1) - 1
        if symmetric:
            return Range(0.0, 0.0, eta, -top, top, 1, 0, 1.0, 0)
        return Range(0.0, 0.0, eta, -top - 1, top, 0, 0, 1.0, 0)


class Saturation(C.Structure):
    """State of the saturation-driven estimator of one quantizer (band, target, patience, streak)."""
    _fields_ = [("alpha_min", C.c_float), ("alpha_max", C.c_float), ("alpha_target", C.c_float),
                ("tau", C.c_int32), ("streak", C.c_int32)]

    @staticmethod
    def new(alpha_min=1e-5, alpha_max=1e-3, alpha_target=1e-4, tau=2):
        return Saturation(alpha_min, alpha_max, alpha_target, tau, 0)


def lib():
    global _lib
    if _lib is None:
        if os.environ.get("HQ_ORACLE_SANITIZE") == "1":       # the instrumented build, see build_sanitized.py
            from . import build_sanitized
            path = build_sanitized.build(force=False)
        else:
            path = _build.build(force=False)
        L = C.CDLL(path)
        i8p, i32p, i64p, f32p = (C.POINTER(t) for t in (C.c_int8, C.c_int32, C.c_int64, C.c_float))
        PP = C.POINTER(Problem)
        L.hqo_num_threads.restype = C.c_int
        L.hqo_out_hw.argtypes = [PP, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.hqo_fwd.argtypes = [PP, i8p, C.c_int, i8p, i32p]
        L.hqo_fwd_rows.argtypes = [PP, i8p, C.c_int, i8p, i64p, C.c_int64, i32p]
        L.hqo_dgrad.argtypes = [PP, i8p, C.c_int, i8p, i32p]
        L.hqo_dgrad_rows.argtypes = [PP, i8p, C.c_int, i8p, i64p, C.c_int64, i32p]
        L.hqo_wgrad.argtypes = [PP, i8p, C.c_int, i8p, C.c_int, i32p]
        L.hqo_minmax.argtypes = [i32p, C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.hqo_qparams.argtypes = [C.c_float, C.c_float, C.c_int, C.c_int, C.c_int,
                                  C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        L.hqo_requant.argtypes = [i32p, C.c_int64, C.c_float, C.c_float, C.c_int, C.c_int, C.c_int,
                                  i8p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.hqo_requant_sr.argtypes = [i32p, C.c_int64, C.c_float, C.c_float, C.c_int, C.c_int, C.c_int,
                                     C.c_uint64, C.c_uint64, i8p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.hqo_sr_bits.argtypes = [C.c_uint64, C.c_uint64]
        L.hqo_sr_bits.restype = C.c_uint32
        L.hqo_range_update.argtypes = [C.POINTER(Range), C.c_int32, C.c_int32, C.c_float]
        L.hqo_ln_fixed.argtypes = [C.c_float]
        L.hqo_ln_fixed.restype = C.c_float
        L.hqo_range_update_saturation.argtypes = [C.POINTER(Range), C.POINTER(Saturation), C.c_uint64, C.c_uint64,
                                                  C.c_uint64, C.c_int32, C.c_int32, C.c_float]
        L.hqo_wgrad_scale.argtypes = [i32p, C.c_int64, C.c_float, C.c_float, f32p]
        L.hqo_quantize_weights.argtypes = [f32p, C.c_int64, i8p, f32p]
        L.hqo_range_update_real.argtypes = [C.POINTER(Range), C.c_float, C.c_float]
        L.hqo_quantize_tensor_sr.argtypes = [f32p, C.c_int64, C.c_float, C.c_int, C.c_int, C.c_int, C.c_uint64, i8p,
                                             C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), f32p, f32p]
        L.hqo_quantize_tensor.argtypes = [f32p, C.c_int64, C.c_float, C.c_int, C.c_int, C.c_int, i8p,
                                          C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), f32p, f32p]
        for f in ("hqo_fwd", "hqo_fwd_rows", "hqo_dgrad", "hqo_dgrad_rows", "hqo_wgrad"):
            getattr(L, f).restype = C.c_int
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _chk(a, dtype, shape=None):
    assert a.dtype == dtype and a.flags.c_contiguous, (a.dtype, a.flags)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def num_threads():
    return lib().hqo_num_threads()


def fwd(p, X, zx, W):
    """Zero-point-free forward accumulator, int32 [B,OH,OW,Cout] (Sec. 3.1)."""
    _chk(X, np.int8, p.in_shape()); _chk(W, np.int8, p.w_shape())
    out = np.empty(p.out_shape(), np.int32)
    bad = lib().hqo_fwd(C.byref(p), _p(X, C.c_int8), int(zx), _p(W, C.c_int8), _p(out, C.c_int32))
    assert bad == 0, "accumulator does not fit 32 bits"
    return out


def fwd_rows(p, X, zx, W, rows):
    _chk(X, np.int8, p.in_shape()); _chk(W, np.int8, p.w_shape())
    rows = np.ascontiguousarray(rows, np.int64)
    out = np.empty((len(rows), p.Cout), np.int32)
    bad = lib().hqo_fwd_rows(C.byref(p), _p(X, C.c_int8), int(zx), _p(W, C.c_int8),
                             _p(rows, C.c_int64), len(rows), _p(out, C.c_int32))
    assert bad == 0
    return out


def dgrad(p, dY, zg, W):
    """Zero-point-free input-gradient accumulator, int32 [B,H,W,C] (Sec. 3.1)."""
    _chk(dY, np.int8, p.out_shape()); _chk(W, np.int8, p.w_shape())
    out = np.empty(p.in_shape(), np.int32)
    bad = lib().hqo_dgrad(C.byref(p), _p(dY, C.c_int8), int(zg), _p(W, C.c_int8), _p(out, C.c_int32))
    assert bad == 0
    return out


def dgrad_rows(p, dY, zg, W, rows):
    _chk(dY, np.int8, p.out_shape()); _chk(W, np.int8, p.w_shape())
    rows = np.ascontiguousarray(rows, np.int64)
    out = np.empty((len(rows), p.C), np.int32)
    bad = lib().hqo_dgrad_rows(C.byref(p), _p(dY, C.c_int8), int(zg), _p(W, C.c_int8),
                               _p(rows, C.c_int64), len(rows), _p(out, C.c_int32))
    assert bad == 0
    return out


def wgrad(p, X, zx, dY, zg):
    """Zero-point-free weight-gradient accumulator, int32, shaped like the weights (Sec. 3.1)."""
    _chk(X, np.int8, p.in_shape()); _chk(dY, np.int8, p.out_shape())
    out = np.empty(p.w_shape(), np.int32)
    bad = lib().hqo_wgrad(C.byref(p), _p(X, C.c_int8), int(zx), _p(dY, C.c_int8), int(zg),
                          _p(out, C.c_int32))
    assert bad == 0
    return out


def minmax(c):
    """eq. (1) over the accumulator output."""
    c = np.ascontiguousarray(c, np.int32)
    mn, mx = C.c_int32(), C.c_int32()
    lib().hqo_minmax(_p(c, C.c_int32), c.size, C.byref(mn), C.byref(mx))
    return mn.value, mx.value


def qparams(qmin, qmax, symmetric, qlo, qhi):
    s, z = C.c_float(), C.c_int32()
    lib().hqo_qparams(float(qmin), float(qmax), int(symmetric), int(qlo), int(qhi), C.byref(s), C.byref(z))
    return np.float32(s.value), z.value


def requant(c, acc_scale, s_y, z_y, qlo, qhi):
    """Static quantization of accumulator outputs; returns (codes, clip_lo, clip_hi)."""
    c = np.ascontiguousarray(c, np.int32)
    out = np.empty(c.shape, np.int8)
    lo, hi = C.c_uint64(), C.c_uint64()
    lib().hqo_requant(_p(c, C.c_int32), c.size, float(acc_scale), float(s_y), int(z_y), int(qlo), int(qhi),
                      _p(out, C.c_int8), C.byref(lo), C.byref(hi))
    return out, lo.value, hi.value


def sr_bits(idx, seed):
    """The 32 random bits stochastic rounding draws for element ``idx`` under ``seed``."""
    return int(lib().hqo_sr_bits(int(idx), int(seed)))


def requant_stochastic(c, acc_scale, s_y, z_y, qlo, qhi, seed, idx0=0):
    """Static quantization with stochastic rounding (Sec. 5, experimental setup); element i of
    the flattened tensor draws its random bits from (idx0 + i, seed).  Returns (codes, clip_lo, clip_hi)."""
    c = np.ascontiguousarray(c, np.int32)
    out = np.empty(c.shape, np.int8)
    lo, hi = C.c_uint64(), C.c_uint64()
    lib().hqo_requant_sr(_p(c, C.c_int32), c.size, float(acc_scale), float(s_y), int(z_y), int(qlo), int(qhi),
                         int(idx0), int(seed), _p(out, C.c_int8), C.byref(lo), C.byref(hi))
    return out, lo.value, hi.value


def range_update(r, acc_min, acc_max, acc_scale):
    """eq. (2)-(3) in place on ``r``; the first call sets q^0."""
    lib().hqo_range_update(C.byref(r), int(acc_min), int(acc_max), float(acc_scale))
    return r


def ln_fixed(x):
    """The fixed-sequence fp32 logarithm the saturation-driven update uses."""
    return np.float32(lib().hqo_ln_fixed(float(np.float32(x))))


def range_update_saturation(r, sat, out, acc_scale):
    """Saturation-driven update in place on ``r`` / ``sat`` from the statistics ``out`` of the tensor
    just quantized (a dict as returned by quantize_static / quantize_dynamic)."""
    lib().hqo_range_update_saturation(C.byref(r), C.byref(sat), int(out["clip_lo"]), int(out["clip_hi"]),
                                      int(out["count"]), int(out["acc_min"]), int(out["acc_max"]), float(acc_scale))
    return r


def saturation_step(c, a_scale, r, sat, seed=None):
    """One iteration under the saturation-driven estimator: the first batch is quantized dynamically
    and sets q^0 (Sec. 4.1); later ones statically with the range in ``r``.  In both cases the clip
    counts of this batch then decide whether the range moves (the first batch clips nothing, so it
    counts as one iteration below the band), the same order of steps as in_hindsight_step."""
    if not r.initialized:
        out = quantize_dynamic(c, a_scale, r.symmetric, r.qlo, r.qhi)
        range_update(r, out["acc_min"], out["acc_max"], a_scale)      # sets q^0
    else:
        out = quantize_static(c, a_scale, r, seed)
    range_update_saturation(r, sat, out, a_scale)
    return out


def range_update_real(r, gmin, gmax):
    """eq. (2)-(3) in place on ``r`` from a tensor's minimum and maximum in real units."""
    lib().hqo_range_update_real(C.byref(r), float(np.float32(gmin)), float(np.float32(gmax)))
    return r


def quantize_tensor(x, scale, zero_point, qlo, qhi, seed=None):
    """Static quantization of a real-valued tensor with a given quantizer (Sec. 3.2); with a
    seed, stochastic rounding.  Returns dict(codes, clip_lo, clip_hi, min, max, count)."""
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.int8)
    lo, hi = C.c_uint64(), C.c_uint64()
    mn, mx = C.c_float(), C.c_float()
    if seed is None:
        lib().hqo_quantize_tensor(_p(x, C.c_float), x.size, float(scale), int(zero_point), int(qlo), int(qhi),
                                  _p(out, C.c_int8), C.byref(lo), C.byref(hi), C.byref(mn), C.byref(mx))
    else:
        lib().hqo_quantize_tensor_sr(_p(x, C.c_float), x.size, float(scale), int(zero_point), int(qlo), int(qhi),
                                     int(seed), _p(out, C.c_int8), C.byref(lo), C.byref(hi), C.byref(mn), C.byref(mx))
    return dict(codes=out, clip_lo=lo.value, clip_hi=hi.value, min=np.float32(mn.value), max=np.float32(mx.value),
                count=x.size)


def tensor_step(x, r, mode="hindsight", seed=None):
    """One iteration for a real-valued tensor with range state ``r``.
    "hindsight": Sec. 4.1 -- the first batch is quantized with its own min-max, which becomes q^0;
    later batches with the pre-computed q^t; the tensor's min-max then moves the range (eq. (2)-(3)).
    "current": eq. (1), every batch with its own min-max (r only takes q^0 and the updates).
    "running": the range is first moved by eq. (2)-(3) with this tensor, then used (Sec. 4.1).
    A seed selects stochastic rounding on the in-hindsight (static) iterations."""
    x = np.ascontiguousarray(x, np.float32)
    gmin, gmax = x.min(), x.max()
    if mode == "running":
        range_update_real(r, gmin, gmax)
        out = quantize_tensor(x, r.scale, r.zero_point, r.qlo, r.qhi)
        out.update(scale=np.float32(r.scale), zero_point=r.zero_point)
        return out
    if mode == "current" or not r.initialized:
        if not r.initialized:
            range_update_real(r, gmin, gmax)                           # sets q^0
        s, z = qparams(gmin, gmax, r.symmetric, r.qlo, r.qhi)
        seed = None                                                    # the dynamic passes round to nearest
    else:
        s, z = np.float32(r.scale), r.zero_point
    out = quantize_tensor(x, s, z, r.qlo, r.qhi, seed)
    out.update(scale=np.float32(s), zero_point=int(z))
    range_update_real(r, gmin, gmax)                                   # q^{t+1}
    return out


def quantize_weights(w):
    """Q_W with the current min-max of the tensor (Sec. 3.1; Sec. 5): returns (codes, scale);
    symmetric grid -127..127, zero point 0."""
    w = np.ascontiguousarray(w, np.float32)
    out = np.empty(w.shape, np.int8)
    s = C.c_float()
    lib().hqo_quantize_weights(_p(w, C.c_float), w.size, _p(out, C.c_int8), C.byref(s))
    return out, np.float32(s.value)


def wgrad_scale(c, sx, sg):
    c = np.ascontiguousarray(c, np.int32)
    out = np.empty(c.shape, np.float32)
    lib().hqo_wgrad_scale(_p(c, C.c_int32), c.size, float(sx), float(sg), _p(out, C.c_float))
    return out


def acc_scale(sa, sb):
    """Real value of one accumulator unit: the fp32 product of the operand scales."""
    return np.float32(np.float32(sa) * np.float32(sb))


# ---------------------------------------------------------------------------
# The two ways of quantizing an accumulator output (Sec. 3.2) and the
# in-hindsight step built on the static one (Sec. 4.1).
# ---------------------------------------------------------------------------

def quantize_static(c, a_scale, r, seed=None):
    """Static quantization with the pre-computed range held in ``r`` (step 1 of Sec. 4);
    the statistics of the current tensor are gathered on the side (step 2).  With a ``seed``
    the rounding is stochastic (gradients, Sec. 5), otherwise to nearest even.
    Returns dict(codes, scale, zero_point, acc_min, acc_max, clip_lo, clip_hi, count)."""
    mn, mx = minmax(c)
    if seed is None:
        codes, lo, hi = requant(c, a_scale, r.scale, r.zero_point, r.qlo, r.qhi)
    else:
        codes, lo, hi = requant_stochastic(c, a_scale, r.scale, r.zero_point, r.qlo, r.qhi, seed)
    return dict(codes=codes, scale=np.float32(r.scale), zero_point=r.zero_point,
                acc_min=mn, acc_max=mx, clip_lo=lo, clip_hi=hi, count=c.size)


def quantize_dynamic(c, a_scale, symmetric, qlo, qhi, seed=None):
    """Dynamic quantization: the range is the min-max of the tensor itself, eq. (1); with a seed,
    stochastic rounding."""
    mn, mx = minmax(c)
    gmin = np.float32(a_scale) * np.float32(mn)
    gmax = np.float32(a_scale) * np.float32(mx)
    s, z = qparams(gmin, gmax, symmetric, qlo, qhi)
    if seed is None:
        codes, lo, hi = requant(c, a_scale, s, z, qlo, qhi)
    else:
        codes, lo, hi = requant_stochastic(c, a_scale, s, z, qlo, qhi, seed)
    return dict(codes=codes, scale=s, zero_point=z, acc_min=mn, acc_max=mx,
                clip_lo=lo, clip_hi=hi, count=c.size)


def in_hindsight_step(c, a_scale, r, seed=None):
    """One iteration of in-hindsight min-max for one tensor (Sec. 4.1).

    t = 0 (``r`` not initialised): the range of the first batch is its own min-max,
    so the tensor is quantized dynamically and q^0 is set from it.  Later iterations
    quantize statically with q^t.  In both cases the statistics of this tensor then
    move the range to q^{t+1} by eq. (2)-(3)."""
    if not r.initialized:
        out = quantize_dynamic(c, a_scale, r.symmetric, r.qlo, r.qhi)
        range_update(r, out["acc_min"], out["acc_max"], a_scale)      # sets q^0
    else:
        out = quantize_static(c, a_scale, r, seed)
    range_update(r, out["acc_min"], out["acc_max"], a_scale)          # q^{t+1}
    return out
