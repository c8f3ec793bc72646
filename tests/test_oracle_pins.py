"""Pins of the CPU oracle against things other than itself: values the paper prints,
closed forms, brute force in Python integers, NumPy int64 matmul on an explicit im2col
matrix, adjoint identities.  No GPU needed."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import traffic
from oracle import Problem, Range

HERE = os.path.dirname(os.path.abspath(__file__))
f32 = np.float32


# --------------------------------------------------------------------------- P1
def test_traffic_model_reproduces_table5():
    """eq. (4)/(5) at b_w=b_a=8, b_acc=32 give the KB printed in Table 5 (rows 1,2,3,5 to the
    printed integer; row 4's printed KB do not follow from its stated shape -- they are those of
    a 144-channel 56x56 layer without the weight term -- so only its ratio is pinned)."""
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "table5_memory.txt"))
            if not l.startswith("#") and l.strip()]
    assert len(rows) == 5
    for i, (net, kind, ci, co, w, h, s_kb, d_kb, delta) in enumerate(rows):
        ci, co, w, h, s_kb, d_kb, delta = map(int, (ci, co, w, h, s_kb, d_kb, delta))
        k, dw = int(kind[0]), kind.endswith("dw")
        s = traffic.kib(traffic.static_bits(ci, co, k, w, h, depthwise=dw))
        d = traffic.kib(traffic.dynamic_bits(ci, co, k, w, h, depthwise=dw))
        assert round((d / s - 1) * 100) == delta
        if i != 3:
            assert abs(s - s_kb) <= 0.5 and abs(d - d_kb) <= 0.5, (net, kind, s, d)
        else:
            assert 2 * 144 * 56 * 56 / 1024 == s_kb and 10 * 144 * 56 * 56 / 1024 == d_kb


def test_traffic_model_terms():
    # dynamic - static is exactly one save and one load of the accumulator output
    assert traffic.dynamic_bits(3, 5, 3, 7, 11) - traffic.static_bits(3, 5, 3, 7, 11) == 2 * 5 * 7 * 11 * 32
    assert traffic.static_bits(3, 5, 3, 7, 11) == (3 * 5 * 9 + 3 * 77 + 5 * 77) * 8


# --------------------------------------------------------------------------- P6
def test_linear_brute_force_tiny():
    cases = []
    g = np.random.default_rng(0)
    for M, K, N in [(1, 1, 1), (2, 3, 4), (4, 4, 4), (3, 5, 2)]:
        cases.append((g.integers(-128, 128, (M, K)), g.integers(-128, 128, (N, K)), int(g.integers(-128, 128))))
    cases.append((np.full((4, 4), -128), np.full((4, 4), -128), 0))
    cases.append((np.full((4, 4), 127), np.full((4, 4), 127), -128))
    cases.append((np.eye(4, dtype=np.int64) * 127, np.arange(16).reshape(4, 4) - 8, 0))
    for A, Wt, z in cases:
        M, K = A.shape; N = Wt.shape[0]
        p = Problem.linear(M, K, N)
        got = oracle.fwd(p, A.astype(np.int8).reshape(p.in_shape()), z, Wt.astype(np.int8).reshape(p.w_shape()))
        for m in range(M):
            for n in range(N):
                want = sum((int(A[m, k]) - z) * int(Wt[n, k]) for k in range(K))
                assert got.reshape(M, N)[m, n] == want


def test_linear_matches_numpy_int64_matmul():
    g = np.random.default_rng(1)
    for M, K, N in [(37, 129, 53), (256, 512, 64), (5, 1000, 7)]:
        A = g.integers(-128, 128, (M, K), dtype=np.int8)
        Wt = g.integers(-128, 128, (N, K), dtype=np.int8)
        z = -128
        p = Problem.linear(M, K, N)
        got = oracle.fwd(p, A.reshape(p.in_shape()), z, Wt.reshape(p.w_shape())).reshape(M, N)
        want = (A.astype(np.int64) - z) @ Wt.astype(np.int64).T
        assert np.array_equal(got, want)
        # linear dgrad and wgrad are the two other matmuls
        G = g.integers(-128, 128, (M, N), dtype=np.int8)
        dx = oracle.dgrad(p, G.reshape(p.out_shape()), 3, Wt.reshape(p.w_shape())).reshape(M, K)
        assert np.array_equal(dx, (G.astype(np.int64) - 3) @ Wt.astype(np.int64))
        dw = oracle.wgrad(p, A.reshape(p.in_shape()), z, G.reshape(p.out_shape()), 3).reshape(N, K)
        assert np.array_equal(dw, (G.astype(np.int64) - 3).T @ (A.astype(np.int64) - z))


# --------------------------------------------------------------------------- P7
def im2col(X, z, R, S, stride, pad):
    """Explicit patch matrix [B*OH*OW, R*S*C] of (X - z) with zeros outside the image."""
    B, H, W, C = X.shape
    OH, OW = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    Xp = np.zeros((B, H + 2 * pad, W + 2 * pad, C), np.int64)
    Xp[:, pad:pad + H, pad:pad + W, :] = X.astype(np.int64) - z
    cols = np.empty((B, OH, OW, R, S, C), np.int64)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, r, s, :] = Xp[:, r:r + stride * OH:stride, s:s + stride * OW:stride, :]
    return cols.reshape(B * OH * OW, R * S * C), OH, OW


CONV_CASES = [  # B, H, W, Cin, Cout, R, S, stride, pad
    (2, 5, 6, 3, 4, 3, 3, 1, 1),
    (1, 7, 7, 4, 5, 3, 3, 2, 1),
    (2, 8, 6, 2, 3, 1, 1, 2, 0),
    (1, 9, 9, 4, 2, 7, 7, 2, 3),
    (3, 4, 4, 5, 6, 1, 1, 1, 0),
    (1, 6, 5, 3, 2, 3, 3, 1, 0),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_matches_im2col_matmul(case):
    B, H, W, Cin, Cout, R, S, stride, pad = case
    g = np.random.default_rng(hash(case) % 2**32)
    X = g.integers(-128, 128, (B, H, W, Cin), dtype=np.int8)
    Wt = g.integers(-128, 128, (Cout, R, S, Cin), dtype=np.int8)
    z = int(g.integers(-128, 128))
    p = Problem.conv(B, H, W, Cin, Cout, R, S, stride, pad)
    cols, OH, OW = im2col(X, z, R, S, stride, pad)
    assert p.out_hw() == (OH, OW)
    want = cols @ Wt.astype(np.int64).reshape(Cout, -1).T
    got = oracle.fwd(p, X, z, Wt)
    assert np.array_equal(got.reshape(-1, Cout), want)
    rows = g.permutation(B * OH * OW)[:7]
    assert np.array_equal(oracle.fwd_rows(p, X, z, Wt, rows), want[rows])


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_dgrad_wgrad_adjoint_identities(case):
    """<conv(X,W), G> = <X, dgrad(G,W)> = <W, wgrad(X,G)> in exact integers, for one-hot probes of
    every position: this fixes every element of dgrad and wgrad, not just an inner product."""
    B, H, W, Cin, Cout, R, S, stride, pad = case
    g = np.random.default_rng(hash(case) % 2**32 + 1)
    X = g.integers(-128, 128, (B, H, W, Cin), dtype=np.int8)
    Wt = g.integers(-128, 128, (Cout, R, S, Cin), dtype=np.int8)
    p = Problem.conv(B, H, W, Cin, Cout, R, S, stride, pad)
    OH, OW = p.out_hw()
    G = g.integers(-128, 128, (B, OH, OW, Cout), dtype=np.int8)
    zx, zg = int(g.integers(-128, 128)), int(g.integers(-20, 20))
    cols, _, _ = im2col(X, zx, R, S, stride, pad)
    Gm = G.astype(np.int64).reshape(-1, Cout) - zg
    # wgrad = G^T . cols   (textbook: derivative of cols @ W^T w.r.t. W)
    want_dw = (Gm.T @ cols).reshape(Cout, R, S, Cin)
    assert np.array_equal(oracle.wgrad(p, X, zx, G, zg), want_dw)
    # dgrad = col2im(G . W): scatter-add of the patch-matrix gradient
    dcols = (Gm @ Wt.astype(np.int64).reshape(Cout, -1)).reshape(B, OH, OW, R, S, Cin)
    dXp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), np.int64)
    for r in range(R):
        for s in range(S):
            dXp[:, r:r + stride * OH:stride, s:s + stride * OW:stride, :] += dcols[:, :, :, r, s, :]
    want_dx = dXp[:, pad:pad + H, pad:pad + W, :]
    got_dx = oracle.dgrad(p, G, zg, Wt)
    assert np.array_equal(got_dx, want_dx)
    rows = g.permutation(B * H * W)[:9]
    assert np.array_equal(oracle.dgrad_rows(p, G, zg, Wt, rows), want_dx.reshape(-1, Cin)[rows])
    # the scalar identities
    y = oracle.fwd(p, X, zx, Wt).astype(np.int64)
    assert int((y * (G.astype(np.int64) - zg)).sum()) == int(((X.astype(np.int64) - zx) * want_dx).sum()) \
        == int((Wt.astype(np.int64) * want_dw).sum())


DW_CASES = [(2, 5, 6, 3, 3, 3, 1, 1), (1, 7, 8, 4, 3, 3, 2, 1), (1, 6, 6, 2, 5, 5, 1, 2)]


@pytest.mark.parametrize("case", DW_CASES)
def test_depthwise_is_per_channel_conv(case):
    """A depthwise layer is C independent single-channel convolutions."""
    B, H, W, Ch, R, S, stride, pad = case
    g = np.random.default_rng(hash(case) % 2**32)
    X = g.integers(-128, 128, (B, H, W, Ch), dtype=np.int8)
    Wd = g.integers(-128, 128, (R, S, Ch), dtype=np.int8)
    p = Problem.depthwise(B, H, W, Ch, R, S, stride, pad)
    OH, OW = p.out_hw()
    G = g.integers(-128, 128, (B, OH, OW, Ch), dtype=np.int8)
    zx, zg = -128, 5
    y, dx, dw = oracle.fwd(p, X, zx, Wd), oracle.dgrad(p, G, zg, Wd), oracle.wgrad(p, X, zx, G, zg)
    rows = g.permutation(B * OH * OW)[:5]
    assert np.array_equal(oracle.fwd_rows(p, X, zx, Wd, rows), y.reshape(-1, Ch)[rows])
    rows = g.permutation(B * H * W)[:5]
    assert np.array_equal(oracle.dgrad_rows(p, G, zg, Wd, rows), dx.reshape(-1, Ch)[rows])
    for c in range(Ch):
        cols, _, _ = im2col(X[..., c:c + 1], zx, R, S, stride, pad)
        wc = Wd[..., c].astype(np.int64).reshape(-1)
        assert np.array_equal(y[..., c].reshape(-1), cols @ wc)
        gm = G[..., c].astype(np.int64).reshape(-1) - zg
        assert np.array_equal(dw[..., c].reshape(-1), gm @ cols)
        dcols = np.outer(gm, wc).reshape(B, OH, OW, R, S)
        dXp = np.zeros((B, H + 2 * pad, W + 2 * pad), np.int64)
        for r in range(R):
            for s in range(S):
                dXp[:, r:r + stride * OH:stride, s:s + stride * OW:stride] += dcols[:, :, :, r, s]
        assert np.array_equal(dx[..., c], dXp[:, pad:pad + H, pad:pad + W])


def test_minmax_brute():
    g = np.random.default_rng(3)
    c = g.integers(-2**31, 2**31, 1001).astype(np.int32)
    assert oracle.minmax(c) == (int(min(c.tolist())), int(max(c.tolist())))
    assert oracle.minmax(np.array([7], np.int32)) == (7, 7)


# --------------------------------------------------------------------------- P8
def test_qparams_hand_values():
    # asymmetric: [0, 255 s] -> scale s, zero point at the bottom of the grid
    s, z = oracle.qparams(0.0, 255 * 0.5, 0, -128, 127)
    assert s == f32(0.5) and z == -128
    # [-1, 3]: width 4, scale 4/255, zero point rne(-128 + 63.75) = -64
    s, z = oracle.qparams(-1.0, 3.0, 0, -128, 127)
    assert s == f32(4.0) / f32(255.0) and z == -64
    # range not containing zero is widened to it: [2, 4] behaves as [0, 4]
    assert oracle.qparams(2.0, 4.0, 0, -128, 127) == oracle.qparams(0.0, 4.0, 0, -128, 127)
    assert oracle.qparams(-4.0, -2.0, 0, -128, 127) == (f32(4.0) / f32(255.0), 127)
    # symmetric: scale = max|.|/127, zero point 0
    s, z = oracle.qparams(-2.54, 1.0, 1, -127, 127)
    assert s == f32(2.54) / f32(127) and z == 0
    s, z = oracle.qparams(-1.0, 12.7, 1, -127, 127)
    assert s == f32(12.7) / f32(127) and z == 0
    # degenerate ranges
    assert oracle.qparams(0.0, 0.0, 0, -128, 127) == (f32(1.0), -128)
    assert oracle.qparams(0.0, 0.0, 1, -127, 127) == (f32(1.0), 0)


def test_quantize_dequantize_idempotent_monotone_in_grid():
    g = np.random.default_rng(4)
    for sym, bits in [(0, 8), (1, 8), (0, 6), (1, 6), (0, 4), (1, 4), (0, 2), (1, 2)]:
        r0 = oracle.Range.new(0.9, bool(sym), bits)
        qlo, qhi = r0.qlo, r0.qhi
        assert qhi == 2 ** (bits - 1) - 1 and qlo == (-qhi if sym else -qhi - 1)      # b-bit grid
        for _ in range(20):
            lo, hi = -abs(g.normal()) * 10 ** g.uniform(-3, 3), abs(g.normal()) * 10 ** g.uniform(-3, 3)
            s, z = oracle.qparams(lo, hi, sym, qlo, qhi)
            assert s > 0 and qlo <= z <= qhi
            codes = np.arange(qlo, qhi + 1)
            # dequantized code, re-expressed in accumulator units of size s, quantizes back to itself
            back, nlo, nhi = oracle.requant((codes - z).astype(np.int32), s, s, z, qlo, qhi)
            assert np.array_equal(back, codes) and nlo == 0 and nhi == 0
            # real zero is exactly representable: accumulator 0 -> zero point
            assert oracle.requant(np.zeros(1, np.int32), s, s, z, qlo, qhi)[0][0] == z
            # monotone and inside the grid on a wide sweep, acc unit = s/7
            c = np.arange(-4000, 4000, dtype=np.int32)
            q, nlo, nhi = oracle.requant(c, f32(s) / f32(7), s, z, qlo, qhi)
            assert np.all(np.diff(q.astype(int)) >= 0) and q.min() >= qlo and q.max() <= qhi


# --------------------------------------------------------------------------- P9
def round_half_even(fr):
    fl = math.floor(fr)
    d = fr - fl
    if d > Fraction(1, 2) or (d == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


@pytest.mark.parametrize("num,den", [(1, 2), (1, 4), (3, 8), (5, 16), (1, 1), (3, 2), (7, 64), (1, 1024)])
def test_requant_rounding_exhaustive_vs_integer_arithmetic(num, den):
    """m = num/den is exact in fp32 and c*m is exact for |c| < 2^17, so the rounded value has an
    integer-arithmetic definition: round_half_even(c*num/den).  Includes every .5 tie."""
    c = np.arange(-70000, 70000, dtype=np.int32)
    z, qlo, qhi = 3, -(2**20), 2**20          # grid wide open: nothing clamps
    # int8 output would wrap; use a narrow window for codes and a wide one for counting
    got, nlo, nhi = oracle.requant(c, f32(num), f32(den), z, -128, 127)
    want = np.array([min(max(round_half_even(Fraction(int(v) * num, den)) + z, -128), 127) for v in c.tolist()])
    assert np.array_equal(got, want)
    r = np.array([round_half_even(Fraction(int(v) * num, den)) + z for v in c.tolist()])
    assert nlo == int((r < -128).sum()) and nhi == int((r > 127).sum())


# --------------------------------------------------------------------------- P10
def test_clip_counts_brute_force_and_saturation_ratio():
    g = np.random.default_rng(5)
    c = g.integers(-3000, 3000, 5000).astype(np.int32)
    a_scale = f32(0.01)
    for lo, hi, sym in [(-10.0, 10.0, 0), (-5.0, 20.0, 0), (-3.0, 3.0, 1), (-100.0, 100.0, 0), (0.0, 12.0, 0)]:
        qlo, qhi = (-127, 127) if sym else (-128, 127)
        s, z = oracle.qparams(lo, hi, sym, qlo, qhi)
        codes, nlo, nhi = oracle.requant(c, a_scale, s, z, qlo, qhi)
        m = f32(a_scale) / f32(s)
        r = np.rint((c.astype(np.float32) * m).astype(np.float32)).astype(np.int64) + z
        assert nlo == int((r < qlo).sum()) and nhi == int((r > qhi).sum())
        inside = int(((r >= qlo) & (r <= qhi)).sum())
        assert nlo + nhi + inside == c.size
        assert np.array_equal(codes, np.clip(r, qlo, qhi))
        # saturation ratio (Sec. 4 footnote): share of values outside the grid; real-valued count
        # may differ only by values within half a step of an edge
        real = c.astype(np.float64) * float(a_scale)
        rlo, rhi = float(s) * (qlo - z), float(s) * (qhi - z)
        outside = int((real < rlo - 0.5 * float(s)).sum() + (real > rhi + 0.5 * float(s)).sum())
        assert abs((nlo + nhi) - outside) <= int((np.abs(real - rlo) <= 0.51 * float(s)).sum()
                                                 + (np.abs(real - rhi) <= 0.51 * float(s)).sum())
    # a range that contains the data clips nothing
    s, z = oracle.qparams(-30.0, 30.0, 0, -128, 127)
    assert oracle.requant(c, a_scale, s, z, -128, 127)[1:] == (0, 0)


# --------------------------------------------------------------------------- P2-P4
def test_range_update_init_and_special_momenta():
    r = Range.new(eta=0.9)
    assert r.initialized == 0
    oracle.range_update(r, -100, 300, f32(0.5))            # t = 0: q^0 = min/max of first batch
    assert r.initialized == 1 and (r.qmin, r.qmax) == (-50.0, 150.0)
    assert (f32(r.scale), r.zero_point) == oracle.qparams(-50.0, 150.0, 0, -128, 127)
    # q^1 from the same statistics stays at q^0 (up to fp32 rounding of the two products)
    oracle.range_update(r, -100, 300, f32(0.5))
    assert abs(r.qmin + 50.0) <= 50.0 * 2e-7 and abs(r.qmax - 150.0) <= 150.0 * 2e-7
    # eta = 0: the range is the previous tensor's min-max
    r0 = Range.new(eta=0.0); oracle.range_update(r0, -1, 1, f32(1.0)); oracle.range_update(r0, -7, 9, f32(2.0))
    assert (r0.qmin, r0.qmax) == (-14.0, 18.0)
    # eta = 1: the range never leaves q^0
    r1 = Range.new(eta=1.0); oracle.range_update(r1, -1, 1, f32(1.0))
    for k in range(5):
        oracle.range_update(r1, -1000 * k, 1000 * k, f32(3.0))
    assert (r1.qmin, r1.qmax) == (-1.0, 1.0)


def test_range_update_one_step_by_hand():
    r = Range.new(eta=0.75, symmetric=True)
    oracle.range_update(r, -8, 16, f32(0.25))              # q^0 = (-2, 4)
    oracle.range_update(r, -16, 40, f32(0.25))             # g = (-4, 10)
    # (1-0.75)*(-4) + 0.75*(-2) = -2.5 ; 0.25*10 + 0.75*4 = 5.5  (all exact in fp32)
    assert (r.qmin, r.qmax) == (-2.5, 5.5)
    assert f32(r.scale) == f32(5.5) / f32(127) and r.zero_point == 0


def test_range_update_constant_statistics_is_a_fixed_point():
    r = Range.new(eta=0.9)
    oracle.range_update(r, -10, 10, f32(1.0))
    oracle.range_update(r, -1000, 3000, f32(0.01))
    for _ in range(400):
        oracle.range_update(r, -1000, 3000, f32(0.01))
    assert abs(r.qmin + 10.0) < 1e-4 and abs(r.qmax - 30.0) < 1e-4


@pytest.mark.parametrize("ratio,eta", [(1.05, 0.9), (0.8, 0.9), (1.3, 0.5), (0.5, 0.3)])
def test_range_update_geometric_drift_closed_form(ratio, eta):
    """Statistics g_t = g_0 r^t.  The recursion q^{t+1} = (1-eta) g_t + eta q^t with q^0 = g_0 solves to
    q^t = eta^t g_0 + (1-eta) g_0 (eta^t - r^t)/(eta - r)."""
    r = Range.new(eta=eta)
    g0 = 2.0
    oracle.range_update(r, -1000, 1000, f32(g0 / 1000))     # q^0 = (-2, 2)
    for t in range(0, 30):
        # state now holds q^t; feed the statistics of tensor t
        want = eta ** t * g0 + (1 - eta) * g0 * (eta ** t - ratio ** t) / (eta - ratio)
        assert abs(r.qmax - want) <= 1e-5 * abs(want), (t, r.qmax, want)
        assert abs(r.qmin + want) <= 1e-5 * abs(want)
        oracle.range_update(r, -1000, 1000, f32(g0 * ratio ** t / 1000))
    if ratio > eta and ratio > 1:
        # growing tensors: the in-hindsight range settles at (1-eta)/(r-eta) of the current one
        assert abs(r.qmax / (g0 * ratio ** 30) - (1 - eta) / (ratio - eta)) < 0.02


# --------------------------------------------------------------------------- P5
def test_static_with_current_range_equals_dynamic():
    """Static and dynamic quantization differ only in when the range is known (Sec. 3.2):
    handing the static path the tensor's own min-max must reproduce the dynamic result."""
    g = np.random.default_rng(6)
    for sym in (0, 1):
        c = (g.laplace(0, 300, 20000)).astype(np.int32)
        a_scale = f32(3e-4)
        dyn = oracle.quantize_dynamic(c, a_scale, sym, *((-127, 127) if sym else (-128, 127)))
        r = Range.new(symmetric=bool(sym))
        oracle.range_update(r, dyn["acc_min"], dyn["acc_max"], a_scale)
        st = oracle.quantize_static(c, a_scale, r)
        assert np.array_equal(st["codes"], dyn["codes"])
        assert (st["scale"], st["zero_point"]) == (dyn["scale"], dyn["zero_point"])
        assert st["clip_lo"] == dyn["clip_lo"] == 0 and st["clip_hi"] == dyn["clip_hi"] == 0
        # the extreme values land on the ends of the grid that the range touches
        codes = dyn["codes"].astype(int)
        if sym:
            assert max(abs(codes.min()), abs(codes.max())) == 127
        else:
            assert codes.min() == -128 and codes.max() == 127


def test_in_hindsight_sequence_uses_previous_range():
    """At iteration t >= 1 the codes must come from q^t, which depends only on tensors 0..t-1."""
    g = np.random.default_rng(7)
    a_scale = f32(1e-3)
    tensors = [(g.normal(0, 1000 * 1.5 ** t, 4096)).astype(np.int32) for t in range(4)]
    r = Range.new(eta=0.9)
    hist = []
    for t, c in enumerate(tensors):
        before = (r.scale, r.zero_point, r.initialized)
        out = oracle.in_hindsight_step(c, a_scale, r)
        if t == 0:
            assert np.array_equal(out["codes"], oracle.quantize_dynamic(c, a_scale, 0, -128, 127)["codes"])
        else:
            want, _, _ = oracle.requant(c, a_scale, before[0], before[1], -128, 127)
            assert np.array_equal(out["codes"], want)
            assert out["clip_lo"] + out["clip_hi"] > 0          # growing tensors overflow yesterday's range
        hist.append((r.qmin, r.qmax))
    # independent replay of eq. (2)-(3) in float64
    mn = [float(a_scale) * int(c.min()) for c in tensors]
    q = mn[0]
    q = 0.1 * mn[0] + 0.9 * q
    for t in range(1, 4):
        q = 0.1 * mn[t] + 0.9 * q
    assert abs(hist[-1][0] - q) <= 1e-5 * abs(q)


# ---------------------------------------------------------------------------------------
# Stochastic rounding (the paper's gradient quantizer, Sec. 5 experimental setup)
# ---------------------------------------------------------------------------------------
def _py_sr_bits(idx, seed):
    """The generator in Python integers, 32-bit wrap-around written out."""
    M = 0xffffffff
    h = idx & M
    h ^= h >> 16; h = (h * 0x85ebca6b) & M; h = (h + (seed & M)) & M
    h ^= (((idx >> 32) & M) * 0x85ebca77 + ((seed >> 32) & M)) & M
    h ^= h >> 13; h = (h * 0xc2b2ae35) & M; h ^= h >> 16
    h = (h * 0x9e3779b1) & M; h ^= h >> 15
    return h


def test_sr_bits_match_integer_arithmetic_and_depend_on_every_input():
    g = np.random.default_rng(5)
    for _ in range(200):
        idx, seed = int(g.integers(0, 2**63)), int(g.integers(0, 2**63))
        assert oracle.sr_bits(idx, seed) == _py_sr_bits(idx, seed)
    # flipping any single bit of the index or the seed flips about half of the output bits
    flips = []
    for bit in range(64):
        for which in range(2):
            d = []
            for k in range(64):
                idx, seed = int(g.integers(0, 2**63)), int(g.integers(0, 2**63))
                a = oracle.sr_bits(idx, seed)
                b = oracle.sr_bits(idx ^ (1 << bit), seed) if which == 0 else oracle.sr_bits(idx, seed ^ (1 << bit))
                d.append(bin(a ^ b).count("1"))
            flips.append(np.mean(d))
    assert min(flips) > 11.0 and max(flips) < 21.0, (min(flips), max(flips))


def test_sr_bits_are_uniform_over_consecutive_elements():
    """What the rounding uses: the top 24 bits of consecutive element indices.  Chi-square over
    256 equal bins, lag-1 correlation, and independence of two seeds' streams."""
    n = 1 << 16
    for seed in (0, 1, 0xdeadbeefcafe):
        u = np.array([oracle.sr_bits(i, seed) >> 8 for i in range(n)], dtype=np.float64) / 2.0**24
        counts = np.bincount((u * 256).astype(int), minlength=256)
        chi2 = float(((counts - n / 256) ** 2 / (n / 256)).sum())
        assert chi2 < 360.0, (seed, chi2)                   # 255 dof: mean 255, sd 22.6
        assert abs(u.mean() - 0.5) < 4 * (1 / 12 / n) ** 0.5
        assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.02
    a = np.array([oracle.sr_bits(i, 7) >> 8 for i in range(n)], dtype=np.float64)
    b = np.array([oracle.sr_bits(i, 8) >> 8 for i in range(n)], dtype=np.float64)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.02


def test_stochastic_rounding_is_a_floor_or_ceil_and_unbiased():
    """Gupta et al. (2015) as the paper uses it: x rounds up with probability x - floor(x).  Every
    code is floor(x) or floor(x) + 1, whole numbers are kept, the mean over many draws is x, and the
    share of round-ups follows the fraction (so the comparison is the right way round)."""
    n = 200000
    for c_val, a_scale, s_y in ((7, 0.3, 1.0), (-7, 0.3, 1.0), (3, 0.25, 1.0), (-3, 0.25, 1.0), (9, 0.1, 1.0), (40, 0.5, 2.0)):
        m = np.float32(a_scale) / np.float32(s_y)
        x = float(np.float32(c_val) * m)
        c = np.full(n, c_val, dtype=np.int32)
        codes, lo, hi = oracle.requant_stochastic(c, a_scale, s_y, 0, -128, 127, seed=99)
        fl = int(np.floor(x))
        assert set(np.unique(codes).tolist()) <= {fl, fl + 1} and lo == 0 and hi == 0
        p = x - fl
        ups = float((codes == fl + 1).mean())
        assert abs(ups - p) < 4 * max(p * (1 - p) / n, 1e-12) ** 0.5 + 1e-6, (x, ups, p)
        assert abs(codes.astype(np.float64).mean() - x) < 4 * max(p * (1 - p) / n, 1e-12) ** 0.5 + 1e-6
    # whole numbers never move, with any draw
    c = np.arange(-100, 100, dtype=np.int32)
    assert np.array_equal(oracle.requant_stochastic(c, 1.0, 1.0, 0, -128, 127, seed=3)[0], c.astype(np.int8))
    # the decision of element i is the comparison of its own draw with its own fraction
    g = np.random.default_rng(0)
    c = g.integers(-5000, 5000, 5000).astype(np.int32)
    a_scale, s_y, z = np.float32(0.0123), np.float32(0.31), -5
    codes, lo, hi = oracle.requant_stochastic(c, a_scale, s_y, z, -128, 127, seed=0x1234567890, idx0=10**12)
    m = a_scale / s_y
    want, wlo, whi = [], 0, 0
    for i, ci in enumerate(c):
        x = np.float32(ci) * m
        f = np.floor(x)
        u = np.float32(_py_sr_bits(10**12 + i, 0x1234567890) >> 8) * np.float32(2.0**-24)
        r = float(f + 1 if np.float32(x - f) > u else f)
        if r < -128 - z: r = -128 - z; wlo += 1
        if r > 127 - z: r = 127 - z; whi += 1
        want.append(int(r) + z)
    assert np.array_equal(codes, np.array(want, dtype=np.int8)) and (lo, hi) == (wlo, whi) and wlo > 0 and whi > 0


def test_stochastic_rounding_against_nearest_and_in_the_step():
    """Never further than one grid step from the nearest-even code; with the same seed the same codes;
    statistics (min / max, and with them the range update) do not depend on the rounding mode."""
    g = np.random.default_rng(4)
    c = g.integers(-20000, 20000, (64, 48)).astype(np.int32)
    a_scale = np.float32(1e-4)
    r1, r2 = oracle.Range.new(0.9, True), oracle.Range.new(0.9, True)
    o1 = oracle.in_hindsight_step(c, a_scale, r1)
    o2 = oracle.in_hindsight_step(c, a_scale, r2, seed=11)          # first iteration: dynamic, nearest-even on both
    assert np.array_equal(o1["codes"], o2["codes"])
    c2 = (c * 0.9).astype(np.int32)
    o1 = oracle.in_hindsight_step(c2, a_scale, r1)
    o2 = oracle.in_hindsight_step(c2, a_scale, r2, seed=11)
    o3 = oracle.quantize_static(c2, a_scale, oracle.Range.new(0.9, True) if False else r2, seed=11)
    d = o2["codes"].astype(int) - o1["codes"].astype(int)
    assert np.abs(d).max() == 1 and (d != 0).mean() > 0.2
    assert (o1["acc_min"], o1["acc_max"]) == (o2["acc_min"], o2["acc_max"])
    assert (r1.qmin, r1.qmax, r1.scale) == (r2.qmin, r2.qmax, r2.scale)
    assert not np.array_equal(o2["codes"], oracle.quantize_static(c2, a_scale, r2, seed=12)["codes"])


def test_weight_quantizer_current_min_max():
    """Q_W (Sec. 3.1, Sec. 5): hand values, the extreme maps to +-127, an all-zero tensor keeps
    scale 1, codes are within half a step of the weight, monotone, and a fixed point of
    quantize(dequantize(.))."""
    codes, s = oracle.quantize_weights(np.array([0.0, 1.27, -1.27, 0.635, 0.005, -0.0151, 0.64], np.float32))
    assert s == f32(1.27) / f32(127) and codes.tolist() == [0, 127, -127, 64, 0, -2, 64]
    codes, s = oracle.quantize_weights(np.zeros(5, np.float32))
    assert s == f32(1.0) and not codes.any()
    g = np.random.default_rng(8)
    w = (g.standard_normal(20000) * 0.05).astype(np.float32)
    codes, s = oracle.quantize_weights(w)
    assert s == np.abs(w).max() / f32(127) and np.abs(codes).max() == 127 and codes.min() >= -127
    assert np.abs(w.astype(np.float64) - float(s) * codes) .max() <= 0.5 * float(s) * (1 + 1e-6)
    order = np.argsort(w, kind="stable")
    assert (np.diff(codes[order].astype(int)) >= 0).all()
    again, s2 = oracle.quantize_weights((f32(s) * codes.astype(np.float32)).astype(np.float32))
    assert np.array_equal(again, codes) and abs(float(s2) - float(s)) <= 1e-6 * float(s)
    # ties go to the even code: 0.5 and 1.5 steps of a tensor whose scale is exactly 1/64
    codes, s = oracle.quantize_weights(np.array([127 / 64, 0.5 / 64, 1.5 / 64, 2.5 / 64, -0.5 / 64, -1.5 / 64], np.float32))
    assert s == f32(1 / 64) and codes.tolist() == [127, 0, 2, 2, 0, -2]


def test_real_tensor_quantizer_hand_values_bounds_and_statistics():
    """Static quantization of a real-valued tensor (Sec. 3.2): hand values with ties, clip counts,
    exact minimum / maximum, the half-step error bound inside the range (fp64 brute force), and
    agreement with the accumulator path for integer-valued inputs."""
    # scale 1/4, zero point -3, full asymmetric grid: x = k/4 -> code k - 3; ties to the even integer
    x = np.array([0.0, 0.25, -0.25, 0.125, 0.375, -0.125, -0.375, 32.5, 32.75, 33.0, -31.25, -31.5, 1e6, -1e6], np.float32)
    o = oracle.quantize_tensor(x, 0.25, -3, -128, 127)
    assert o["codes"].tolist() == [-3, -2, -4, -3, -1, -3, -5, 127, 127, 127, -128, -128, 127, -128]
    assert (o["clip_lo"], o["clip_hi"]) == (2, 3)          # 32.5 -> code 127 exactly: inside; 32.75, 33, 1e6 above; -31.5, -1e6 below
    assert o["min"] == f32(-1e6) and o["max"] == f32(1e6) and o["count"] == x.size
    g = np.random.default_rng(21)
    for sym in (0, 1):
        x = (g.standard_normal(30000) * 3).astype(np.float32)
        lo, hi = np.percentile(x, 1), np.percentile(x, 99)
        qlo, qhi = (-127, 127) if sym else (-128, 127)
        s, z = oracle.qparams(lo, hi, sym, qlo, qhi)
        o = oracle.quantize_tensor(x, s, z, qlo, qhi)
        assert o["min"] == x.min() and o["max"] == x.max()
        ideal = x.astype(np.float64) / float(s) + z             # unrounded code in fp64
        inside = (ideal > qlo + 1e-3) & (ideal < qhi - 1e-3)
        assert np.abs(o["codes"][inside] - ideal[inside]).max() <= 0.5 + 1e-4
        assert np.all(o["codes"][ideal >= qhi] == qhi) and np.all(o["codes"][ideal <= qlo] == qlo)
        # clipped = rounded code outside the grid: ideal beyond the edge by more than half a step
        margin = 1e-3
        assert int((ideal < qlo - 0.5 - margin).sum()) <= o["clip_lo"] <= int((ideal < qlo - 0.5 + margin).sum())
        assert int((ideal > qhi + 0.5 + margin).sum()) <= o["clip_hi"] <= int((ideal > qhi + 0.5 - margin).sum())
        assert o["clip_lo"] > 50 and o["clip_hi"] > 50
        # integer-valued reals of unit 1 are accumulators of scale 1
        c = g.integers(-5000, 5000, 4000).astype(np.int32)
        codes, nlo, nhi = oracle.requant(c, 1.0, f32(37.5), z, qlo, qhi)
        o = oracle.quantize_tensor(c.astype(np.float32), f32(37.5), z, qlo, qhi)
        assert np.array_equal(o["codes"], codes) and (o["clip_lo"], o["clip_hi"]) == (nlo, nhi)


def test_real_tensor_stochastic_rounding_is_floor_or_ceil_and_unbiased():
    """Stochastic rounding of a real-valued tensor: every code is floor or ceil of x/s (fp64 brute
    force), the mean over many elements of one value approaches it, whole numbers never move, the
    decision of element i is the one its own draw gives, and the seed matters."""
    s, z = f32(0.25), 5
    x = np.full(200000, 0.3, np.float32)                 # x/s = 1.2
    o = oracle.quantize_tensor(x, s, z, -128, 127, seed=3)
    vals = o["codes"].astype(int) - z
    assert set(np.unique(vals)) == {1, 2} and abs(vals.mean() - 1.2) < 0.005
    assert o["min"] == f32(0.3) and o["max"] == f32(0.3) and o["clip_lo"] + o["clip_hi"] == 0
    for i in (0, 1, 77, 199999):                         # up iff fraction > u_i
        u = (oracle.sr_bits(i, 3) >> 8) / 2.0 ** 24
        frac = float(f32(0.3) * (f32(1.0) / s)) - 1.0
        assert vals[i] == (2 if frac > u else 1)
    g = np.random.default_rng(6)
    x = (g.standard_normal(50000) * 2).astype(np.float32)
    o = oracle.quantize_tensor(x, s, z, -128, 127, seed=9)
    ideal = x.astype(np.float64) / 0.25
    d = (o["codes"].astype(int) - z) - ideal
    assert d.min() > -1 - 1e-5 and d.max() < 1 + 1e-5 and abs(d.mean()) < 0.01
    assert not np.array_equal(o["codes"], oracle.quantize_tensor(x, s, z, -128, 127, seed=10)["codes"])
    whole = np.arange(-20, 20).astype(np.float32) * s
    assert np.array_equal(oracle.quantize_tensor(whole, s, z, -128, 127, seed=1)["codes"], np.arange(-20, 20) + z)
    # clip counts follow the rounded value: far outside always clips
    o = oracle.quantize_tensor(np.array([100.0, -100.0, 0.0], np.float32), s, z, -128, 127, seed=1)
    assert o["codes"].tolist() == [127, -128, 5] and (o["clip_lo"], o["clip_hi"]) == (1, 1)


def test_real_tensor_step_follows_the_three_estimators():
    """Sec. 4.1 / eq. (1)-(3) on real-valued tensors: which range quantizes batch t under each
    estimator, checked against the recursion evaluated in fp64 by hand."""
    eta = 0.9
    mins = [-1.0, -2.0, -0.5, -4.0, -1.5]
    maxs = [3.0, 1.0, 6.0, 2.0, 2.5]
    g = np.random.default_rng(5)
    batches = []
    for lo, hi in zip(mins, maxs):
        x = g.uniform(lo, hi, 1000).astype(np.float32)
        x[0], x[1] = lo, hi
        batches.append(x)
    grid = 255.0
    # in hindsight: batch 0 with its own range; batch t with the average of batches < t
    r = oracle.Range.new(eta, False)
    qmin = qmax = None
    for t, x in enumerate(batches):
        o = oracle.tensor_step(x, r, "hindsight")
        if t == 0:
            used = (mins[0], maxs[0]); qmin, qmax = mins[0], maxs[0]
        else:
            used = (qmin, qmax)
        assert abs(float(o["scale"]) - (used[1] - used[0]) / grid) <= 1e-6 * (used[1] - used[0]) / grid
        qmin, qmax = (1 - eta) * mins[t] + eta * qmin, (1 - eta) * maxs[t] + eta * qmax
        assert abs(r.qmin - qmin) <= 1e-6 * abs(qmin) and abs(r.qmax - qmax) <= 1e-6 * abs(qmax)
        if t > 0 and (mins[t] < used[0] or maxs[t] > used[1]):
            assert o["clip_lo"] + o["clip_hi"] > 0                 # the estimate of the past does not cover this batch
    # current min-max: always the batch's own range, so nothing clips
    r = oracle.Range.new(eta, False)
    for t, x in enumerate(batches):
        o = oracle.tensor_step(x, r, "current")
        assert abs(float(o["scale"]) - (maxs[t] - mins[t]) / grid) <= 1e-6 and o["clip_lo"] + o["clip_hi"] == 0
    assert abs(r.qmin - qmin) <= 1e-6 * abs(qmin)                   # the state still follows eq. (2)-(3)
    # running min-max: batch t with the average that already includes batch t
    r = oracle.Range.new(eta, False)
    qmin, qmax = mins[0], maxs[0]
    for t, x in enumerate(batches):
        o = oracle.tensor_step(x, r, "running")
        if t > 0:
            qmin, qmax = (1 - eta) * mins[t] + eta * qmin, (1 - eta) * maxs[t] + eta * qmax
        assert abs(float(o["scale"]) - (qmax - qmin) / grid) <= 1e-6 * (qmax - qmin) / grid
    # symmetric gradients: scale from the larger magnitude
    r = oracle.Range.new(eta, True)
    o = oracle.tensor_step(np.array([-3.0, 1.0, 0.5], np.float32), r, "hindsight")
    assert o["scale"] == f32(3.0) / f32(127) and o["zero_point"] == 0 and o["codes"].tolist() == [-127, 42, 21]


def test_workload_shapes_match_the_configurations():
    import workloads as wl
    L = wl.c2_layer()
    assert (L.B * 56 * 56, 9 * 64, 64) == (401408, 576, 64)
    assert wl.fused_bytes(L, "fwd") == 2 * 128 * 56 * 56 * 64 + 576 * 64
    assert wl.dynamic_bytes(L, "fwd") - wl.fused_bytes(L, "fwd") == 8 * 128 * 56 * 56 * 64
    assert 2 * wl.macs(L) == 2 * 401408 * 576 * 64
    layers = wl.resnet18_layers()
    assert len(layers) == 21
    assert [l.Cout for l in layers if l.name.endswith("conv0")] == [64, 128, 256, 512]
    assert wl.out_hw(layers[0]) == (112, 112) and wl.out_hw(layers[5]) == (28, 28)
    assert abs(wl.c3_grad_scale(49) - 1e-3) < 1e-12 and wl.c3_grad_scale(0) == 1.0


# --------------------------------------------------------------------------- FP32 weight gradient
def _rne_f32(x):
    """Exact rational -> nearest fp32 (ties to even), computed in integers: the one rounding an
    IEEE single-precision operation performs on its exact result."""
    x = Fraction(x)
    if x == 0:
        return f32(0.0)
    sign, ax = (-1 if x < 0 else 1), abs(x)
    e = ax.numerator.bit_length() - ax.denominator.bit_length()       # 2^(e-1) < ax < 2^(e+1)
    if Fraction(2) ** e > ax:
        e -= 1                                                          # now 2^e <= ax < 2^(e+1)
    ulp_exp = max(e - 23, -149)                                         # subnormals share one spacing
    q = ax / Fraction(2) ** ulp_exp
    n, rem = divmod(q.numerator, q.denominator)
    twice = 2 * rem
    if twice > q.denominator or (twice == q.denominator and (n & 1)):
        n += 1
    v = sign * Fraction(n) * Fraction(2) ** ulp_exp
    assert abs(v) < Fraction(2) ** 128
    out = f32(float(v))                                                 # v is representable: exact
    assert Fraction(float(out)) == v
    return out


def _fr(x):
    return Fraction(float(x))


def test_fp32_weight_gradient_scale_is_pinned_by_exact_rationals():
    """Sec. 3.1 keeps the weight gradient in FP32: dW = (s_x * s_g) * float(c), the scale product
    rounded first, then one multiply per element.  Expectations come from exact rational
    arithmetic with one explicit rounding per operation; the cases include triples on which the
    other association s_x * (s_g * c), and a double-precision product rounded once, give
    different bits, so an oracle with either of those fails here."""
    assert _rne_f32(Fraction(1, 3)) == f32(1.0) / f32(3.0) and _rne_f32(Fraction(16777217)) == f32(16777216.0)
    assert _rne_f32(Fraction(16777219)) == f32(16777220.0) and _rne_f32(Fraction(-5, 2 ** 151)) == f32(-2.0 ** -149)

    # hand values, exact in fp32 (powers of two and small integers)
    got = oracle.wgrad_scale(np.array([0, 1, -1, 3, -7, 2 ** 24, -2 ** 31], np.int32), 0.5, 0.25)
    assert got.tolist() == [0.0, 0.125, -0.125, 0.375, -0.875, 2097152.0, -268435456.0]
    assert oracle.acc_scale(0.5, 0.25) == f32(0.125) and oracle.acc_scale(3.0, 0.0625) == f32(0.1875)

    g = np.random.default_rng(20210504)
    differs_assoc = differs_double = differs_conv = 0
    for _ in range(300):
        sx = f32(g.uniform(1e-3, 0.1)); sg = f32(g.uniform(1e-6, 1e-2))
        c = np.concatenate([g.integers(-2 ** 31, 2 ** 31, 48), g.integers(-3000, 3000, 16),
                            [2 ** 24 + 1, 2 ** 25 + 3, -(2 ** 30) - 65, 2 ** 31 - 1]]).astype(np.int32)
        s = _rne_f32(_fr(sx) * _fr(sg))
        assert oracle.acc_scale(sx, sg) == s and oracle.acc_scale(sg, sx) == s
        got = oracle.wgrad_scale(c, sx, sg)
        for ci, gi in zip(c.tolist(), got):
            cf = _rne_f32(Fraction(ci))                                # int32 -> fp32 conversion rounds
            want = _rne_f32(_fr(s) * _fr(cf))
            assert gi == want and np.signbit(gi) == np.signbit(want), (sx, sg, ci, gi, want)
            differs_assoc += _rne_f32(_fr(sx) * _fr(_rne_f32(_fr(sg) * _fr(cf)))) != want
            differs_double += _rne_f32(_fr(sx) * _fr(sg) * ci) != want
            differs_conv += _rne_f32(_fr(s) * ci) != want
    # the cases do tell the three plausible mistakes apart from the definition
    assert differs_assoc > 100 and differs_double > 100 and differs_conv > 100


def test_accumulator_unit_feeds_the_range_update_as_one_fp32_product():
    """The real value of one accumulator unit is the fp32 product s_a * s_b (one rounding); the
    statistics enter eq. (2)-(3) as that product times the integer extreme (a second rounding)."""
    g = np.random.default_rng(7)
    for _ in range(50):
        sa = f32(g.uniform(1e-3, 0.1)); sb = f32(g.uniform(1e-4, 0.05))
        mn, mx = int(g.integers(-2 ** 30, 0)), int(g.integers(1, 2 ** 30))
        r = oracle.Range.new(0.9, False)
        a = oracle.acc_scale(sa, sb)
        oracle.range_update(r, mn, mx, a)                               # sets q^0 = min-max of the first batch
        assert f32(r.qmin) == _rne_f32(_fr(a) * _fr(_rne_f32(Fraction(mn))))
        assert f32(r.qmax) == _rne_f32(_fr(a) * _fr(_rne_f32(Fraction(mx))))


# --------------------------------------------------------------------------- saturation-driven update
def test_fixed_sequence_logarithm_is_a_logarithm():
    """The fp32 logarithm the saturation-driven update evaluates with a fixed operation sequence
    agrees with the mathematical one to 1e-6 (absolute, or relative for large magnitudes)."""
    g = np.random.default_rng(11)
    xs = np.concatenate([10.0 ** g.uniform(-30, 0, 4000), g.uniform(0.4, 1.0, 4000),
                         [1.0, 0.5, 0.25, 2.0 ** -20, 0.70710678, 0.70710689, 2e-38]]).astype(np.float32)
    for x in xs:
        got, want = float(oracle.ln_fixed(x)), math.log(float(x))
        assert abs(got - want) <= 1e-6 * max(1.0, abs(want)), (x, got, want)
    assert oracle.ln_fixed(1.0) == 0.0
    assert oracle.ln_fixed(2.0 ** -8) * f32(2.0) == oracle.ln_fixed(2.0 ** -16)      # e * ln 2, exactly


def _sat_out(clip, count, mn=-1000, mx=1000):
    return dict(clip_lo=clip // 2, clip_hi=clip - clip // 2, count=count, acc_min=mn, acc_max=mx)


def test_saturation_update_band_streak_and_rescaling_by_hand():
    """Sec. 4 names the saturation ratio as a statistic; the rule pinned here (DESIGN reading): inside
    the band nothing moves; outside it for more than tau iterations in a row the range is rescaled by
    ln(alpha_target) / ln(alpha)."""
    r = oracle.Range.new(0.9, True)
    sat = oracle.Saturation.new(alpha_min=2.0 ** -12, alpha_max=2.0 ** -6, alpha_target=2.0 ** -8, tau=2)
    # first call: q^0 from the first batch's min-max
    oracle.range_update_saturation(r, sat, _sat_out(0, 4096, -500, 750), 0.01)
    assert (r.qmin, r.qmax, r.initialized, sat.streak) == (f32(0.01) * f32(-500), f32(0.01) * f32(750), 1, 0)
    q0 = (r.qmin, r.qmax)
    # inside the band (2^-12 <= alpha <= 2^-6): nothing moves, at the edges too
    for clip in (1 << 8, 1 << 4, 1 << 10):                                     # alpha = 2^-8, 2^-12, 2^-6 of 2^16
        oracle.range_update_saturation(r, sat, _sat_out(clip, 1 << 16), 0.01)
        assert (r.qmin, r.qmax) == q0 and sat.streak == 0
    # too much clipping (alpha = 2^-4), but only twice in a row, then back inside: no update
    for _ in range(2):
        oracle.range_update_saturation(r, sat, _sat_out(1 << 12, 1 << 16), 0.01)
    assert (r.qmin, r.qmax) == q0 and sat.streak == 2
    oracle.range_update_saturation(r, sat, _sat_out(1 << 8, 1 << 16), 0.01)
    assert (r.qmin, r.qmax) == q0 and sat.streak == 0
    # three times in a row (more than tau = 2): rescaled by ln(2^-8) / ln(2^-4) = 2, exactly
    for k in range(3):
        oracle.range_update_saturation(r, sat, _sat_out(1 << 12, 1 << 16), 0.01)
        assert sat.streak == (k + 1) % 3
    assert (r.qmin, r.qmax) == (f32(2) * q0[0], f32(2) * q0[1])
    assert r.scale == f32(2) * q0[1] / f32(127)                                # quantizer re-derived (symmetric grid)
    # too little clipping (alpha = 2^-16 < alpha_min): after three iterations the range halves
    for _ in range(3):
        oracle.range_update_saturation(r, sat, _sat_out(1, 1 << 16), 0.01)
    assert (r.qmin, r.qmax) == q0
    # nothing clipped at all: the ratio is taken as half an element, 1 / (2 count)
    for _ in range(3):
        oracle.range_update_saturation(r, sat, _sat_out(0, 1 << 15), 0.01)
    assert (r.qmin, r.qmax) == (f32(0.5) * q0[0], f32(0.5) * q0[1])
    # everything clipped: the ratio is capped at 1/2, the range grows by ln(2^-8) / ln(1/2) = 8
    for _ in range(3):
        oracle.range_update_saturation(r, sat, _sat_out(1 << 15, 1 << 15), 0.01)
    assert (r.qmin, r.qmax) == (f32(4) * q0[0], f32(4) * q0[1])
    # no statistics: nothing happens
    before = (r.qmin, r.qmax, sat.streak)
    oracle.range_update_saturation(r, sat, _sat_out(0, 0), 0.01)
    assert (r.qmin, r.qmax, sat.streak) == before


@pytest.mark.parametrize("start", [0.25, 4.0])
def test_saturation_update_reaches_the_laplace_quantile(start):
    """For a zero-mean Laplace(0, b) tensor a fraction exp(-q / b) lies beyond +-q, so the rescaled
    range must land on q' = b ln(1 / alpha_target) whatever range it started from, and the next
    batch then saturates at about alpha_target (the inverse-CDF step of Sec. 4's saturation variant)."""
    g = np.random.default_rng(3)
    b, a_scale, target, n = 400.0, f32(1e-3), 1e-3, 1 << 21
    sat = oracle.Saturation.new(alpha_min=5e-4, alpha_max=2e-3, alpha_target=target, tau=0)
    r = oracle.Range.new(0.9, True)
    q_star = b * math.log(1 / target)                                          # in accumulator units
    r.qmin, r.qmax, r.initialized = -start * q_star * float(a_scale), start * q_star * float(a_scale), 1
    lib_range = oracle.qparams(r.qmin, r.qmax, 1, -127, 127)
    r.scale, r.zero_point = float(lib_range[0]), int(lib_range[1])
    ratios = []
    for t in range(3):
        c = np.rint(g.laplace(0, b, n)).astype(np.int32)
        out = oracle.quantize_static(c, a_scale, r)
        ratios.append((out["clip_lo"] + out["clip_hi"]) / n)
        oracle.range_update_saturation(r, sat, out, a_scale)
    if start < 1:
        assert abs(ratios[0] - math.exp(-start * math.log(1 / target))) < 0.01  # started too narrow: e^(-q/b)
    else:
        assert ratios[0] == 0                                                  # started too wide: nothing clips
    # started too narrow: one step lands on the quantile; too wide: the unseen tail is taken as half an
    # element, so the first step overshoots downwards and the second corrects it
    assert abs(r.qmax / (q_star * float(a_scale)) - 1) < 0.08
    assert 0.5 * target < ratios[2] < 2 * target


def test_saturation_step_orders_the_first_batch_like_in_hindsight_min_max():
    """First batch: quantized with its own min-max (nothing clips), which also becomes q^0; its clip
    counts then enter the saturation rule like any other batch's (one iteration below the band)."""
    c = np.array([-700, -3, 0, 5, 900, 12], np.int32)
    r, sat = oracle.Range.new(0.9, True), oracle.Saturation.new(1e-3, 1e-1, 1e-2, tau=3)
    out = oracle.saturation_step(c, f32(0.5), r, sat)
    assert (r.qmin, r.qmax, r.initialized, sat.streak) == (-350.0, 450.0, 1, 1)
    assert out["clip_lo"] + out["clip_hi"] == 0 and out["codes"].tolist() == [-99, 0, 0, 1, 127, 2]
    # second batch, statically with q^0: one of six values clips (alpha = 1/6 > alpha_max), streak 2
    out = oracle.saturation_step(np.array([-700, -3, 0, 5, 2000, 12], np.int32), f32(0.5), r, sat)
    assert out["clip_hi"] == 1 and out["codes"][4] == 127 and sat.streak == 2 and (r.qmin, r.qmax) == (-350.0, 450.0)
