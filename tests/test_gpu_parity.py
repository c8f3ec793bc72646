"""GPU parity: the HIP library (through its C-ABI binding) against the CPU oracle, element by
element, on the same seeded inputs.  Integer results (codes, accumulators, min/max, clip
counts) must match bit for bit; the fp32 range state within 1e-6 relative."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H(hq):
    import hq_harness
    return hq_harness


def rand_layer_inputs(L, seed, x_asym=True, g_asym=False):
    g = np.random.default_rng(seed)
    X = wl.relu_activation(g, wl.in_shape(L)) if x_asym else \
        wl.to_symmetric_codes(g.standard_normal(wl.in_shape(L), dtype=np.float32), 3.0 / 127)
    W = wl.he_weight(g, L)
    if g_asym:
        dY = wl.to_asymmetric_codes(g.laplace(0, 1e-3, wl.out_shape(L)).astype(np.float32) + np.float32(4e-4))
    else:
        dY = wl.laplace_gradient(g, wl.out_shape(L), 1e-3)
    return X, W, dY


# ---------------------------------------------------------------------------------------
# Config 1: single linear layer, 4 iterations, forward + dgrad + wgrad
# ---------------------------------------------------------------------------------------
def test_c1_linear_four_iterations(H, hq):
    y_track = H.TensorTrack(0.9, symmetric=False)
    g_track = H.TensorTrack(0.9, symmetric=True)
    Wdev = None
    for t in range(4):
        L, X, W, dY = wl.c1_inputs(t)
        if Wdev is None:
            Wdev = H.DevWeights(L, W)
        Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
        y_track.step(L, "fwd", X, W, Xd, Wdev)
        g_track.step(L, "dgrad", dY, W, dYd, Wdev)
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref)
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


# ---------------------------------------------------------------------------------------
# Small shapes spanning several tiles with ragged tails, strides, 1x1, odd channel counts
# ---------------------------------------------------------------------------------------
SMALL = [
    wl.linear("lin_ragged", 300, 80, 72),            # M, N tails; K not a multiple of 64
    wl.linear("lin_fc", 37, 512, 1000),              # N = 1000: dgrad reduces over 1000 (not /16)
    wl.linear("lin_k24", 130, 24, 36),               # K % 16 != 0 forward
    wl.conv("c3x3_16", 2, 9, 16, 32, 3),             # small conv, ragged M
    wl.conv("c3x3_s2", 2, 12, 32, 48, 3, stride=2),  # stride 2: dgrad with missing taps
    wl.conv("c1x1_s2", 3, 10, 16, 64, 1, stride=2, pad=0),
    wl.conv("c3x3_c24", 1, 7, 24, 40, 3),            # channels % 16 != 0 on both sides
    wl.conv("c3x3_wide", 1, 10, 64, 160, 3),         # N > 128: two column tiles, second ragged
    wl.conv("c5x5", 1, 9, 16, 16, 5),
    wl.conv("c3x3_nopad", 2, 8, 16, 16, 3, pad=0),
    wl.conv("c3x3_big", 4, 28, 128, 128, 3),         # the 128x128-tile paths of all three kernels
    wl.conv("band_c64", 3, 30, 64, 64, 3),           # weights-resident path, one-row bands
    wl.conv("band_c64_n48", 2, 17, 64, 48, 3),       # ... with a ragged column tile
    wl.conv("band_c64_s2", 2, 22, 64, 64, 3, stride=2),
    wl.conv("band_1x1_c32", 2, 20, 32, 192, 1),      # three column chunks per tile
    wl.conv("band_1x1_c192", 2, 20, 192, 32, 1),
    wl.conv("band_multi_tile", 128, 36, 64, 64, 3),  # 4 bands per image of 9 rows: two tiles per band, second ragged
    wl.conv("wband_14", 3, 14, 64, 64, 3),           # weight-gradient band = one whole image, 28 pixels of padding
    wl.depthwise("dw_strips", 3, 40, 48),            # depthwise strips with a ragged last strip
    wl.conv("bandw_multi_img", 3, 10, 128, 192, 3),  # streamed-weights path: tiles of two whole images (last one short), ragged channel chunk
    wl.conv("bandw_rows", 2, 30, 192, 128, 3),       # ... tiles of rows, last tile of an image short; wgrad blocks 3 x 2
    wl.conv("first_layer", 2, 23, 4, 48, 7, stride=2),   # 4-channel first layer: direct kernel, ragged channel block, odd size
    wl.conv("first_layer_c8", 2, 19, 8, 32, 3),      # 8-channel first layer: packed weight gradient, general forward
    wl.conv("c5x5_s3", 2, 17, 16, 32, 5, stride=3),  # stride 3: nine pixel classes in the input gradient
    wl.conv("band_early_tail", 128, 24, 64, 64, 3),  # bands of 288 pixels: the 32-pixel last tile is taken in the first half step
    wl.LayerShape("c2x1_s3", wl.CONV, 1, 2, 10, 4, 2, 1, 3, 0, 36),   # filter of width 1 and height 2 (division by 1 in the tap arithmetic)
    wl.LayerShape("c1x3_w1", wl.CONV, 2, 9, 1, 16, 1, 1, 1, 0, 32),   # images one pixel wide
    wl.conv("gemm128_conv", 5, 58, 144, 136, 3),     # general kernel with 128 x 128 tiles (264 of them), ragged in both directions
    wl.linear("gemm128_lin", 20000, 256, 200),       # ... linear layer, 314 tiles
    wl.conv("gemm64_small_images", 40, 4, 512, 256, 3),   # 4 x 4 images under a long reduction: 64 x 64 tiles
    wl.conv("band_w64", 2, 64, 64, 64, 3),           # weights-resident kernel, patch rows of more than 64 pixels (two chunks per thread)
    wl.LayerShape("band_w126", wl.CONV, 1, 9, 126, 64, 3, 3, 1, 1, 48),   # ... the widest rows it takes, ragged tiles and columns
    wl.conv("c1x1_s2_n24", 2, 11, 24, 32, 1, stride=2, pad=0),           # pixel classes that no tap reaches, filled in 4-byte pieces
    wl.LayerShape("c2x2_s3", wl.CONV, 2, 14, 17, 32, 2, 2, 3, 0, 48),      # ... five of nine classes, 16-byte pieces, non-square image
    wl.linear("wgrad_one_split", 96, 2048, 2048),    # weight gradient with one writer per sum (256 tiles, no pixel splits)
]


@pytest.mark.parametrize("L", SMALL, ids=[l.name for l in SMALL])
def test_small_shapes_all_ops(H, hq, L):
    y_track, g_track = H.TensorTrack(0.9, False), H.TensorTrack(0.9, True)
    Wdev = None
    for t in range(3):
        X, W, dY = rand_layer_inputs(L, 1000 + t)
        if Wdev is None:
            W0, Wdev = W, H.DevWeights(L, W)
        Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
        y_track.step(L, "fwd", X, W0, Xd, Wdev)
        g_track.step(L, "dgrad", dY, W0, dYd, Wdev)
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref)
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


# ---------------------------------------------------------------------------------------
# 3-channel (RGB) first layers: forward (fused and dynamic) and weight gradient; 3-byte pixels
# ---------------------------------------------------------------------------------------
def random_staged_first_layers(n, seed, C):
    """Seeded random first layers of the kind whose input rows are staged in LDS: even stride, width a multiple
    of 4, at most 8 taps per filter row and 7 filter rows, 16 .. 64 output channels."""
    g = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < n:
        R, S = int(g.integers(1, 8)), int(g.integers(1, 9))
        L = wl.LayerShape("staged%d_c%d" % (len(shapes), C), wl.CONV, int(g.choice([1, 2, 3, 5])), int(g.integers(4, 60)),
                          4 * int(g.integers(2, 40)), C, R, S, int(g.choice([2, 2, 4])), int(g.integers(0, min(R, S))),
                          16 * int(g.integers(1, 5)))
        OH, OW = (L.H + 2 * L.pad - L.R) // L.stride + 1, (L.W + 2 * L.pad - L.S) // L.stride + 1
        if OH >= 1 and OW >= 1 and L.B * OH * OW * L.Cout * L.R * L.S * C < 4e8:
            shapes.append(L)
    return shapes


RGB = [
    wl.conv("rgb_stem", 2, 37, 3, 64, 7, stride=2),                      # the ResNet stem's geometry on a small odd image
    wl.conv("rgb_3x3", 3, 20, 3, 64, 3),                                 # VGG's first layer
    wl.conv("rgb_3x3_n16", 1, 9, 3, 16, 3, stride=1, pad=0),             # one column group, no padding
    wl.conv("rgb_5x5_s3", 2, 23, 3, 48, 5, stride=3, pad=1),             # ragged channel block
    wl.LayerShape("rgb_7x10", wl.CONV, 2, 15, 31, 3, 7, 10, 2, 4, 32),   # widest filter row the kernel takes (30 bytes)
    wl.LayerShape("rgb_w1", wl.CONV, 3, 12, 1, 3, 3, 1, 1, 0, 32),       # images one pixel wide
    wl.LayerShape("rgb_1x1", wl.CONV, 1, 5, 7, 3, 1, 1, 1, 0, 16),       # a word holds one pixel and a byte of the next
    wl.conv("rgb_one_pixel", 1, 1, 3, 16, 3),                            # 3 bytes of input in all: every word reaches past the tensor
    # rows staged in LDS (even stride, width a multiple of 4): several bands per image with a short last one
    wl.LayerShape("rgb_staged_224x100", wl.CONV, 1, 100, 224, 3, 7, 7, 2, 3, 64),
    wl.LayerShape("rgb_staged_s2_w28", wl.CONV, 3, 18, 28, 3, 5, 5, 2, 2, 48),   # ragged channel block, one band per image
    wl.LayerShape("rgb_staged_s4", wl.CONV, 2, 21, 16, 3, 3, 8, 4, 1, 16),       # stride 4, eight taps per filter row (the most)
    wl.LayerShape("rgb_s4_nine_taps", wl.CONV, 2, 21, 16, 3, 3, 9, 4, 1, 16),    # nine taps: not staged
    wl.LayerShape("c4_staged_224x60", wl.CONV, 1, 60, 224, 4, 7, 7, 2, 3, 64),   # the same kernel on 4-byte pixels
    wl.LayerShape("c4_staged_s2_w12", wl.CONV, 5, 9, 12, 4, 3, 8, 2, 0, 32),     # widest filter row (32 bytes), no padding
]


RGB += random_staged_first_layers(16, 31, 3)


@pytest.mark.parametrize("L", RGB, ids=["%s_b%d_%dx%d_%dx%d_s%d_p%d_n%d" % (l.name, l.B, l.H, l.W, l.R, l.S, l.stride, l.pad, l.Cout) for l in RGB])
@pytest.mark.parametrize("g_asym", [False, True], ids=["gsym", "gasym"])
def test_rgb_first_layer(H, hq, L, g_asym):
    y_track = H.TensorTrack(0.9, False)
    Wdev = None
    for t in range(3):
        g = np.random.default_rng([77, t])
        X = wl.normal_image(g, wl.in_shape(L))                            # signed image, zero point inside the grid
        W = wl.he_weight(g, L)
        if g_asym:
            dY = wl.to_asymmetric_codes(g.laplace(0, 1e-3, wl.out_shape(L)).astype(np.float32) + np.float32(4e-4))
        else:
            dY = wl.laplace_gradient(g, wl.out_shape(L), 1e-3)
        if Wdev is None:
            W0, Wdev = W, H.DevWeights(L, W)
        Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
        y_track.step(L, "fwd", X, W0, Xd, Wdev)                           # t = 0 dynamic, then fused
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref)
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))
    if L.C != 3:
        return
    # the input gradient of a 3-channel layer is refused, not computed wrongly
    with pytest.raises(hq.HqError) as e:
        H.gpu_quantized_op(L, "dgrad", dYd, Wdev, hq.new_range(0.9, True), hq.new_stats(1), "fused")
    assert e.value.code == hq.HQ_E_BADSHAPE


@pytest.mark.parametrize("L", [wl.LayerShape("rgb_wgrad_9x2_n72", wl.CONV, 2, 17, 11, 3, 9, 2, 1, 1, 72),     # more filter rows and output channels than the forward kernel takes
                               wl.LayerShape("rgb_wgrad_2x10_n4", wl.CONV, 1, 6, 24, 3, 2, 10, 2, 0, 4)], ids=lambda l: l.name)
def test_rgb_weight_gradient_beyond_the_forward_limits(H, hq, L):
    """The weight gradient of a 3-channel layer takes any filter height and any output channel count that is a
    multiple of 4; the forward call refuses the same shape instead of computing it wrongly."""
    g = np.random.default_rng([78, L.R])
    X = wl.normal_image(g, wl.in_shape(L))
    dY = wl.to_asymmetric_codes(g.laplace(0, 1e-3, wl.out_shape(L)).astype(np.float32) + np.float32(4e-4))
    Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
    dW, dWa = H.gpu_wgrad(L, Xd, dYd)
    ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
    assert np.array_equal(dWa, ref)
    assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))
    Wdev = H.DevWeights(L, wl.he_weight(g, L))
    with pytest.raises(hq.HqError) as e:
        H.gpu_quantized_op(L, "fwd", Xd, Wdev, hq.new_range(0.9, False), hq.new_stats(1), "fused")
    assert e.value.code == hq.HQ_E_BADSHAPE


def random_shapes(n, seed):
    """Seeded random layer shapes inside the documented limits (channels % 4 == 0, pad < filter size,
    at least one output pixel): non-square images and filters, strides 1..3, channel counts around the
    kernels' tile sizes.  Small enough for the oracle."""
    g = np.random.default_rng(seed)
    chans = [4, 8, 12, 16, 20, 24, 32, 36, 48, 64, 64, 72, 96, 128, 128, 132, 192, 256]
    shapes = []
    while len(shapes) < n:
        kind = g.choice([wl.CONV, wl.CONV, wl.CONV, wl.LINEAR, wl.DEPTHWISE])
        i = len(shapes)
        if kind == wl.LINEAR:
            shapes.append(wl.LayerShape("rnd%d_lin" % i, wl.LINEAR, int(g.integers(1, 400)), 1, 1, int(g.choice(chans)) * int(g.integers(1, 3)),
                                        1, 1, 1, 0, int(g.choice(chans))))
            continue
        R, S = (int(g.choice([1, 2, 3, 3, 3, 5])),) * 2 if g.random() < 0.7 else (int(g.integers(1, 5)), int(g.integers(1, 5)))
        if kind == wl.DEPTHWISE:
            R = S = 3
        pad = int(g.integers(0, min(R, S)))
        stride = int(g.choice([1, 1, 1, 2, 2, 3]))
        Hh, Ww = int(g.integers(max(R - 2 * pad, 1), 26)), int(g.integers(max(S - 2 * pad, 1), 26))
        C = int(g.choice(chans))
        Cout = C if kind == wl.DEPTHWISE else int(g.choice(chans))
        if kind == wl.DEPTHWISE and pad != 1:
            pad = 1
        B = int(g.integers(1, 5))
        OH, OW = (Hh + 2 * pad - R) // stride + 1, (Ww + 2 * pad - S) // stride + 1
        if OH < 1 or OW < 1 or B * OH * OW * Cout * R * S * (1 if kind == wl.DEPTHWISE else C) > 60e6:
            continue
        shapes.append(wl.LayerShape("rnd%d_%s" % (i, "dw" if kind == wl.DEPTHWISE else "conv"), int(kind), B, Hh, Ww, C, R, S,
                                    stride, pad, Cout))
    return shapes


def random_fast_path_shapes(n, seed):
    """Seeded random geometry for the shapes the specialised kernels take: 3x3 with 64 input channels
    (weights in LDS, bands and tiles of all lengths), 1x1 with 32 / 192, 3x3 with 128+ channels on both
    sides (streamed weights), 4-channel first layers, depthwise strips, and the banded weight gradient."""
    g = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < n:
        fam = int(g.integers(0, 6))
        i = len(shapes)
        B = int(g.choice([1, 2, 3, 5, 17, 64, 130, 257]))
        Hh, Ww = int(g.integers(3, 41)), int(g.integers(3, 41))
        if fam == 0:      # weights-resident 3x3
            L = wl.LayerShape("fp%d_band3" % i, wl.CONV, B, Hh, Ww, 64, 3, 3, int(g.choice([1, 1, 2])), int(g.integers(0, 3)),
                              16 * int(g.integers(1, 6)))
        elif fam == 1:    # weights-resident 1x1
            L = wl.LayerShape("fp%d_band1" % i, wl.CONV, B, Hh, Ww, int(g.choice([32, 192])), 1, 1, int(g.choice([1, 1, 2])), 0,
                              16 * int(g.integers(1, 14)))
        elif fam == 2:    # streamed weights
            L = wl.LayerShape("fp%d_bandw" % i, wl.CONV, B, Hh, Ww, 64 * int(g.integers(2, 5)), 3, 3, 1, 1, 16 * int(g.integers(8, 17)))
        elif fam == 3:    # first layer
            S = int(g.integers(1, 9))
            R = int(g.integers(1, 8))
            L = wl.LayerShape("fp%d_first" % i, wl.CONV, B, Hh + 6, Ww + 6, 4, R, S, int(g.integers(1, 4)), int(g.integers(0, min(R, S))),
                              16 * int(g.integers(1, 5)))
        elif fam == 4:    # depthwise strips
            L = wl.LayerShape("fp%d_dw" % i, wl.DEPTHWISE, B, Hh + 20, Ww + 20, 4 * int(g.integers(1, 81)), 3, 3, int(g.choice([1, 2])), 1, 0)
            L = L._replace(Cout=L.C)
        else:             # banded weight gradient (also 3x3 forward paths)
            L = wl.LayerShape("fp%d_wband" % i, wl.CONV, B, Hh, Ww, 64 * int(g.integers(1, 4)), 3, 3, 1, 1, 64 * int(g.integers(1, 4)))
        OH, OW = (L.H + 2 * L.pad - L.R) // L.stride + 1, (L.W + 2 * L.pad - L.S) // L.stride + 1
        macs = L.B * OH * OW * L.Cout * L.R * L.S * (1 if L.kind == wl.DEPTHWISE else L.C)
        if OH < 1 or OW < 1 or macs > 1.0e9 or L.B * L.H * L.W * L.C > 3e7:
            continue
        shapes.append(L)
    return shapes


def random_wide_band_shapes(n, seed):
    """3x3 layers with 64 input channels on images 58 .. 132 pixels wide: around the two patch-row widths
    of the weights-resident kernel (64 and 126 output pixels at stride 1) and past them (gather kernel)."""
    g = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < n:
        L = wl.LayerShape("wide%d" % len(shapes), wl.CONV, int(g.choice([1, 2, 3])), int(g.integers(3, 14)), int(g.integers(58, 133)),
                          64, 3, 3, int(g.choice([1, 1, 2])), int(g.integers(0, 3)), 16 * int(g.integers(1, 6)))
        OH, OW = (L.H + 2 * L.pad - 3) // L.stride + 1, (L.W + 2 * L.pad - 3) // L.stride + 1
        if OH >= 1 and OW >= 1:
            shapes.append(L)
    return shapes


RANDOM = (random_shapes(40, 20260) + random_shapes(50, 7) + random_fast_path_shapes(48, 11) + random_wide_band_shapes(12, 5) +
          random_staged_first_layers(16, 32, 4))


@pytest.mark.parametrize("L", RANDOM, ids=["%s_b%d_%dx%d_c%d_%dx%d_s%d_p%d_n%d" % (l.name, l.B, l.H, l.W, l.C, l.R, l.S, l.stride, l.pad, l.Cout)
                                           for l in RANDOM])
def test_random_shapes_all_ops(H, hq, L):
    # every third shape with the zero point on the gradient side instead of the input side
    swap = sum(map(ord, L.name)) % 3 == 0
    y_track, g_track = H.TensorTrack(0.9, swap), H.TensorTrack(0.9, not swap)
    Wdev = None
    for t in range(2):
        X, W, dY = rand_layer_inputs(L, 3000 + t, x_asym=not swap, g_asym=swap)
        if Wdev is None:
            W0, Wdev = W, H.DevWeights(L, W)
        Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
        y_track.step(L, "fwd", X, W0, Xd, Wdev)
        # the fused iteration of every other shape rounds the input gradient stochastically
        g_track.step(L, "dgrad", dY, W0, dYd, Wdev, seed=0xabcdef12345 + L.B if t == 1 and len(L.name) % 2 else None)
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref)
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


def test_weight_prepare_layouts_and_sums(H, hq):
    L = wl.conv("prep", 1, 6, 24, 40, 3)
    W = wl.he_weight(np.random.default_rng(5), L)
    Wd = H.DevWeights(L, W)
    torch.cuda.synchronize()
    w = W.codes.astype(np.int64)
    assert np.array_equal(Wd.wsum.cpu().numpy(), w.sum(axis=(1, 2, 3)))
    assert np.array_equal(Wd.wdsum.cpu().numpy(), w.sum(axis=(0, 1, 2)))
    assert np.array_equal(Wd.Wd.cpu().numpy().reshape(L.C, L.R, L.S, L.Cout), W.codes.transpose(3, 1, 2, 0))


@pytest.mark.parametrize("n", [1, 3, 36864, 147456 + 5, 2359296])
def test_weight_quantizer(H, hq, n):
    """Q_W with the tensor's current min-max (Sec. 3.1, Sec. 5): codes and scale bit for bit."""
    g = np.random.default_rng(n)
    for w in ((g.standard_normal(n) * 0.05).astype(np.float32), np.zeros(n, np.float32),
              (g.standard_normal(n) * 1e-3 + 0.7).astype(np.float32)):
        want, s = oracle.quantize_weights(w)
        Wf = H.dev(w)
        Wq = torch.empty(n, dtype=torch.int8, device="cuda")
        wq = hq.new_qparams(123.0, 7)
        hq.hq_weight_quantize(Wf, n, Wq, wq)
        torch.cuda.synchronize()
        q = H.read_qparams(wq)
        assert np.float32(q["scale"]) == s and int(q["zero_point"]) == 0
        assert np.array_equal(Wq.cpu().numpy(), want)


def test_asymmetric_gradients_and_symmetric_inputs(H, hq):
    """Zero points on the gradient side (the paper quantizes gradients asymmetrically in its
    ablations, Sec. 5.1) and none on the input side."""
    for L in (wl.conv("asym_g", 2, 8, 16, 32, 3), wl.conv("asym_g_s2", 1, 9, 32, 16, 3, stride=2),
              wl.depthwise("asym_dw", 2, 9, 24),
              wl.conv("asym_wband_img", 5, 7, 64, 128, 3),     # weight-gradient bands of 4 images, last one short
              wl.conv("asym_wband_rows", 2, 20, 128, 64, 3)):  # bands of rows with pixels past the band's end
        X, W, dY = rand_layer_inputs(L, 77, x_asym=False, g_asym=True)
        assert dY.zero_point != 0 and X.zero_point == 0
        Wdev, Xd, dYd = H.DevWeights(L, W), H.DevTensor(X), H.DevTensor(dY)
        g_track = H.TensorTrack(0.9, symmetric=False)
        for _ in range(2):
            g_track.step(L, "dgrad", dY, W, dYd, Wdev)
        y_track = H.TensorTrack(0.9, symmetric=True)
        for _ in range(2):
            y_track.step(L, "fwd", X, W, Xd, Wdev)
        for Xq, Xdev in ((X, Xd), (wl.relu_activation(np.random.default_rng(3), wl.in_shape(L)), None)):
            Xdev = Xdev or H.DevTensor(Xq)
            dW, dWa = H.gpu_wgrad(L, Xdev, dYd)
            ref = oracle.wgrad(H.oracle_problem(L), Xq.codes, Xq.zero_point, dY.codes, dY.zero_point)
            assert np.array_equal(dWa, ref)
            assert np.array_equal(dW, oracle.wgrad_scale(ref, Xq.scale, dY.scale))


# ---------------------------------------------------------------------------------------
# Depthwise (config 4's middle layer, small)
# ---------------------------------------------------------------------------------------
DW = [wl.depthwise("dw3", 2, 11, 24), wl.depthwise("dw3_s2", 2, 12, 32, stride=2),
      wl.depthwise("dw3_192", 1, 14, 192), wl.depthwise("dw3_320", 1, 7, 320)]


@pytest.mark.parametrize("L", DW, ids=[l.name for l in DW])
def test_depthwise_all_ops(H, hq, L):
    y_track, g_track = H.TensorTrack(0.9, False), H.TensorTrack(0.9, True)
    X0, W, dY0 = rand_layer_inputs(L, 31)
    Wdev = H.DevWeights(L, W)
    for t in range(3):
        X, _, dY = rand_layer_inputs(L, 31 + t)
        Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
        y_track.step(L, "fwd", X, W, Xd, Wdev)
        g_track.step(L, "dgrad", dY, W, dYd, Wdev)
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref)
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


# ---------------------------------------------------------------------------------------
# Invariants on the GPU path
# ---------------------------------------------------------------------------------------
def test_fused_with_current_range_equals_dynamic(H, hq):
    """Sec. 3.2: static and dynamic quantization differ only in when the range is known."""
    L = wl.conv("p5", 2, 14, 32, 64, 3)
    X, W, _ = rand_layer_inputs(L, 9)
    Wdev, Xd = H.DevWeights(L, W), H.DevTensor(X)
    for sym in (False, True):
        r, st = hq.new_range(0.9, sym), hq.new_stats()
        dyn_codes, dyn_q = H.gpu_quantized_op(L, "fwd", Xd, Wdev, r, st, "dynamic")   # also sets q^0 = current min-max
        st_dyn = H.read_stats(st)
        hq.hq_stats_reset(st)
        codes, q = H.gpu_quantized_op(L, "fwd", Xd, Wdev, r, st, "fused")
        st_f = H.read_stats(st)
        assert np.array_equal(codes, dyn_codes) and q == dyn_q
        for f in ("acc_min", "acc_max", "clip_lo", "clip_hi", "count"):
            assert st_f[f] == st_dyn[f]
        assert st_f["clip_lo"] == 0 and st_f["clip_hi"] == 0


def test_running_min_max_mode(H, hq):
    """Sec. 4.1, last paragraph: eq. (2)-(3) with the current tensor's statistics, then quantize."""
    L = wl.linear("run", 64, 64, 32)
    r, st = hq.new_range(0.9, False), hq.new_stats()
    ref = oracle.Range.new(0.9, False)
    for t in range(3):
        g = np.random.default_rng(50 + t)
        X = wl.relu_activation(g, wl.in_shape(L), gain=1.5 ** t)
        W = wl.he_weight(np.random.default_rng(50), L)
        Wdev, Xd = H.DevWeights(L, W), H.DevTensor(X)
        codes, q = H.gpu_quantized_op(L, "fwd", Xd, Wdev, r, st, "dynamic", hq.HQ_DYN_RUNNING)
        stats = H.read_stats(st)
        hq.hq_stats_reset(st)
        c = H.oracle_acc(L, "fwd", X, W)
        a_scale = oracle.acc_scale(X.scale, W.scale)
        mn, mx = oracle.minmax(c)
        oracle.range_update(ref, mn, mx, a_scale)
        want, lo, hi = oracle.requant(c, a_scale, ref.scale, ref.zero_point, ref.qlo, ref.qhi)
        assert np.array_equal(codes, want)
        assert (int(stats["clip_lo"]), int(stats["clip_hi"])) == (lo, hi)
        H.assert_range_close(H.read_range(r), ref)


@pytest.mark.parametrize("L", [wl.conv("dynsr_band", 2, 20, 64, 64, 3), wl.conv("dynsr_gemm", 2, 9, 24, 40, 3),
                               wl.conv("dynsr_s2", 2, 12, 32, 48, 3, stride=2), wl.depthwise("dynsr_dw", 2, 13, 48),
                               wl.linear("dynsr_lin", 37, 72, 80)], ids=lambda l: l.name)
def test_dynamic_estimators_with_stochastic_rounding(H, hq, L):
    """The two dynamic estimators on the input gradient with stochastic rounding in the second
    pass: current min-max (eq. (1)) and running min-max (Sec. 4.1), three iterations each, codes,
    quantizer, clip counts and range state against the oracle with the same seeds."""
    for mode in ("current", "running"):
        r, st, ref = hq.new_range(0.9, True), hq.new_stats(), oracle.Range.new(0.9, True)
        Wdev, W0 = None, None
        for t in range(3):
            X, W, dY = rand_layer_inputs(L, 880 + t)
            dY = wl.QTensor(dY.codes, np.float32(dY.scale * 0.7 ** t), dY.zero_point)      # shrinking gradients
            if Wdev is None:
                W0, Wdev = W, H.DevWeights(L, W)
            seed = 0xd1b54a32d192ed03 * (t + 1) % 2 ** 64
            codes, q = H.gpu_quantized_op(L, "dgrad", H.DevTensor(dY), Wdev, r, st, "dynamic",
                                          hq.HQ_DYN_RUNNING if mode == "running" else hq.HQ_DYN_CURRENT, seed=seed)
            stats = H.read_stats(st)
            if mode == "current":
                hq.hq_range_update(r, st)
            else:
                hq.hq_stats_reset(st)
            c = H.oracle_acc(L, "dgrad", dY, W0)
            a_scale = oracle.acc_scale(dY.scale, W0.scale)
            mn, mx = oracle.minmax(c)
            if mode == "running":
                oracle.range_update(ref, mn, mx, a_scale)
                want, lo, hi = oracle.requant_stochastic(c, a_scale, ref.scale, ref.zero_point, ref.qlo, ref.qhi, seed)
                ws, wz = np.float32(ref.scale), ref.zero_point
            else:
                if not ref.initialized:
                    oracle.range_update(ref, mn, mx, a_scale)
                o = oracle.quantize_dynamic(c, a_scale, True, ref.qlo, ref.qhi, seed)
                want, lo, hi, ws, wz = o["codes"], o["clip_lo"], o["clip_hi"], o["scale"], o["zero_point"]
                oracle.range_update(ref, mn, mx, a_scale)
            assert np.float32(q["scale"]) == ws and int(q["zero_point"]) == wz
            assert np.array_equal(codes, want), int((codes != want).sum())
            assert (int(stats["clip_lo"]), int(stats["clip_hi"])) == (lo, hi)
            H.assert_range_close(H.read_range(r), ref)
        nearest, _ = H.gpu_quantized_op(L, "dgrad", H.DevTensor(dY), Wdev, r, st, "dynamic", hq.HQ_DYN_CURRENT)
        hq.hq_stats_reset(st)
        if mode == "current":
            assert not np.array_equal(nearest, codes) and np.abs(nearest.astype(int) - codes.astype(int)).max() <= 1


def test_statistics_merge_until_consumed(H, hq):
    """Two launches into the same statistics record give the union; hq_range_update with an
    empty record leaves the range alone."""
    L = wl.linear("merge", 96, 32, 32)
    W = wl.he_weight(np.random.default_rng(1), L)
    Wdev = H.DevWeights(L, W)
    r, st = hq.new_range(0.9, False), hq.new_stats()
    Xs = [wl.relu_activation(np.random.default_rng(s), wl.in_shape(L), gain=g) for s, g in ((1, 1.0), (2, 3.0))]
    H.gpu_quantized_op(L, "fwd", H.DevTensor(Xs[0]), Wdev, r, st, "dynamic")
    hq.hq_range_update(r, st)
    before = H.read_range(r).copy()
    hq.hq_range_update(r, st)                      # empty record: no change
    assert H.read_range(r) == before
    mins, maxs = [], []
    for X in Xs:
        H.gpu_quantized_op(L, "fwd", H.DevTensor(X), Wdev, r, st, "fused")
        mn, mx = oracle.minmax(H.oracle_acc(L, "fwd", X, W))
        mins.append(mn); maxs.append(mx)
    s = H.read_stats(st)
    assert int(s["acc_min"]) == min(mins) and int(s["acc_max"]) == max(maxs) and int(s["count"]) == 2 * 96 * 32


def test_repeat_runs_are_bit_identical(H, hq):
    L = wl.conv("rep", 2, 14, 64, 64, 3)
    X, W, dY = rand_layer_inputs(L, 4)
    Wdev, Xd, dYd = H.DevWeights(L, W), H.DevTensor(X), H.DevTensor(dY)
    r, st = hq.new_range(0.9, False), hq.new_stats()
    H.gpu_quantized_op(L, "fwd", Xd, Wdev, r, st, "dynamic")
    outs = []
    for _ in range(3):
        hq.hq_stats_reset(st)
        codes, _ = H.gpu_quantized_op(L, "fwd", Xd, Wdev, r, st, "fused")
        outs.append((codes, H.read_stats(st), H.gpu_wgrad(L, Xd, dYd)[1]))
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0]) and o[1] == outs[0][1] and np.array_equal(o[2], outs[0][2])


# ---------------------------------------------------------------------------------------
# Stochastic rounding of the input gradient (the paper's gradient quantizer, Sec. 5)
# ---------------------------------------------------------------------------------------
SR_SHAPES = [wl.conv("sr_c64", 2, 20, 64, 64, 3),                 # weights-resident kernel, one-row bands
             wl.conv("sr_band_tiles", 128, 36, 64, 64, 3),        # ... two tiles per band, the second ragged
             wl.conv("sr_band_n48", 2, 17, 48, 64, 3),            # ... ragged column tile (dX has 48 channels)
             wl.conv("sr_band_1x1", 2, 20, 192, 32, 1),           # ... 1x1, three column chunks (reduction over 32)
             wl.conv("sr_band_1x1_c192", 2, 20, 32, 192, 1),      # ... 1x1, reduction over 192
             wl.conv("sr_n64", 2, 20, 64, 48, 3),                 # general kernel, 256 x 64 tiles
             wl.conv("sr_c128", 2, 14, 128, 128, 3),              # streamed-weights kernel
             wl.conv("sr_bandw_rows", 2, 30, 128, 192, 3),        # ... tiles of rows, last one short; dX has 128 channels
             wl.conv("sr_bandw_imgs", 3, 10, 192, 128, 3),        # ... tiles of whole images, ragged channel chunk
             wl.conv("sr_c128_s2", 2, 14, 128, 128, 3, stride=2), # general kernel, 128 x 128 tiles
             wl.conv("sr_s2", 2, 12, 32, 48, 3, stride=2),        # strided classes
             wl.conv("sr_c24", 1, 9, 24, 40, 3),                  # 4-byte reduction path, ragged column groups
             wl.conv("sr_n8", 3, 7, 16, 8, 1, pad=0),             # fewer than 16 output columns... of dX: C = 16
             wl.linear("sr_lin", 300, 72, 80),
             wl.LayerShape("sr_c5x5_s3", wl.CONV, 2, 17, 17, 16, 5, 5, 3, 2, 32),
             wl.depthwise("sr_dw", 2, 13, 48), wl.depthwise("sr_dw_s2", 2, 12, 32, stride=2)]


@pytest.mark.parametrize("L", SR_SHAPES, ids=[l.name for l in SR_SHAPES])
def test_stochastic_rounding_dgrad(H, hq, L):
    """Codes, clip counts and statistics bit for bit against the oracle with the same seed per
    iteration; the seed changes the codes, the tiling does not enter (the oracle has none)."""
    for g_asym in (False, True):
        g_track = H.TensorTrack(0.9, symmetric=not g_asym)
        Wdev, W0 = None, None
        for t in range(3):
            X, W, dY = rand_layer_inputs(L, 500 + t, g_asym=g_asym)
            if Wdev is None:
                W0, Wdev = W, H.DevWeights(L, W)
            dYd = H.DevTensor(dY)
            g_track.step(L, "dgrad", dY, W0, dYd, Wdev, seed=0x9e3779b97f4a7c15 * (t + 1) % 2**64)
        # same tensor, same range, two seeds: different codes, never more than one step apart
        a, _ = H.gpu_quantized_op(L, "dgrad", dYd, Wdev, g_track.r, g_track.st, seed=1)
        b, _ = H.gpu_quantized_op(L, "dgrad", dYd, Wdev, g_track.r, g_track.st, seed=2)
        hq.hq_stats_reset(g_track.st)
        assert not np.array_equal(a, b) and np.abs(a.astype(int) - b.astype(int)).max() <= 1


def _real_batch(kind, n, t, seed):
    g = np.random.default_rng([seed, t, n])
    if kind == "act":
        return wl.real_activation(g, n, gain=1.05 ** t)
    return wl.real_gradient(g, n, 1e-3 * 0.8 ** t)


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 4096 * 3 + 5, 1_000_003])
@pytest.mark.parametrize("kind", ["act", "grad"])
def test_real_tensor_in_hindsight_quantizer(H, hq, n, kind):
    """Element-wise quantizer of FP32 tensors over four iterations (dynamic for the first batch, then
    in hindsight): codes, quantizer, clip counts, minimum / maximum bit for bit; range state after
    each update within 1e-6."""
    sym = kind == "grad"
    r, st = hq.new_range(0.9, sym), hq.new_stats(1)
    ref = oracle.Range.new(0.9, sym)
    Q = torch.empty(max(n, 1), dtype=torch.int8, device="cuda")
    qp = hq.new_qparams(0.0, 99)
    for t in range(4):
        x = _real_batch(kind, n, t, 31)
        xd = torch.from_numpy(x).cuda()
        if n == 0:
            hq.hq_tensor_quantize(xd, 0, r, Q, qp, st)
            assert int(H.read_stats(st)["count"]) == 0
            hq.hq_range_update(r, st)
            assert int(H.read_range(r)["initialized"]) == 0
            hq.hq_tensor_quantize_dynamic(hq.HQ_DYN_CURRENT, xd, 0, r, Q, qp, st)
            got = H.read_qparams(qp)
            assert float(got["scale"]) == 1.0 and int(got["zero_point"]) == 0
            continue
        seed = (0x9e3779b97f4a7c15 * (t + 1)) % 2 ** 64 if kind == "grad" and t >= 2 else None   # gradients: the last two rounded stochastically
        want = oracle.tensor_step(x, ref, "hindsight", seed)
        if t == 0:
            hq.hq_tensor_quantize_dynamic(hq.HQ_DYN_CURRENT, xd, n, r, Q, qp, st)
        elif seed is not None:
            hq.hq_tensor_quantize_sr(xd, n, r, seed, Q, qp, st)
        else:
            hq.hq_tensor_quantize(xd, n, r, Q, qp, st)
        got_st, got_qp = H.read_stats(st), H.read_qparams(qp)
        hq.hq_range_update(r, st)
        codes = Q[:n].cpu().numpy()
        assert np.float32(got_qp["scale"]) == want["scale"] and int(got_qp["zero_point"]) == want["zero_point"]
        assert np.array_equal(codes, want["codes"]), int((codes != want["codes"]).sum())
        assert int(got_st["fp32_keys"]) == 1 and int(got_st["count"]) == n
        assert (int(got_st["clip_lo"]), int(got_st["clip_hi"])) == (want["clip_lo"], want["clip_hi"])
        key = lambda k: np.array([k ^ ((k >> 31) & 0x7fffffff)], np.int32).view(np.float32)[0]
        assert key(int(got_st["acc_min"])) == want["min"] and key(int(got_st["acc_max"])) == want["max"]
        H.assert_range_close(H.read_range(r), ref)
        assert int(H.read_stats(st)["count"]) == 0 and int(H.read_stats(st)["fp32_keys"]) == 0
        if t >= 2 and n > 1000 and kind == "act":
            assert want["clip_hi"] > 0                      # growing activations: the past range clips


@pytest.mark.parametrize("mode", ["current", "running"])
def test_real_tensor_dynamic_quantizers(H, hq, mode):
    """eq. (1) and the running variant on FP32 tensors, asymmetric and symmetric, 4- and 8-bit grids."""
    n = 70_001
    for sym, bits in [(False, 8), (True, 8), (False, 4), (True, 4)]:
        r, st = hq.new_range(0.9, sym, bits=bits), hq.new_stats(1)
        ref = oracle.Range.new(0.9, sym, bits)
        Q = torch.empty(n, dtype=torch.int8, device="cuda")
        qp = hq.new_qparams(0.0, 99)
        for t in range(3):
            x = _real_batch("grad" if sym else "act", n, t, 57)
            if not sym:
                x -= np.float32(0.3)                       # a range that does not start at zero
            want = oracle.tensor_step(x, ref, mode)
            hq.hq_tensor_quantize_dynamic(hq.HQ_DYN_RUNNING if mode == "running" else hq.HQ_DYN_CURRENT,
                                          torch.from_numpy(x).cuda(), n, r, Q, qp, st)
            got_st, got_qp = H.read_stats(st), H.read_qparams(qp)
            if mode == "current":
                hq.hq_range_update(r, st)
            else:
                hq.hq_stats_reset(st)
            assert np.float32(got_qp["scale"]) == want["scale"] and int(got_qp["zero_point"]) == want["zero_point"]
            assert np.array_equal(Q.cpu().numpy(), want["codes"])
            assert (int(got_st["clip_lo"]), int(got_st["clip_hi"])) == (want["clip_lo"], want["clip_hi"])
            H.assert_range_close(H.read_range(r), ref)


def test_two_layer_chain_runs_on_the_device_without_the_host(H, hq):
    """FP32 image -> Q_X -> conv -> conv -> (FP32 loss gradient -> Q_G) -> dgrad -> dgrad, both
    weight gradients, FP32 master weights through Q_W: every quantizer parameter is handed from
    call to call as a device pointer, all six range states are updated by one launch, and nothing
    is read back before the iteration's end.  Three iterations (the first dynamic), every tensor
    compared with the oracle doing the same chain."""
    L1, L2 = wl.conv("chain1", 3, 18, 16, 64, 3), wl.conv("chain2", 3, 18, 64, 64, 3)
    p1, p2 = H.hq_problem(L1), H.hq_problem(L2)
    o1, o2 = H.oracle_problem(L1), H.oracle_problem(L2)
    g = np.random.default_rng(99)
    Wf = [(g.standard_normal(wl.w_shape(L)) * np.sqrt(2.0 / (9 * L.C))).astype(np.float32) for L in (L1, L2)]
    # device state: ranges 0..5 = x0, y1, y2, g2 (loss gradient), g1, g0
    sym = [False, False, False, True, True, True]
    R, ST = hq.new_ranges(sym), hq.new_stats(6)
    rp = lambda i: R.data_ptr() + i * hq.RANGE.itemsize
    sp = lambda i: ST.data_ptr() + i * hq.STATS.itemsize
    refs = [oracle.Range.new(0.9, f) for f in sym]
    i8 = lambda shape: torch.empty(shape, dtype=torch.int8, device="cuda")
    qps = [hq.new_qparams(0.0, 0) for _ in range(6)]
    wq = [hq.new_qparams(0.0, 0) for _ in range(2)]
    Wq = [i8(w.shape) for w in Wf]
    Wd = [i8(w.size) for w in Wf]
    wsum = [torch.empty(L.Cout, dtype=torch.int32, device="cuda") for L in (L1, L2)]
    wdsum = [torch.empty(L.C, dtype=torch.int32, device="cuda") for L in (L1, L2)]
    ws_n = max(hq.hq_workspace_bytes(e, p) for e in (hq.HQ_ENTRY_WGRAD, hq.HQ_ENTRY_DYNAMIC_FWD, hq.HQ_ENTRY_DYNAMIC_DGRAD)
               for p in (p1, p2))
    ws = torch.empty(ws_n, dtype=torch.uint8, device="cuda")
    x0q, y1, y2 = i8(wl.in_shape(L1)), i8(wl.out_shape(L1)), i8(wl.out_shape(L2))
    g2, g1, g0 = i8(wl.out_shape(L2)), i8(wl.in_shape(L2)), i8(wl.in_shape(L1))
    dW = [torch.empty(w.shape, dtype=torch.float32, device="cuda") for w in Wf]
    dWa = [torch.empty(w.shape, dtype=torch.int32, device="cuda") for w in Wf]
    for t in range(3):
        x0 = (g.standard_normal(wl.in_shape(L1)) * 1.1 ** t).astype(np.float32)
        gl = wl.real_gradient(g, wl.nelem(wl.out_shape(L2)), 1e-3 * 0.7 ** t).reshape(wl.out_shape(L2))
        for w in Wf:
            w *= np.float32(0.97)                                   # the master weights move
        # ---- device: one stream, no synchronisation inside the iteration
        x0d, gld = torch.from_numpy(x0).cuda(), torch.from_numpy(gl).cuda()
        for k, p in enumerate((p1, p2)):
            hq.hq_weight_quantize(torch.from_numpy(Wf[k]).cuda(), Wf[k].size, Wq[k], wq[k])
            hq.hq_weight_prepare(p, Wq[k], Wd[k], wsum[k], wdsum[k])
        if t == 0:
            dyn = hq.HQ_DYN_CURRENT
            hq.hq_tensor_quantize_dynamic(dyn, x0d, x0.size, rp(0), x0q, qps[0], sp(0))
            hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_FWD, dyn, p1, x0q, qps[0], Wq[0], wq[0], wsum[0], rp(1), y1, qps[1], sp(1), ws, ws_n)
            hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_FWD, dyn, p2, y1, qps[1], Wq[1], wq[1], wsum[1], rp(2), y2, qps[2], sp(2), ws, ws_n)
            hq.hq_tensor_quantize_dynamic(dyn, gld, gl.size, rp(3), g2, qps[3], sp(3))
            hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_DGRAD, dyn, p2, g2, qps[3], Wd[1], wq[1], wdsum[1], rp(4), g1, qps[4], sp(4), ws, ws_n)
            hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_DGRAD, dyn, p1, g1, qps[4], Wd[0], wq[0], wdsum[0], rp(5), g0, qps[5], sp(5), ws, ws_n)
        else:
            hq.hq_tensor_quantize(x0d, x0.size, rp(0), x0q, qps[0], sp(0))
            hq.hq_gemm_fwd(p1, x0q, qps[0], Wq[0], wq[0], wsum[0], rp(1), y1, qps[1], sp(1))
            hq.hq_gemm_fwd(p2, y1, qps[1], Wq[1], wq[1], wsum[1], rp(2), y2, qps[2], sp(2))
            hq.hq_tensor_quantize(gld, gl.size, rp(3), g2, qps[3], sp(3))
            hq.hq_gemm_dgrad(p2, g2, qps[3], Wd[1], wq[1], wdsum[1], rp(4), g1, qps[4], sp(4))
            hq.hq_gemm_dgrad(p1, g1, qps[4], Wd[0], wq[0], wdsum[0], rp(5), g0, qps[5], sp(5))
        hq.hq_gemm_wgrad(p2, y1, qps[1], g2, qps[3], dW[1], dWa[1], ws, ws_n)
        hq.hq_gemm_wgrad(p1, x0q, qps[0], g1, qps[4], dW[0], dWa[0], ws, ws_n)
        hq.hq_range_update_batch(R, ST, 6)
        torch.cuda.synchronize()
        # ---- oracle: the same chain
        wc = [oracle.quantize_weights(w) for w in Wf]
        ox0 = oracle.tensor_step(x0, refs[0])
        oy1 = oracle.in_hindsight_step(oracle.fwd(o1, ox0["codes"], ox0["zero_point"], wc[0][0]),
                                       oracle.acc_scale(ox0["scale"], wc[0][1]), refs[1])
        oy2 = oracle.in_hindsight_step(oracle.fwd(o2, oy1["codes"], oy1["zero_point"], wc[1][0]),
                                       oracle.acc_scale(oy1["scale"], wc[1][1]), refs[2])
        og2 = oracle.tensor_step(gl, refs[3])
        og1 = oracle.in_hindsight_step(oracle.dgrad(o2, og2["codes"], og2["zero_point"], wc[1][0]),
                                       oracle.acc_scale(og2["scale"], wc[1][1]), refs[4])
        og0 = oracle.in_hindsight_step(oracle.dgrad(o1, og1["codes"], og1["zero_point"], wc[0][0]),
                                       oracle.acc_scale(og1["scale"], wc[0][1]), refs[5])
        odw2 = oracle.wgrad(o2, oy1["codes"], oy1["zero_point"], og2["codes"], og2["zero_point"])
        odw1 = oracle.wgrad(o1, ox0["codes"], ox0["zero_point"], og1["codes"], og1["zero_point"])
        for name, dev_t, want in (("x0", x0q, ox0), ("y1", y1, oy1), ("y2", y2, oy2), ("g2", g2, og2), ("g1", g1, og1), ("g0", g0, og0)):
            got = dev_t.cpu().numpy()
            assert np.array_equal(got, want["codes"].reshape(got.shape)), (t, name, int((got != want["codes"].reshape(got.shape)).sum()))
        for k, want in enumerate((ox0, oy1, oy2, og2, og1, og0)):
            q = H.read_qparams(qps[k])
            assert np.float32(q["scale"]) == want["scale"] and int(q["zero_point"]) == want["zero_point"], (t, k)
        assert np.array_equal(dWa[1].cpu().numpy(), odw2) and np.array_equal(dWa[0].cpu().numpy(), odw1)
        assert np.array_equal(dW[1].cpu().numpy(), oracle.wgrad_scale(odw2, oy1["scale"], og2["scale"]))
        assert np.array_equal(dW[0].cpu().numpy(), oracle.wgrad_scale(odw1, ox0["scale"], og1["scale"]))
        rr = hq.from_device(R, hq.RANGE)
        for k in range(6):
            H.assert_range_close(rr[k], refs[k])


@pytest.mark.parametrize("L", [wl.conv("graph_band", 4, 20, 64, 64, 3), wl.conv("graph_gemm", 2, 9, 24, 40, 3),
                               wl.depthwise("graph_dw", 2, 13, 48)], ids=lambda l: l.name)
def test_side_stream_and_graph_replay(H, hq, L):
    """The library only launches kernels on the stream it is handed (no allocation, no memset, no
    synchronisation), so a layer step can run on a side stream and be captured into a graph.  Three
    eager steps on the default stream give the expected sequence (the range state moves every step);
    the same step captured once on a side stream and replayed three times, with other work and
    synchronisations between the replays, must reproduce it bit for bit."""
    X, W, dY = rand_layer_inputs(L, 4242)
    Wdev, Xd, dYd = H.DevWeights(L, W), H.DevTensor(X), H.DevTensor(dY)
    p = H.hq_problem(L)
    R, ST = hq.new_ranges([False, True]), hq.new_stats(2)
    rs, ss = hq.RANGE.itemsize, hq.STATS.itemsize
    Y = torch.empty(wl.out_shape(L), dtype=torch.int8, device="cuda")
    dX = torch.empty(wl.in_shape(L), dtype=torch.int8, device="cuda")
    dW = torch.empty(wl.w_shape(L), dtype=torch.float32, device="cuda")
    yq, dxq = hq.new_qparams(0, 0), hq.new_qparams(0, 0)
    nws = max(hq.hq_workspace_bytes(e, p) for e in (hq.HQ_ENTRY_WGRAD, hq.HQ_ENTRY_DYNAMIC_FWD, hq.HQ_ENTRY_DYNAMIC_DGRAD))
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    # initialise both ranges dynamically, then keep that state as the common starting point
    hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_FWD, hq.HQ_DYN_CURRENT, p, Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, R[:rs], Y, yq, ST[:ss], ws, nws)
    hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_DGRAD, hq.HQ_DYN_CURRENT, p, dYd.codes, dYd.qp, Wdev.Wd, Wdev.qp, Wdev.wdsum, R[rs:], dX, dxq,
                       ST[ss:], ws, nws)
    hq.hq_range_update_batch(R, ST, 2)
    torch.cuda.synchronize()
    R0 = R.clone()

    def step():
        hq.hq_gemm_fwd(p, Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, R[:rs], Y, yq, ST[:ss])
        hq.hq_gemm_dgrad(p, dYd.codes, dYd.qp, Wdev.Wd, Wdev.qp, Wdev.wdsum, R[rs:], dX, dxq, ST[ss:])
        hq.hq_gemm_wgrad(p, Xd.codes, Xd.qp, dYd.codes, dYd.qp, dW, None, ws, nws)
        hq.hq_range_update_batch(R, ST, 2)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (Y, dX, dW, R, yq, dxq)]

    eager = []
    for _ in range(3):
        # the data scale drifts so that consecutive steps differ
        Xd.qp.copy_(hq.new_qparams(float(X.scale) * (1.3 ** len(eager)), X.zero_point))
        step()
        eager.append(snapshot())
    assert not torch.equal(eager[0][0], eager[2][0])
    # side stream, eager
    R.copy_(R0)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        Xd.qp.copy_(hq.new_qparams(float(X.scale), X.zero_point))
        step()
    side.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(snapshot(), eager[0]))
    # captured once, replayed three times
    R.copy_(R0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    R.copy_(R0)                                           # capturing does not run the step; make sure of the start state anyway
    hq.hq_stats_reset(ST, 2)
    for k in range(3):
        Xd.qp.copy_(hq.new_qparams(float(X.scale) * (1.3 ** k), X.zero_point))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        assert all(torch.equal(a, b) for a, b in zip(got, eager[k])), "replay %d differs from the eager step" % k
        junk = torch.randn(1 << 16, device="cuda").sum()      # unrelated eager work between replays
        torch.cuda.synchronize()


RIDE = [wl.conv("ride_band", 4, 20, 64, 64, 3), wl.conv("ride_tiles", 2, 9, 24, 40, 3), wl.conv("ride_first", 2, 23, 4, 48, 7, stride=2),
        wl.conv("ride_c128", 2, 14, 128, 128, 3), wl.depthwise("ride_dw3", 2, 13, 48), wl.depthwise("ride_dw_s2", 2, 12, 32, stride=2),
        wl.linear("ride_lin", 96, 2048, 2048)]


@pytest.mark.parametrize("L", RIDE, ids=[l.name for l in RIDE])
def test_wgrad_with_range_updates_riding_along(H, hq, L):
    """hq_gemm_wgrad_update = hq_gemm_wgrad + hq_range_update_batch: same weight gradient, same
    ranges, statistics consumed, on every weight-gradient path; two steps in a row."""
    X, W, dY = rand_layer_inputs(L, 6100)
    Wdev, Xd, dYd = H.DevWeights(L, W), H.DevTensor(X), H.DevTensor(dY)
    p = H.hq_problem(L)
    rs, ss = hq.RANGE.itemsize, hq.STATS.itemsize
    nws = max(hq.hq_workspace_bytes(e, p) for e in (hq.HQ_ENTRY_WGRAD, hq.HQ_ENTRY_DYNAMIC_FWD, hq.HQ_ENTRY_DYNAMIC_DGRAD))
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    Y = torch.empty(wl.out_shape(L), dtype=torch.int8, device="cuda")
    dX = torch.empty(wl.in_shape(L), dtype=torch.int8, device="cuda")
    yq, dxq = hq.new_qparams(0, 0), hq.new_qparams(0, 0)
    results = []
    for fused_update in (False, True):
        R, ST = hq.new_ranges([False, True]), hq.new_stats(2)
        dW = torch.zeros(wl.w_shape(L), dtype=torch.float32, device="cuda")
        dWa = torch.zeros(wl.w_shape(L), dtype=torch.int32, device="cuda")
        hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_FWD, hq.HQ_DYN_CURRENT, p, Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, R[:rs], Y, yq,
                           ST[:ss], ws, nws)
        hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_DGRAD, hq.HQ_DYN_CURRENT, p, dYd.codes, dYd.qp, Wdev.Wd, Wdev.qp, Wdev.wdsum, R[rs:], dX,
                           dxq, ST[ss:], ws, nws)
        hq.hq_range_update_batch(R, ST, 2)
        snaps = []
        for step in range(2):
            Xd.qp.copy_(hq.new_qparams(float(X.scale) * 1.2 ** step, X.zero_point))
            hq.hq_gemm_fwd(p, Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, R[:rs], Y, yq, ST[:ss])
            hq.hq_gemm_dgrad(p, dYd.codes, dYd.qp, Wdev.Wd, Wdev.qp, Wdev.wdsum, R[rs:], dX, dxq, ST[ss:])
            if fused_update:
                hq.hq_gemm_wgrad_update(p, Xd.codes, Xd.qp, dYd.codes, dYd.qp, dW, dWa, ws, nws, R, ST, 2)
            else:
                hq.hq_gemm_wgrad(p, Xd.codes, Xd.qp, dYd.codes, dYd.qp, dW, dWa, ws, nws)
                hq.hq_range_update_batch(R, ST, 2)
            torch.cuda.synchronize()
            st = hq.from_device(ST, hq.STATS)
            assert (st["count"] == 0).all() and (st["acc_min"] == 2**31 - 1).all() and (st["part"]["clip_hi"] == 0).all()
            snaps.append([t.clone() for t in (dW, dWa, R, Y, dX)])
        results.append(snaps)
        Xd.qp.copy_(hq.new_qparams(float(X.scale), X.zero_point))
    for a, b in zip(results[0], results[1]):
        assert all(torch.equal(x, y) for x, y in zip(a, b))
    ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
    assert np.array_equal(results[1][1][1].cpu().numpy(), ref)
    assert not torch.equal(results[1][0][2], results[1][1][2])          # the ranges did move between the steps


NARROW = [wl.conv("nb_band", 2, 20, 64, 64, 3), wl.conv("nb_gemm", 2, 9, 24, 40, 3),
          wl.conv("nb_bandw", 1, 12, 128, 128, 3), wl.conv("nb_first", 2, 23, 4, 48, 7, stride=2),
          wl.depthwise("nb_dw", 2, 13, 48), wl.linear("nb_lin", 300, 72, 80)]


@pytest.mark.parametrize("bits", [2, 4, 6])
@pytest.mark.parametrize("L", NARROW, ids=[l.name for l in NARROW])
def test_output_grids_narrower_than_eight_bits(H, hq, L, bits):
    """The range state carries its grid (qlo, qhi): a b-bit output grid in 8-bit storage goes
    through every kernel's epilogue unchanged, bit for bit, with the clip counts of that grid;
    the last iteration rounds the gradient stochastically."""
    y_track, g_track = H.TensorTrack(0.9, False, bits=bits), H.TensorTrack(0.9, True, bits=bits)
    Wdev = None
    for t in range(3):
        X, W, dY = rand_layer_inputs(L, 7000 + 10 * bits + t)
        if Wdev is None:
            W0, Wdev = W, H.DevWeights(L, W)
        Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
        y, _ = y_track.step(L, "fwd", X, W0, Xd, Wdev)
        g, _ = g_track.step(L, "dgrad", dY, W0, dYd, Wdev, seed=77 if t == 2 else None)
        top = 2 ** (bits - 1) - 1
        assert y.min() >= -top - 1 and y.max() <= top and g.min() >= -top and g.max() <= top


# ---------------------------------------------------------------------------------------
# Degenerate tensors and ranges
# ---------------------------------------------------------------------------------------
def _const_tensor(shape, code, scale, zp):
    from collections import namedtuple
    Q = namedtuple("Q", "codes scale zero_point")
    return Q(np.full(shape, code, dtype=np.int8), np.float32(scale), int(zp))


@pytest.mark.parametrize("L", [wl.conv("deg_band", 2, 20, 64, 64, 3), wl.conv("deg_gemm", 2, 9, 24, 40, 3),
                               wl.conv("deg_bandw", 1, 12, 128, 128, 3), wl.depthwise("deg_dw", 1, 10, 32),
                               wl.linear("deg_lin1", 1, 4, 4)], ids=lambda l: l.name)
def test_degenerate_tensors(H, hq, L):
    """All-zero tensors (the range collapses to a point and the quantizer falls back to scale 1),
    then extreme codes on both operands (largest accumulators, one-sided ranges), then an ordinary
    tensor quantized with the collapsed / one-sided range it inherits (everything clips)."""
    g = np.random.default_rng(12)
    W = wl.he_weight(g, L)
    Wmax = W._replace(codes=np.where(g.random(W.codes.shape) < 0.5, 127, -127).astype(np.int8))
    for Wq in (W, Wmax):
        Wdev = H.DevWeights(L, Wq)
        y_track, g_track = H.TensorTrack(0.9, False), H.TensorTrack(0.9, True)
        X_seq = [_const_tensor(wl.in_shape(L), -128, 0.02, -128),          # real zeros on the unsigned grid
                 _const_tensor(wl.in_shape(L), -128, 0.02, -128),          # again: fused path with the collapsed range
                 _const_tensor(wl.in_shape(L), 127, 0.02, -128),           # every input at the top code
                 wl.relu_activation(g, wl.in_shape(L))]
        G_seq = [_const_tensor(wl.out_shape(L), 0, 1e-4, 0), _const_tensor(wl.out_shape(L), 0, 1e-4, 0),
                 _const_tensor(wl.out_shape(L), -127, 1e-4, 0), wl.laplace_gradient(g, wl.out_shape(L), 1e-3)]
        for X, dY in zip(X_seq, G_seq):
            Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
            y_track.step(L, "fwd", X, Wq, Xd, Wdev)
            g_track.step(L, "dgrad", dY, Wq, dYd, Wdev)
            dW, dWa = H.gpu_wgrad(L, Xd, dYd)
            ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
            assert np.array_equal(dWa, ref)
            assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


@pytest.mark.parametrize("eta", [0.0, 1.0, 0.5])
def test_special_momenta_on_device(H, hq, eta):
    """Eq. (2)-(3) with eta = 0 (the range is last iteration's min-max), eta = 1 (the range never
    moves after its initialisation) and 0.5, over a tensor that grows 1.6x per iteration."""
    L = wl.conv("eta", 2, 12, 32, 32, 3)
    W = wl.he_weight(np.random.default_rng(2), L)
    Wdev = H.DevWeights(L, W)
    y_track = H.TensorTrack(eta, False)
    for t in range(4):
        X = wl.relu_activation(np.random.default_rng(20 + t), wl.in_shape(L), gain=1.6 ** t)
        _, ref = y_track.step(L, "fwd", X, W, H.DevTensor(X), Wdev)
        if t >= 2 and eta > 0.0:
            assert ref["clip_hi"] > 0                     # the lagging range clips the grown tensor


# ---------------------------------------------------------------------------------------
# Error behaviour (nothing is launched on error)
# ---------------------------------------------------------------------------------------
def test_error_codes(H, hq):
    L = wl.conv("err", 1, 8, 16, 16, 3)
    X, W, dY = rand_layer_inputs(L, 2)
    Wdev, Xd = H.DevWeights(L, W), H.DevTensor(X)
    r, st = hq.new_range(), hq.new_stats()
    out = torch.empty(wl.out_shape(L), dtype=torch.int8, device="cuda")
    outq = hq.new_qparams(0, 0)
    bad = hq.problem(hq.HQ_CONV2D, 1, 8, 8, 18, 3, 3, 1, 1, 16)         # C % 4 != 0
    with pytest.raises(hq.HqError) as e:
        hq.hq_gemm_fwd(bad, Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, r, out, outq, st)
    assert e.value.code == hq.HQ_E_BADSHAPE
    with pytest.raises(hq.HqError) as e:
        hq.hq_gemm_fwd(H.hq_problem(L), None, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, r, out, outq, st)
    assert e.value.code == hq.HQ_E_BADARG
    with pytest.raises(hq.HqError) as e:                                   # misaligned codes
        hq.hq_gemm_fwd(H.hq_problem(L), Xd.codes.data_ptr() + 4, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, r, out, outq, st)
    assert e.value.code == hq.HQ_E_BADARG
    ws = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(hq.HqError) as e:
        hq.hq_gemm_dynamic(hq.HQ_ENTRY_DYNAMIC_FWD, 0, H.hq_problem(L), Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum,
                           r, out, outq, st, ws, 64)
    assert e.value.code == hq.HQ_E_WORKSPACE
    with pytest.raises(hq.HqError) as e:
        hq.hq_gemm_dynamic(7, 0, H.hq_problem(L), Xd.codes, Xd.qp, Wdev.W, Wdev.qp, Wdev.wsum, r, out, outq, st, ws, 64)
    assert e.value.code == hq.HQ_E_BADARG
    sink = torch.full((2 * 256,), 7, dtype=torch.int32, device="cuda")
    assert hq.hq_probe_mfma_rate(2, 3, sink) == 2 * 4 * 3 * 8 * 2 * 32 ** 3
    with pytest.raises(hq.HqError) as e:
        hq.hq_probe_mfma_rate(0, 3, sink)
    assert e.value.code == hq.HQ_E_BADARG
    lin_bad = hq.problem(hq.HQ_LINEAR, 8, 2, 1, 16, 1, 1, 1, 0, 16)
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, lin_bad) == 0
    torch.cuda.synchronize()
    s = H.read_stats(st)
    assert int(s["count"]) == 0                                             # nothing ran


def test_batched_range_update(H, hq):
    """eq. (2)-(3) for several quantizers in one launch: three range states in one array (two fed by
    layers of different shapes, one that sees no data), updated together after each iteration."""
    La, Lb = wl.conv("batch_a", 2, 9, 16, 32, 3), wl.linear("batch_b", 70, 48, 64)
    ranges, stats = hq.new_ranges([False, True, False]), hq.new_stats(3)
    rs, ss = hq.RANGE.itemsize, hq.STATS.itemsize
    tracks = [H.TensorTrack(0.9, sym, state=(ranges[i * rs:(i + 1) * rs], stats[i * ss:(i + 1) * ss]))
              for i, sym in enumerate((False, True, False))]
    Xa, Wa, dYa = rand_layer_inputs(La, 5)
    Xb, Wb, dYb = rand_layer_inputs(Lb, 6)
    Wda, Wdb = H.DevWeights(La, Wa), H.DevWeights(Lb, Wb)
    for t in range(3):
        Xa_t = wl.relu_activation(np.random.default_rng(100 + t), wl.in_shape(La))
        dYb_t = wl.laplace_gradient(np.random.default_rng(200 + t), wl.out_shape(Lb), 1e-2 * 0.7 ** t)
        tracks[0].step(La, "fwd", Xa_t, Wa, H.DevTensor(Xa_t), Wda, update=False)
        tracks[1].step(Lb, "dgrad", dYb_t, Wb, H.DevTensor(dYb_t), Wdb, update=False)
        hq.hq_range_update_batch(ranges, stats, 3)
        torch.cuda.synchronize()
        for tr in tracks[:2]:
            H.assert_range_close(H.read_range(tr.r), tr.ref)
            st = H.read_stats(tr.st)
            assert int(st["count"]) == 0 and int(st["acc_min"]) == 2**31 - 1
        idle = H.read_range(tracks[2].r)
        assert int(idle["initialized"]) == 0 and float(idle["qmin"]) == 0.0 and float(idle["qmax"]) == 0.0


# ---------------------------------------------------------------------------------------
# Saturation-driven range update (Sec. 4: the saturation ratio as the statistic)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("op", ["dgrad", "fwd"])
def test_saturation_driven_update_follows_a_drifting_tensor(H, hq, op):
    """Twelve iterations of one layer whose data operand shrinks 0.7x per iteration and jumps up 30x at
    iteration 8: the range waits for more than tau = 1 iterations outside the band, then moves by the
    Laplace quantile rule.  Codes, statistics, quantizer, range and streak against the oracle after
    every iteration; the range must have moved in both directions."""
    L = wl.conv("sat_conv", 4, 20, 32, 48, 3)
    sym = op == "dgrad"
    g = np.random.default_rng(99)
    W = wl.he_weight(g, L)
    Wdev = H.DevWeights(L, W)
    r, st = hq.new_range(0.9, sym), hq.new_stats(1)
    sat = hq.new_saturation(alpha_min=2e-4, alpha_max=5e-3, alpha_target=1e-3, tau=1)
    ref_r, ref_sat = oracle.Range.new(0.9, sym), oracle.Saturation.new(2e-4, 5e-3, 1e-3, 1)
    widths, moved = [], []
    for t in range(12):
        gain = 0.7 ** t * (30.0 if t >= 8 else 1.0)
        if sym:
            A = wl.laplace_gradient(g, wl.out_shape(L), 1e-3)
        else:
            A = wl.relu_activation(g, wl.in_shape(L))
        A = wl.QTensor(A.codes, np.float32(A.scale * gain), A.zero_point)     # same kind of codes, real values scaled
        Adev = H.DevTensor(A)
        a_scale = oracle.acc_scale(A.scale, W.scale)
        c = H.oracle_acc(L, op, A, W)
        before = (ref_r.qmin, ref_r.qmax)
        want = oracle.saturation_step(c, a_scale, ref_r, ref_sat)
        codes, q = H.gpu_quantized_op(L, op, Adev, Wdev, r, st, "dynamic" if t == 0 else "fused")
        got_st = H.read_stats(st)
        hq.hq_range_update_saturation(r, st, sat)
        H.assert_stats_equal(got_st, want, a_scale)
        assert np.float32(q["scale"]) == want["scale"] and int(q["zero_point"]) == want["zero_point"]
        assert np.array_equal(codes, want["codes"])
        H.assert_range_close(H.read_range(r), ref_r)
        got_sat = hq.from_device(sat, hq.SATURATION)[0]
        assert int(got_sat["streak"]) == ref_sat.streak and int(got_sat["tau"]) == 1
        assert int(H.read_stats(st)["count"]) == 0
        widths.append(ref_r.qmax - ref_r.qmin)
        moved.append(t > 0 and (ref_r.qmin, ref_r.qmax) != before)
    assert any(widths[t] < widths[t - 1] for t in range(1, 8)) and widths[-1] > widths[7]
    assert 2 <= sum(moved) < 11                          # it moved, and not on every iteration
