"""GPU parity at the full sizes of the configurations, in the launch configuration bench.py
times.  The oracle computes whole tensors where that takes seconds (configs 2-4) and sampled
rows elsewhere; statistics are compared exactly wherever the oracle has the whole tensor."""
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


def test_c2_full_size_three_iterations(H, hq):
    """conv3x3 64->64 @56x56, batch 128: dynamic init then two in-hindsight forward passes with the
    activation scale growing 1.05x per iteration; dgrad and wgrad once."""
    track = H.TensorTrack(0.9, symmetric=False)
    Wdev = None
    clip = []
    for t in range(3):
        L, X, W = wl.c2_inputs(t)
        if Wdev is None:
            Wdev = H.DevWeights(L, W)
        _, ref = track.step(L, "fwd", X, W, H.DevTensor(X), Wdev)
        clip.append((ref["clip_lo"] + ref["clip_hi"]) / ref["count"])
    assert clip[0] == 0.0
    dY = wl.laplace_gradient(wl.rng(2, 0, 2), wl.out_shape(L), 1e-3)
    gtrack = H.TensorTrack(0.9, symmetric=True)
    dYd = H.DevTensor(dY)
    for _ in range(2):
        gtrack.step(L, "dgrad", dY, W, dYd, Wdev)
    gtrack.step(L, "dgrad", dY, W, dYd, Wdev, seed=0x243f6a8885a308d3)        # stochastic rounding, whole tensor
    dW, dWa = H.gpu_wgrad(L, H.DevTensor(X), dYd)
    ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
    assert np.array_equal(dWa, ref) and np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


def test_c3_full_size_backward(H, hq):
    """conv3x3 128->128 @28x28, batch 128: dgrad with in-hindsight vs dynamic ranges over decaying,
    outlier-laden gradients (iterations 0, 1, 25 of the 50-step schedule), and wgrad."""
    L = wl.c3_layer()
    track = H.TensorTrack(0.9, symmetric=True)
    Wdev = None
    for t in (0, 1, 25):
        L, X, W, dY = wl.c3_inputs(t)
        if Wdev is None:
            Wdev = H.DevWeights(L, W)
        dYd = H.DevTensor(dY)
        codes, ref = track.step(L, "dgrad", dY, W, dYd, Wdev)
        if t == 25:
            # gradients shrank ~5x per 12 iterations: yesterday's range is too wide, nothing clips,
            # and the grid is under-used (the behaviour the drift closed form predicts)
            assert ref["clip_lo"] + ref["clip_hi"] == 0
            assert np.abs(codes.astype(int)).max() < 127
    dW, dWa = H.gpu_wgrad(L, H.DevTensor(X), dYd)
    ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
    assert np.array_equal(dWa, ref) and np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))


def test_c4_full_size_block(H, hq):
    """MobileNetV2 block, batch 128: expand 1x1, depthwise 3x3, project 1x1; fwd + dgrad + wgrad,
    per-tensor range state per layer (6 range states), init + one in-hindsight iteration."""
    tracks = None
    for t in range(2):
        layers = wl.c4_inputs(t)
        if tracks is None:
            tracks = [(H.TensorTrack(0.9, False), H.TensorTrack(0.9, True), H.DevWeights(L, W), W) for L, X, W, dY in layers]
        for (L, X, _, dY), (yt, gt, Wdev, W) in zip(layers, tracks):
            Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
            yt.step(L, "fwd", X, W, Xd, Wdev)
            gt.step(L, "dgrad", dY, W, dYd, Wdev)
            if t == 1:
                dW, dWa = H.gpu_wgrad(L, Xd, dYd)
                ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
                assert np.array_equal(dWa, ref) and np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale))
            del Xd, dYd
            torch.cuda.empty_cache()


def test_c5_resnet18_stack_small_batch(H, hq):
    """Every layer of the ResNet-18-shaped stack (7x7/2 stem on 3-channel images, 3x3 stages with
    stride-2 downsampling and 1x1/2 shortcuts, FC 512->1000) at batch 4: dynamic init + one
    in-hindsight iteration of fwd and dgrad (no dgrad for the stem), wgrad once; whole tensors
    against the oracle."""
    layers = wl.resnet18_layers(B=4)
    assert len(layers) == 21
    for idx, L in enumerate(layers):
        yt, gt = H.TensorTrack(0.9, False), H.TensorTrack(0.9, True)
        Wdev = None
        for t in range(2):
            X, W, dY = wl.layer_inputs(L, 5, t, idx, image_input=(idx == 0))
            if Wdev is None:
                W0, Wdev = W, H.DevWeights(L, W)
            Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
            yt.step(L, "fwd", X, W0, Xd, Wdev)
            if idx > 0:
                gt.step(L, "dgrad", dY, W0, dYd, Wdev)
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref), L.name
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale)), L.name


def test_vgg16_stack_small_batch(H, hq):
    """Every layer of the VGG16-shaped stack (13 3x3 convs at 64 ... 4 pixels, three linear layers)
    at batch 2: dynamic init + one in-hindsight iteration of fwd and dgrad (no dgrad for the first
    layer), wgrad once; whole tensors against the oracle."""
    layers = wl.vgg16_layers(B=2)
    assert len(layers) == 16 and layers[13].C == 2048
    for idx, L in enumerate(layers):
        yt, gt = H.TensorTrack(0.9, False), H.TensorTrack(0.9, True)
        Wdev = None
        for t in range(2):
            X, W, dY = wl.layer_inputs(L, 6, t, idx, image_input=(idx == 0))
            if Wdev is None:
                W0, Wdev = W, H.DevWeights(L, W)
            Xd, dYd = H.DevTensor(X), H.DevTensor(dY)
            yt.step(L, "fwd", X, W0, Xd, Wdev)
            if idx > 0:
                gt.step(L, "dgrad", dY, W0, dYd, Wdev)
        dW, dWa = H.gpu_wgrad(L, Xd, dYd)
        ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
        assert np.array_equal(dWa, ref), L.name
        assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale)), L.name


@pytest.mark.parametrize("which", ["stem_7x7", "s2_conv0", "s3_short", "s4_conv2", "fc"])
def test_c5_full_batch_sampled(H, hq, which):
    """Batch 256 (the size the step is quoted on): forward and dgrad of representative layers with
    the oracle evaluated on sampled output rows; whole-tensor statistics are checked through
    properties that hold at any size."""
    layers = wl.resnet18_layers(B=256)
    idx = [l.name for l in layers].index(which)
    L = layers[idx]
    X, W, dY = wl.layer_inputs(L, 5, 0, idx, image_input=(idx == 0))
    Wdev, Xd, dYd = H.DevWeights(L, W), H.DevTensor(X), H.DevTensor(dY)
    g = np.random.default_rng(7)
    for op, A, Adev, sym in (("fwd", X, Xd, False), ("dgrad", dY, dYd, True)):
        if op == "dgrad" and idx == 0:
            continue
        r, st = hq.new_range(0.9, sym), hq.new_stats()
        dyn_codes, q0 = H.gpu_quantized_op(L, op, Adev, Wdev, r, st, "dynamic")
        s0 = H.read_stats(st)
        hq.hq_range_update(r, st)
        codes, q = H.gpu_quantized_op(L, op, Adev, Wdev, r, st, "fused")
        s1 = H.read_stats(st)
        nrow = codes.size // codes.shape[-1]
        rows = np.unique(np.concatenate([g.integers(0, nrow, 2000), [0, nrow - 1]]))
        po = H.oracle_problem(L)
        c = oracle.fwd_rows(po, A.codes, A.zero_point, W.codes, rows) if op == "fwd" else \
            oracle.dgrad_rows(po, A.codes, A.zero_point, W.codes, rows)
        a_scale = oracle.acc_scale(A.scale, W.scale)
        # dynamic: the quantizer must be the one the GPU's own min/max imply, codes follow from it
        gmin, gmax = np.float32(a_scale) * np.float32(s0["acc_min"]), np.float32(a_scale) * np.float32(s0["acc_max"])
        sc, z = oracle.qparams(gmin, gmax, int(sym), -127 if sym else -128, 127)
        assert np.float32(q0["scale"]) == sc and int(q0["zero_point"]) == z
        want, _, _ = oracle.requant(c, a_scale, sc, z, -127 if sym else -128, 127)
        assert np.array_equal(dyn_codes.reshape(nrow, -1)[rows], want)
        assert int(s0["acc_min"]) <= c.min() and int(s0["acc_max"]) >= c.max()
        assert int(s0["count"]) == codes.size and int(s0["clip_lo"]) == 0 and int(s0["clip_hi"]) == 0
        # fused: range state after the first update, from the oracle's arithmetic
        ref = oracle.Range.new(0.9, sym)
        oracle.range_update(ref, int(s0["acc_min"]), int(s0["acc_max"]), a_scale)
        oracle.range_update(ref, int(s0["acc_min"]), int(s0["acc_max"]), a_scale)
        assert np.float32(q["scale"]) == np.float32(ref.scale) and int(q["zero_point"]) == ref.zero_point
        want, _, _ = oracle.requant(c, a_scale, ref.scale, ref.zero_point, ref.qlo, ref.qhi)
        assert np.array_equal(codes.reshape(nrow, -1)[rows], want)
        assert (int(s1["acc_min"]), int(s1["acc_max"]), int(s1["count"])) == (int(s0["acc_min"]), int(s0["acc_max"]), codes.size)


C5_LAYERS = [l.name for l in wl.resnet18_layers(B=256)]


@pytest.mark.parametrize("which", C5_LAYERS)
def test_c5_full_batch_whole_tensors(H, hq, which):
    """The ResNet-18-shaped step at batch 256, the size it is quoted on, one layer per case: forward and
    input gradient (none for the stem) through the dynamic first iteration and one in-hindsight
    iteration, and the weight gradient, every output element, statistic and clip count against the
    oracle on the whole tensors.  The oracle's weight gradient sums up to 3.2 M products per element
    in 64 bits and reports whether every sum fits 32 bits, which the 32-bit accumulators of the
    kernels need (Sec. 3.2)."""
    layers = wl.resnet18_layers(B=256)
    idx = C5_LAYERS.index(which)
    L = layers[idx]
    X, W, dY = wl.layer_inputs(L, 5, 0, idx, image_input=(idx == 0))
    Wdev, Xd, dYd = H.DevWeights(L, W), H.DevTensor(X), H.DevTensor(dY)
    for op, A, Adev, sym in (("fwd", X, Xd, False), ("dgrad", dY, dYd, True)):
        if op == "dgrad" and idx == 0:
            continue
        a_scale = oracle.acc_scale(A.scale, W.scale)
        c = H.oracle_acc(L, op, A, W)                      # 64-bit sums, asserted to fit 32 bits
        r, st, ref_r = hq.new_range(0.9, sym), hq.new_stats(), oracle.Range.new(0.9, sym)
        for t in range(2):
            want = oracle.in_hindsight_step(c, a_scale, ref_r)
            codes, q = H.gpu_quantized_op(L, op, Adev, Wdev, r, st, "dynamic" if t == 0 else "fused")
            got_st = H.read_stats(st)
            hq.hq_range_update(r, st)
            H.assert_stats_equal(got_st, want, a_scale)     # min, max, clip counts and count, all with ==
            assert np.float32(q["scale"]) == want["scale"] and int(q["zero_point"]) == want["zero_point"]
            assert np.array_equal(codes, want["codes"]), (L.name, op, t)
            H.assert_range_close(H.read_range(r), ref_r)
            del codes
        del c
    dW, dWa = H.gpu_wgrad(L, Xd, dYd)
    ref = oracle.wgrad(H.oracle_problem(L), X.codes, X.zero_point, dY.codes, dY.zero_point)
    assert np.array_equal(dWa, ref), L.name
    assert np.array_equal(dW, oracle.wgrad_scale(ref, X.scale, dY.scale)), L.name


def test_real_tensor_quantizer_full_size(H, hq):
    """The element-wise quantizer on an FP32 tensor the size of config 2's output (25.7 M values), in the
    launch shape bench.py times: dynamic first batch, in-hindsight second, stochastic third; whole
    tensor against the oracle."""
    n = wl.nelem(wl.out_shape(wl.c2_layer()))
    r, st, ref = hq.new_range(0.9, False), hq.new_stats(1), oracle.Range.new(0.9, False)
    Q = torch.empty(n, dtype=torch.int8, device="cuda")
    qp = hq.new_qparams(0.0, 0)
    for t in range(3):
        x = wl.real_activation(wl.rng(2, t, 77), n, gain=1.05 ** t, shift=-0.2)
        xd = torch.from_numpy(x).cuda()
        seed = 0x6a09e667f3bcc908 if t == 2 else None
        want = oracle.tensor_step(x, ref, "hindsight", seed)
        if t == 0:
            hq.hq_tensor_quantize_dynamic(hq.HQ_DYN_CURRENT, xd, n, r, Q, qp, st)
        elif seed is None:
            hq.hq_tensor_quantize(xd, n, r, Q, qp, st)
        else:
            hq.hq_tensor_quantize_sr(xd, n, r, seed, Q, qp, st)
        got_st = H.read_stats(st)
        hq.hq_range_update(r, st)
        assert np.array_equal(Q.cpu().numpy(), want["codes"])
        assert (int(got_st["clip_lo"]), int(got_st["clip_hi"]), int(got_st["count"])) == (want["clip_lo"], want["clip_hi"], n)
        H.assert_range_close(H.read_range(r), ref)
    assert want["clip_hi"] > 0
