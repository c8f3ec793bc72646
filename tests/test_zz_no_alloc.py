"""hq_gemm_wgrad_static, the weight-gradient entry point that allocates nothing (its workspace
is an array the library holds on the GPU): called through the C ABI, compared bit for bit with
hq_gemm_wgrad on the same inputs, on two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2105_04246_amd as hq
import workloads as wl

pytestmark = pytest.mark.gpu


def _problem(L):
    return hq.problem(L.kind, L.B, L.H, L.W, L.C, L.R, L.S, L.stride, L.pad, L.Cout)


def _operands(L, index):
    X, _, dY = wl.layer_inputs(L, 7, 0, index)
    x = torch.from_numpy(X.codes).cuda()
    g = torch.from_numpy(dY.codes).cuda()
    return x, hq.new_qparams(X.scale, X.zero_point), g, hq.new_qparams(dY.scale, dY.zero_point)


def _run_both(L, index):
    p = _problem(L)
    x, xq, g, gq = _operands(L, index)
    nbytes = hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, p)
    assert 0 < nbytes <= hq.HQ_STATIC_SCRATCH_BYTES
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    shape = wl.w_shape(L)
    ref = torch.empty(shape, dtype=torch.float32, device="cuda")
    ref_acc = torch.empty(shape, dtype=torch.int32, device="cuda")
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    got_acc = torch.full(shape, -1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    L_ = hq.lib()
    vp = ctypes.c_void_p
    rc = L_.hq_gemm_wgrad(ctypes.byref(p), vp(x.data_ptr()), vp(xq.data_ptr()), vp(g.data_ptr()), vp(gq.data_ptr()),
                          vp(ref.data_ptr()), vp(ref_acc.data_ptr()), vp(ws.data_ptr()), nbytes, vp(stream))
    assert rc == hq.HQ_OK
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = L_.hq_gemm_wgrad_static(ctypes.byref(p), vp(x.data_ptr()), vp(xq.data_ptr()), vp(g.data_ptr()),
                                 vp(gq.data_ptr()), vp(got.data_ptr()), vp(got_acc.data_ptr()), vp(stream))
    assert rc == hq.HQ_OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert np.array_equal(got_acc.cpu().numpy(), ref_acc.cpu().numpy()), L.name
    a, b = got.cpu().numpy(), ref.cpu().numpy()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), L.name            # FP32 result bit for bit
    assert np.abs(ref_acc.cpu().numpy()).max() > 0


def test_static_weight_gradient_matches_the_workspace_one_on_two_calls_in_a_row():
    # split-K tile kernel with integer atomics (the scratch must start at zero), 3x3 stride 2, larger first
    _run_both(wl.conv("big_s2", 8, 28, 64, 128, 3, stride=2), 0)
    _run_both(wl.conv("small_s2", 3, 14, 32, 48, 3, stride=2), 1)
    # the banded kernel (per-workgroup partial sums in the scratch), larger first, then a ragged smaller one
    _run_both(wl.conv("band_big", 16, 28, 128, 128, 3), 2)
    _run_both(wl.conv("band_small", 5, 14, 64, 64, 3), 3)
    # linear and depthwise layers take the same entry point
    _run_both(wl.linear("fc", 96, 512, 200), 4)
    _run_both(wl.depthwise("dw", 4, 28, 96), 5)
    _run_both(wl.depthwise("dw_small", 2, 14, 32), 6)


def test_static_weight_gradient_refuses_what_does_not_fit_and_bad_arguments():
    L_ = hq.lib()
    nul = ctypes.c_void_p(0)
    too_big = hq.problem(hq.HQ_LINEAR, 64, 1, 1, 8192, 1, 1, 1, 0, 4096)          # 128 MiB of integer sums
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, too_big) > hq.HQ_STATIC_SCRATCH_BYTES
    one = ctypes.c_void_p(256)
    assert L_.hq_gemm_wgrad_static(ctypes.byref(too_big), one, one, one, one, one, nul, nul) == hq.HQ_E_WORKSPACE
    ok = hq.problem(hq.HQ_LINEAR, 64, 1, 1, 64, 1, 1, 1, 0, 64)
    assert L_.hq_gemm_wgrad_static(ctypes.byref(ok), nul, nul, nul, nul, nul, nul, nul) == hq.HQ_E_BADARG
    bad = hq.problem(hq.HQ_CONV2D, 2, 8, 8, 18, 3, 3, 1, 1, 32)
    assert L_.hq_gemm_wgrad_static(ctypes.byref(bad), one, one, one, one, one, nul, nul) == hq.HQ_E_BADSHAPE
