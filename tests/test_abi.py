"""The C-ABI library loads and exports every entry point that include/hq.h declares
(no GPU needed: nothing is launched), and the binding's struct views match the header."""
import ctypes
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hq_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_entry_points():
    names = declared_functions()
    for f in ("hq_gemm_fwd", "hq_gemm_dgrad", "hq_gemm_wgrad", "hq_range_update", "hq_gemm_dynamic"):
        assert f in names


def test_library_exports_every_declared_symbol():
    import paper_2105_04246_amd as hq
    L = hq.lib()
    for f in declared_functions():
        assert hasattr(L, f), f
    assert sorted(hq.EXPORTS) == declared_functions()
    assert L.hq_error_string(0) == b"ok" and b"shape" in L.hq_error_string(hq.HQ_E_BADSHAPE)


def test_binding_argument_counts_match_the_header():
    import paper_2105_04246_amd as hq
    text = open(os.path.join(ROOT, "include", "hq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    L = hq.lib()
    protos = re.findall(r"\b(hq_[a-z_0-9]+)\s*\(([^)]*)\)\s*;", text)
    assert len(protos) == len(hq.EXPORTS)
    for name, args in protos:
        n = len([a for a in args.split(",") if a.strip()])
        assert len(getattr(L, name).argtypes) == n, name


def test_struct_views_match_header_sizes():
    import paper_2105_04246_amd as hq

    class QP(ctypes.Structure):
        _fields_ = [("scale", ctypes.c_float), ("zero_point", ctypes.c_int32)]

    class RG(ctypes.Structure):
        _fields_ = [("qmin", ctypes.c_float), ("qmax", ctypes.c_float), ("eta", ctypes.c_float),
                    ("qlo", ctypes.c_int32), ("qhi", ctypes.c_int32), ("symmetric", ctypes.c_int32),
                    ("initialized", ctypes.c_int32), ("qp", QP)]

    class PT(ctypes.Structure):
        _fields_ = [("acc_min", ctypes.c_int32), ("acc_max", ctypes.c_int32), ("clip_lo", ctypes.c_uint64),
                    ("clip_hi", ctypes.c_uint64), ("pad", ctypes.c_uint8 * 104)]

    class ST(ctypes.Structure):
        _fields_ = [("acc_min", ctypes.c_int32), ("acc_max", ctypes.c_int32), ("acc_scale", ctypes.c_float),
                    ("fp32_keys", ctypes.c_uint32), ("clip_lo", ctypes.c_uint64), ("clip_hi", ctypes.c_uint64),
                    ("count", ctypes.c_uint64), ("pad", ctypes.c_uint8 * 88), ("part", PT * 64)]

    assert ctypes.sizeof(QP) == hq.QPARAMS.itemsize
    assert ctypes.sizeof(RG) == hq.RANGE.itemsize and RG.qp.offset == hq.RANGE.fields["scale"][1]
    assert ctypes.sizeof(ST) == hq.STATS.itemsize and ST.clip_lo.offset == hq.STATS.fields["clip_lo"][1]
    assert ctypes.sizeof(PT) == 128 and ST.part.offset == hq.STATS.fields["part"][1] == 128
    assert ctypes.sizeof(hq.hq_problem) == 40


def test_host_side_argument_checks_need_no_gpu():
    """Shape / pointer validation happens before anything touches the device."""
    import paper_2105_04246_amd as hq
    L = hq.lib()
    good = hq.problem(hq.HQ_CONV2D, 2, 8, 8, 16, 3, 3, 1, 1, 32)
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_DYNAMIC_FWD, good) == 4 * 2 * 8 * 8 * 32
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_DYNAMIC_DGRAD, good) == 4 * 2 * 8 * 8 * 16
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, good) >= 4 * 32 * 9 * 16
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_FWD, good) == 0
    bad = hq.problem(hq.HQ_CONV2D, 2, 8, 8, 18, 3, 3, 1, 1, 32)
    assert hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, bad) == 0
    nul = ctypes.c_void_p(0)
    assert L.hq_gemm_fwd(ctypes.byref(bad), *([nul] * 10)) == hq.HQ_E_BADSHAPE
    assert L.hq_gemm_fwd(ctypes.byref(good), *([nul] * 10)) == hq.HQ_E_BADARG
    assert L.hq_range_update(nul, nul, nul) == hq.HQ_E_BADARG
    assert L.hq_probe_mfma_rate(4, 4, nul, nul) == hq.HQ_E_BADARG
    assert L.hq_weight_quantize(nul, 16, nul, nul, nul) == hq.HQ_E_BADARG
    assert L.hq_gemm_wgrad_update(ctypes.byref(good), *([nul] * 7), 0, nul, nul, 2, nul) == hq.HQ_E_BADARG
    assert L.hq_gemm_dynamic_sr(hq.HQ_ENTRY_FWD, 0, ctypes.byref(good), *([nul] * 6), 1, *([nul] * 4), 0, nul) == hq.HQ_E_BADARG
    assert L.hq_tensor_quantize(nul, 16, nul, nul, nul, nul, nul) == hq.HQ_E_BADARG
    assert L.hq_tensor_quantize_sr(nul, 16, nul, 5, nul, nul, nul, nul) == hq.HQ_E_BADARG
    assert L.hq_tensor_quantize_dynamic(0, nul, 16, nul, nul, nul, nul, nul) == hq.HQ_E_BADARG
    assert L.hq_tensor_quantize_dynamic(7, nul, 0, ctypes.c_void_p(128), nul, ctypes.c_void_p(128),
                                        ctypes.c_void_p(128), nul) == hq.HQ_E_BADARG      # bad mode, caught before any launch
    # sizes past the documented maxima (31-bit pixel and weight counts, 32-bit byte offsets) are refused
    for huge in (hq.problem(hq.HQ_CONV2D, 1 << 20, 64, 64, 16, 3, 3, 1, 1, 16),          # B*H*W = 2^32
                 hq.problem(hq.HQ_CONV2D, 1 << 16, 64, 64, 64, 1, 1, 1, 0, 4),           # B*H*W*C = 2^34 bytes
                 hq.problem(hq.HQ_LINEAR, 4, 1, 1, 1 << 16, 1, 1, 1, 0, 1 << 15),        # C*Cout = 2^31 weights
                 hq.problem(hq.HQ_CONV2D, 0, 8, 8, 16, 3, 3, 1, 1, 16),                  # empty batch
                 hq.problem(hq.HQ_CONV2D, 1, 2, 2, 16, 5, 5, 1, 1, 16),                  # no output pixel
                 hq.problem(hq.HQ_CONV2D, 1, 8, 8, 16, 3, 3, 1, 3, 16)):                 # padding >= filter size
        assert L.hq_gemm_fwd(ctypes.byref(huge), *([nul] * 10)) == hq.HQ_E_BADSHAPE
        assert L.hq_gemm_dgrad(ctypes.byref(huge), *([nul] * 10)) == hq.HQ_E_BADSHAPE
        assert hq.hq_workspace_bytes(hq.HQ_ENTRY_WGRAD, huge) == 0
    dw_bad = hq.problem(hq.HQ_DEPTHWISE, 1, 8, 8, 16, 3, 3, 1, 1, 32)
    assert L.hq_gemm_fwd(ctypes.byref(dw_bad), *([nul] * 10)) == hq.HQ_E_BADSHAPE
