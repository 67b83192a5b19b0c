"""Access to the testing build of the library (liblq_hip_testing.so, include/lq_testing.h) for the test-suite: the
single-kernel hooks and the capture of one configuration's iterate inside lq_error_table.  Marshalling only."""
import ctypes as C
import os

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TEST_LIB = os.path.join(ROOT, "paper_2311_12023_amd", "liblq_hip_testing.so")

_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(TEST_LIB):
            raise ImportError(f"{TEST_LIB} is missing: build it with `python -m paper_2311_12023_amd.build`")
        L = C.CDLL(TEST_LIB)
        vp, i64, it = C.c_void_p, C.c_int64, C.c_int
        L.lq_test_wide_gemm.argtypes = [it, it, i64, i64, vp, i64, vp, i64, vp, i64, it, it, vp, C.c_size_t, it, vp]
        L.lq_test_wide_gemm_f16.argtypes = [it, it, i64, i64, vp, i64, vp, vp, i64, vp, i64, it, it, vp, C.c_size_t,
                                            C.c_float, vp, C.c_float, vp]
        L.lq_test_wide_gemm_part_floats.restype = C.c_size_t
        L.lq_test_wide_gemm_part_floats.argtypes = [it, it]
        L.lq_test_orthonormalize.argtypes = [vp, it, i64, i64, vp, vp, vp]
        L.lq_test_sym_eig.argtypes = [vp, it, vp, vp, vp, vp]
        L.lq_test_sym_eig_fast.argtypes = [vp, it, vp, vp, vp]
        L.lq_test_lincomb3.argtypes = [vp, C.c_float, vp, C.c_float, vp, C.c_float, it, i64, vp]
        L.lq_test_deflate_rows.argtypes = [vp, vp, it, it, i64, i64, vp]
        L.lq_test_ritz_residual.argtypes = [vp, vp, vp, it, i64, i64, vp, vp]
        L.lq_test_lds_limit.restype = C.c_size_t
        L.lq_test_bucket_code.argtypes = [C.c_int, C.c_float]
        L.lq_test_capture_iterate.argtypes = [it, it, vp, vp]
        _lib = L
    return _lib


def error_table_with_capture(w, rank, cfgs, iters, cfg_index, it, seed=0, params=None, row_w=None, col_w=None):
    """lq_error_table of the testing build with a capture armed: -> (err_sq, storage_bits, trace, Q_it dense tensor of
    configuration cfg_index after iteration `it`, singular values found by the Factorize of iteration it + 1)."""
    import torch
    from paper_2311_12023_amd import lq
    L = load()
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
    L.lq_error_table_workspace_bytes.restype = C.c_size_t
    L.lq_error_table_workspace_bytes.argtypes = [i64, i64, i32, i32, C.POINTER(lq.SvdParams)]
    L.lq_error_table.argtypes = [vp, i64, i64, i32, vp, i32, i32, i32, vp, vp, C.c_uint64, C.POINTER(lq.SvdParams),
                                 vp, vp, vp, vp, C.c_size_t, vp]
    d, k = w.shape
    pp = None if params is None else C.byref(params)
    arr = (lq.Config * len(cfgs))(*cfgs)
    ws = torch.empty(L.lq_error_table_workspace_bytes(d, k, rank, len(cfgs), pp) + 256, dtype=torch.uint8, device=w.device)
    base = (ws.data_ptr() + 255) & ~255
    q = torch.zeros((d, k), dtype=torch.float32, device=w.device)
    sigma = np.full(rank, np.nan)
    e, s = np.zeros(len(cfgs)), np.zeros(len(cfgs))
    tr = np.full((len(cfgs), iters), np.nan)
    assert L.lq_test_capture_iterate(cfg_index, it, q.data_ptr(), sigma.ctypes.data) == 0
    rc = L.lq_error_table(w.data_ptr(), d, k, rank, C.addressof(arr), len(cfgs), iters, 0,
                          None if row_w is None else row_w.data_ptr(), None if col_w is None else col_w.data_ptr(),
                          seed, pp, e.ctypes.data, s.ctypes.data, tr.ctypes.data, base,
                          ws.numel() - (base - ws.data_ptr()), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, rc
    torch.cuda.synchronize()
    return e, s, tr, q, sigma
