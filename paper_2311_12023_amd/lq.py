"""Python binding of the LQ C ABI (include/lq.h): argument marshalling only.

torch supplies device memory and the current stream; every step of the path runs in the HIP
library.  There is no fallback: if the library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblq_hip.so")

V_DTYPES = {"fp32": 0, "bf16": 1, "fp16": 2}


class LqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = _lib.lq_status_string(status).decode()
        if status == -7:
            msg += f" (hipError {_lib.lq_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


class Config(C.Structure):
    """lq_config: (bits b0, block B0, scale_block B1, scale_bits b1, v_dtype b2)."""
    _fields_ = [("bits", C.c_int32), ("block", C.c_int32), ("scale_block", C.c_int32),
                ("scale_bits", C.c_int32), ("v_dtype", C.c_int32)]

    def __repr__(self):
        return f"Config({self.bits},{self.block},{self.scale_block},{self.scale_bits},{self.v_dtype})"


def config(bits, block, scale_block, scale_bits=8, v_dtype="fp32") -> Config:
    return Config(bits, block, scale_block, scale_bits, V_DTYPES[v_dtype] if isinstance(v_dtype, str) else v_dtype)


class SvdParams(C.Structure):
    """lq_svd_params; zero fields select the library defaults."""
    _fields_ = [("first_width", C.c_int32), ("first_tol", C.c_float), ("first_check", C.c_int32),
                ("first_max", C.c_int32), ("warm_width", C.c_int32), ("warm_power", C.c_int32),
                ("warm_power_2", C.c_int32), ("max_batch", C.c_int32), ("gemm_mode", C.c_int32),
                ("streams", C.c_int32), ("init_quantized", C.c_int32), ("warm_power_coarse", C.c_int32),
                ("warm_power_fine", C.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2311_12023_amd.build`")
_lib = C.CDLL(LIB_PATH)

_vp, _i64, _int, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
_lib.lq_status_string.restype = C.c_char_p
_lib.lq_status_string.argtypes = [_int]
_lib.lq_last_hip_error.restype = _int
_lib.lq_nf_codebook.argtypes = [_int, _vp]
_lib.lq_codes_bytes.restype = _sz
_lib.lq_codes_bytes.argtypes = [_i64, _int]
_lib.lq_storage_bits.restype = C.c_double
_lib.lq_storage_bits.argtypes = [_i64, Config]
_lib.lq_nf_quantize.argtypes = [_vp, _i64, Config, _vp, _vp, _vp, _vp]
_lib.lq_nf_dequantize.argtypes = [_vp, _vp, _vp, _i64, Config, _vp, _vp]
_lib.lq_pack_scale_indices.argtypes = [_vp, _i64, _int, _vp, _vp]
_lib.lq_unpack_scale_indices.argtypes = [_vp, _i64, _int, _vp, _vp]
_PP = C.POINTER(SvdParams)
_lib.lq_factorize_workspace_bytes.restype = _sz
_lib.lq_factorize_workspace_bytes.argtypes = [_i64, _i64, _int, _PP]
_lib.lq_factorize.argtypes = [_vp, _i64, _i64, _int, _vp, _vp, C.c_uint64, _PP, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lq_decompose_workspace_bytes.restype = _sz
_lib.lq_decompose_workspace_bytes.argtypes = [_i64, _i64, _int, _PP]
_lib.lq_decompose.argtypes = [_vp, _i64, _i64, _int, Config, _int, _int, _vp, _vp, C.c_uint64, _PP,
                              _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lq_error_table_workspace_bytes.restype = _sz
_lib.lq_error_table_workspace_bytes.argtypes = [_i64, _i64, _int, _int, _PP]
_lib.lq_error_table.argtypes = [_vp, _i64, _i64, _int, _vp, _int, _int, _int, _vp, _vp, C.c_uint64, _PP,
                                _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lq_assign_configs.argtypes = [_vp, _vp, _int, _int, C.c_double, _i64, _vp, _vp, _vp, _vp]
_lib.lq_fisher_row_col_workspace_bytes.restype = _sz
_lib.lq_fisher_row_col_workspace_bytes.argtypes = [_i64, _i64]
_lib.lq_fisher_row_col.argtypes = [_vp, _i64, _i64, _vp, _vp, _vp, _sz, _vp]
_lib.lq_matmul_workspace_bytes.restype = _sz
_lib.lq_matmul_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
_lib.lq_matmul.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, Config, _vp, _vp, _int, _int, _vp, _vp, _sz, _vp]
_lib.lq_matmul_few_rows_static_scratch_bytes.restype = _sz
_lib.lq_matmul_few_rows_static.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, Config, _vp, _vp, _int, _vp, _vp]

_lib.lq_profile_enable.argtypes = [_int]
_lib.lq_profile_class_name.restype = C.c_char_p
_lib.lq_profile_class_name.argtypes = [_int]
_lib.lq_profile_read.argtypes = [_int, _vp, _vp, _vp]


def _check(status, where):
    if status != 0:
        raise LqError(status, where)


def _dev(t, dtype, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _pp(p):
    return None if p is None else C.byref(p)


def nf_codebook(bits: int) -> np.ndarray:
    out = np.zeros(1 << max(bits, 0) if 0 < bits <= 8 else 1, np.float32)
    _check(_lib.lq_nf_codebook(bits, out.ctypes.data), "lq_nf_codebook")
    return out


def codes_bytes(n: int, bits: int) -> int:
    return _lib.lq_codes_bytes(n, bits)


def storage_bits(n: int, cfg: Config) -> float:
    return _lib.lq_storage_bits(n, cfg)


def nf_quantize(x: torch.Tensor, cfg: Config, out=None):
    """Quantize(x, c): -> (codes_packed uint8, scale_idx uint8, v fp32), all on x's device; `out`: such a triple of the
    right sizes to write into instead of new tensors."""
    n = x.numel()
    nb = n // max(cfg.block, 1)
    ng = (nb + max(cfg.scale_block, 1) - 1) // max(cfg.scale_block, 1)
    if out is not None:
        codes, sidx, v = out
        if codes.numel() < codes_bytes(n, cfg.bits) or sidx.numel() < nb or v.numel() < ng:
            raise ValueError("nf_quantize: output buffers too small")
        _dev(codes, torch.uint8, "codes"), _dev(sidx, torch.uint8, "scale_idx"), _dev(v, torch.float32, "v")
    else:
        codes = torch.empty(max(codes_bytes(n, cfg.bits), 1), dtype=torch.uint8, device=x.device)
        sidx = torch.empty(max(nb, 1), dtype=torch.uint8, device=x.device)
        v = torch.empty(max(ng, 1), dtype=torch.float32, device=x.device)
    _check(_lib.lq_nf_quantize(_dev(x, torch.float32, "x"), n, cfg, codes.data_ptr(), sidx.data_ptr(), v.data_ptr(),
                               _stream()), "lq_nf_quantize")
    return codes, sidx, v


def nf_dequantize(codes: torch.Tensor, scale_idx: torch.Tensor, v: torch.Tensor, n: int, cfg: Config,
                  out: torch.Tensor | None = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=codes.device)
    _check(_lib.lq_nf_dequantize(_dev(codes, torch.uint8, "codes"), _dev(scale_idx, torch.uint8, "scale_idx"),
                                 _dev(v, torch.float32, "v"), n, cfg, _dev(out, torch.float32, "out"), _stream()),
           "lq_nf_dequantize")
    return out


def pack_scale_indices(scale_idx: torch.Tensor, scale_bits: int) -> torch.Tensor:
    """One-byte scale indices -> bit stream of scale_bits bits each."""
    out = torch.empty(max(codes_bytes(scale_idx.numel(), scale_bits), 1), dtype=torch.uint8, device=scale_idx.device)
    _check(_lib.lq_pack_scale_indices(_dev(scale_idx, torch.uint8, "scale_idx"), scale_idx.numel(), scale_bits,
                                      out.data_ptr(), _stream()), "lq_pack_scale_indices")
    return out


def unpack_scale_indices(packed: torch.Tensor, count: int, scale_bits: int) -> torch.Tensor:
    out = torch.empty(max(count, 1), dtype=torch.uint8, device=packed.device)
    _check(_lib.lq_unpack_scale_indices(_dev(packed, torch.uint8, "packed"), count, scale_bits, out.data_ptr(),
                                        _stream()), "lq_unpack_scale_indices")
    return out


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(nbytes + 256, dtype=torch.uint8, device=device)


def _aligned_ptr(ws: torch.Tensor) -> int:
    p = ws.data_ptr()
    return (p + 255) & ~255


def factorize(a: torch.Tensor, rank: int, row_w=None, col_w=None, seed: int = 0, params: SvdParams | None = None,
              workspace: torch.Tensor | None = None):
    """Factorize(A, F, r): -> (L1 d x r, L2 r x k, sigma numpy float64[r])."""
    d, k = a.shape
    need = _lib.lq_factorize_workspace_bytes(d, k, rank, _pp(params))
    ws = workspace if workspace is not None else _workspace(need, a.device)
    l1 = torch.empty((d, rank), dtype=torch.float32, device=a.device)
    l2 = torch.empty((rank, k), dtype=torch.float32, device=a.device)
    sigma = np.zeros(max(rank, 1))
    _check(_lib.lq_factorize(_dev(a, torch.float32, "a"), d, k, rank, _dev(row_w, torch.float32, "row_w"),
                             _dev(col_w, torch.float32, "col_w"), seed, _pp(params), l1.data_ptr(), l2.data_ptr(),
                             sigma.ctypes.data, _aligned_ptr(ws), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()),
                             _stream()), "lq_factorize")
    return l1, l2, sigma


def decompose(w: torch.Tensor, rank: int, cfg: Config, iters: int, early_stop: bool = False, row_w=None, col_w=None,
              seed: int = 0, params: SvdParams | None = None, want_dense: bool = False,
              workspace: torch.Tensor | None = None):
    """LQ(W, F, c, r): -> dict(L1, L2, codes, scale_idx, v, Q, err, trace, iters_done, sigma)."""
    d, k = w.shape
    n = d * k
    nb = n // max(cfg.block, 1)
    ng = (nb + max(cfg.scale_block, 1) - 1) // max(cfg.scale_block, 1)
    need = _lib.lq_decompose_workspace_bytes(d, k, rank, _pp(params))
    ws = workspace if workspace is not None else _workspace(need, w.device)
    dev = w.device
    out = dict(L1=torch.empty((d, max(rank, 1)), dtype=torch.float32, device=dev),
               L2=torch.empty((max(rank, 1), k), dtype=torch.float32, device=dev),
               codes=torch.empty(max(codes_bytes(n, cfg.bits), 1), dtype=torch.uint8, device=dev),
               scale_idx=torch.empty(max(nb, 1), dtype=torch.uint8, device=dev),
               v=torch.empty(max(ng, 1), dtype=torch.float32, device=dev),
               Q=torch.empty((d, k), dtype=torch.float32, device=dev) if want_dense else None)
    err = C.c_double(float("nan"))
    done = C.c_int32(0)
    trace = np.full(max(iters, 1), np.nan)
    sigma = np.zeros(max(rank, 1))
    _check(_lib.lq_decompose(_dev(w, torch.float32, "w"), d, k, rank, cfg, iters, int(early_stop),
                             _dev(row_w, torch.float32, "row_w"), _dev(col_w, torch.float32, "col_w"), seed,
                             _pp(params), out["L1"].data_ptr(), out["L2"].data_ptr(), out["codes"].data_ptr(),
                             out["scale_idx"].data_ptr(), out["v"].data_ptr(),
                             None if out["Q"] is None else out["Q"].data_ptr(), C.addressof(err), trace.ctypes.data,
                             C.addressof(done), sigma.ctypes.data, _aligned_ptr(ws),
                             ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream()), "lq_decompose")
    out.update(err=err.value, trace=trace, iters_done=done.value, sigma=sigma)
    return out


def error_table_workspace(d: int, k: int, rank: int, n_cfgs: int, params: SvdParams | None = None, device="cuda"):
    return _workspace(_lib.lq_error_table_workspace_bytes(d, k, rank, n_cfgs, _pp(params)), device)


def error_table(w: torch.Tensor, rank: int, cfgs, iters: int, early_stop: bool = False, row_w=None, col_w=None,
                seed: int = 0, params: SvdParams | None = None, workspace: torch.Tensor | None = None,
                want_trace: bool = False):
    """Algorithm 3 inner loops for one matrix: -> (err_sq, storage_bits[, trace]) numpy float64."""
    d, k = w.shape
    arr = (Config * max(len(cfgs), 1))(*cfgs)
    ws = workspace if workspace is not None else error_table_workspace(d, k, rank, len(cfgs), params, w.device)
    e = np.zeros(max(len(cfgs), 1))
    s = np.zeros(max(len(cfgs), 1))
    tr = np.full((max(len(cfgs), 1), max(iters, 1)), np.nan) if want_trace else None
    _check(_lib.lq_error_table(_dev(w, torch.float32, "w"), d, k, rank, C.addressof(arr), len(cfgs), iters,
                               int(early_stop), _dev(row_w, torch.float32, "row_w"),
                               _dev(col_w, torch.float32, "col_w"), seed, _pp(params), e.ctypes.data, s.ctypes.data,
                               None if tr is None else tr.ctypes.data, _aligned_ptr(ws),
                               ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream()), "lq_error_table")
    return (e, s, tr) if want_trace else (e, s)


def fisher_row_col(f: torch.Tensor):
    """RowAverage / ColAverage of sqrt(F) (Algorithm 4) as Fisher-scale vectors for row_w / col_w."""
    d, k = f.shape
    ws = _workspace(_lib.lq_fisher_row_col_workspace_bytes(d, k), f.device)
    row_w = torch.empty(d, dtype=torch.float32, device=f.device)
    col_w = torch.empty(k, dtype=torch.float32, device=f.device)
    _check(_lib.lq_fisher_row_col(_dev(f, torch.float32, "f"), d, k, row_w.data_ptr(), col_w.data_ptr(),
                                  _aligned_ptr(ws), ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream()),
           "lq_fisher_row_col")
    return row_w, col_w


def release_streams() -> None:
    """Destroys the idle HIP streams the library keeps for lq_error_table's interleaved sub-batches."""
    _check(_lib.lq_release_streams(), "lq_release_streams")


def profile_enable(on: bool) -> None:
    _check(_lib.lq_profile_enable(1 if on else 0), "lq_profile_enable")


def profile_reset() -> None:
    _check(_lib.lq_profile_reset(), "lq_profile_reset")


def profile_read() -> dict:
    """-> {kernel class name: (total_ms, launches, algorithmic work)} for classes that were launched."""
    out = {}
    for cls in range(_lib.lq_profile_num_classes()):
        ms, n, wk = C.c_double(0), C.c_int64(0), C.c_double(0)
        _check(_lib.lq_profile_read(cls, C.addressof(ms), C.addressof(n), C.addressof(wk)), "lq_profile_read")
        if n.value:
            out[_lib.lq_profile_class_name(cls).decode()] = (ms.value, n.value, wk.value)
    return out


def matmul_workspace(m: int, d: int, k: int, rank: int, device="cuda") -> torch.Tensor:
    return _workspace(_lib.lq_matmul_workspace_bytes(m, d, k, rank), device)


def matmul(x: torch.Tensor, codes: torch.Tensor, scale_idx: torch.Tensor, v: torch.Tensor, cfg: Config, k: int,
           l1: torch.Tensor | None = None, l2: torch.Tensor | None = None, precision: int = 0,
           out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X (Q + L1 L2) with Q (d x k) in quantized form, dequantized inside the GEMM."""
    m, d = x.shape
    rank = 0 if l1 is None else l1.shape[1]
    if out is None:
        out = torch.empty((m, k), dtype=torch.float32, device=x.device)
    ws = workspace if workspace is not None else matmul_workspace(m, d, k, rank, x.device)
    _check(_lib.lq_matmul(_dev(x, torch.float32, "x"), m, d, k, _dev(codes, torch.uint8, "codes"),
                          _dev(scale_idx, torch.uint8, "scale_idx"), _dev(v, torch.float32, "v"), cfg,
                          _dev(l1, torch.float32, "l1"), _dev(l2, torch.float32, "l2"), rank, precision,
                          _dev(out, torch.float32, "out"), _aligned_ptr(ws),
                          ws.numel() - (_aligned_ptr(ws) - ws.data_ptr()), _stream()), "lq_matmul")
    return out


def matmul_few_rows_static(x: torch.Tensor, codes: torch.Tensor, scale_idx: torch.Tensor, v: torch.Tensor, cfg: Config,
                           k: int, l1: torch.Tensor | None = None, l2: torch.Tensor | None = None,
                           out: torch.Tensor | None = None) -> torch.Tensor:
    """Y = X (Q + L1 L2) for at most 8 rows of X through the entry point that allocates nothing: its partial sums live
    in the library's fixed device array (lq_matmul_few_rows_static).  `out`: m x k fp32 tensor to write into."""
    m, d = x.shape
    rank = 0 if l1 is None else l1.shape[1]
    if out is None:
        out = torch.empty((m, k), dtype=torch.float32, device=x.device)
    _check(_lib.lq_matmul_few_rows_static(_dev(x, torch.float32, "x"), m, d, k, _dev(codes, torch.uint8, "codes"),
                                          _dev(scale_idx, torch.uint8, "scale_idx"), _dev(v, torch.float32, "v"), cfg,
                                          _dev(l1, torch.float32, "l1"), _dev(l2, torch.float32, "l2"), rank,
                                          _dev(out, torch.float32, "out"), _stream()), "lq_matmul_few_rows_static")
    return out


def assign_configs(err: np.ndarray, storage: np.ndarray, budget_bits: float, node_limit: int = 0):
    """ILPSolve: -> (choice int32[n_matrices], total_err, total_storage, lower_bound).  Host only."""
    err = np.ascontiguousarray(err, np.float64)
    storage = np.ascontiguousarray(storage, np.float64)
    n, c = err.shape
    assert storage.shape == (n, c)
    choice = np.zeros(n, np.int32)
    te, ts, lb = C.c_double(0), C.c_double(0), C.c_double(0)
    _check(_lib.lq_assign_configs(err.ctypes.data, storage.ctypes.data, n, c, float(budget_bits), node_limit,
                                  choice.ctypes.data, C.addressof(te), C.addressof(ts), C.addressof(lb)),
           "lq_assign_configs")
    return choice, te.value, ts.value, lb.value


def lq_lora_decompose(matrices, rank: int, cfgs, bits_per_weight: float, iters: int, fishers=None, seed: int = 0,
                      params: SvdParams | None = None):
    """Algorithm 1 without the finetuning: error tables of all matrices (GetConfig, Algorithm 3), the assignment under
    the budget bits_per_weight * (total number of weights), then the decomposition of every matrix with its chosen
    configuration.  matrices: list of fp32 GPU tensors; fishers: None or a list of (row_w, col_w) pairs.
    -> (choice, list of lq.decompose results, err table, storage table)."""
    n = len(matrices)
    err = np.zeros((n, len(cfgs)))
    sto = np.zeros((n, len(cfgs)))
    for i, w in enumerate(matrices):
        rw, cw = fishers[i] if fishers is not None else (None, None)
        err[i], sto[i] = error_table(w, rank, cfgs, iters, row_w=rw, col_w=cw, seed=seed, params=params)
    budget = bits_per_weight * sum(w.numel() for w in matrices)
    choice, _, _, _ = assign_configs(err, sto, budget)
    outs = []
    for i, w in enumerate(matrices):
        rw, cw = fishers[i] if fishers is not None else (None, None)
        outs.append(decompose(w, rank, cfgs[choice[i]], iters, row_w=rw, col_w=cw, seed=seed, params=params))
    return choice, outs, err, sto
