"""GPU checks of the randomized SVD's building blocks against plain numpy (fp64) references."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    from paper_2311_12023_amd import lq
    import testing_lib
    L = testing_lib.load()
    return torch, lq, L


def up32(x):
    return (x + 31) // 32 * 32


# wgs: workgroups the reduction steps are dealt out to (None: no scratch, reductions are never cut; 0: device default).
# The cases cover shares much shorter than one reduction, shares that run over several problems of a batch with cut
# ends, a single workgroup, and shapes that are ragged against the 256 / 128-column tiles and the 32-deep steps.
@pytest.mark.parametrize("mode,l,big,K,batch,wgs", [
    (0, 32, 200, 160, 1, None), (0, 64, 768, 768, 1, 5), (0, 96, 130, 1040, 3, 7), (0, 128, 1000, 4096, 1, 0),
    (0, 256, 300, 512, 2, None), (0, 96, 1500, 700, 5, 20), (0, 96, 1500, 700, 1, 1), (0, 96, 520, 4096, 1, 64),
    (0, 96, 300, 1000, 7, 6),
    (1, 32, 208, 150, 1, None), (1, 64, 768, 768, 1, 5), (1, 96, 1040, 131, 3, 7), (1, 128, 4096, 1000, 1, 0),
    (1, 256, 512, 300, 2, None), (1, 160, 96, 32, 1, None), (1, 96, 1500, 700, 5, 20), (1, 96, 520, 4096, 1, 64),
    (1, 96, 300, 1000, 7, 6)])
@pytest.mark.parametrize("precision", [0, 1])
def test_wide_gemm(env, mode, l, big, K, batch, wgs, precision):
    torch, lq, L = env
    rng = np.random.default_rng(l * 7 + big + mode)
    ldx = up32(K)
    x = np.zeros((batch, l, ldx), np.float32)
    x[:, :, :K] = rng.standard_normal((batch, l, K))
    a = rng.standard_normal((batch, big, K) if mode == 0 else (batch, K, big)).astype(np.float32)
    ldc = up32(big)
    xt, at = torch.from_numpy(x).cuda(), torch.from_numpy(a).cuda()
    ct = torch.full((batch, l, ldc), 7.0, dtype=torch.float32, device="cuda")
    nfl = 0 if wgs is None else L.lq_test_wide_gemm_part_floats(l, wgs)
    part = torch.full((max(nfl, 1),), float("nan"), dtype=torch.float32, device="cuda")
    rc = L.lq_test_wide_gemm(mode, l, big, K, xt.data_ptr(), ldx, at.data_ptr(), a.shape[2], ct.data_ptr(), ldc, batch,
                             wgs or 0, part.data_ptr() if nfl else None, nfl, precision, None)
    assert rc == 0
    torch.cuda.synchronize()
    got = ct.cpu().numpy()
    a64 = a.astype(np.float64)
    ref = np.matmul(x[:, :, :K].astype(np.float64), a64.transpose(0, 2, 1) if mode == 0 else a64)
    scale = np.sqrt(K)
    # fp32 MFMA: rounding of the accumulation only.  Split bf16: each product carries about 2^-16 relative error
    assert np.max(np.abs(got[:, :, :big] - ref)) < (2e-5 if precision == 0 else 1.5e-4) * scale
    if precision == 1:
        assert np.sqrt(np.mean((got[:, :, :big] - ref) ** 2)) < 2e-5 * scale
    assert np.all(got[:, :, big:] == 7.0)           # columns past the matrix are never written
    # same call again: the summation order is fixed, so the result is too
    ct2 = torch.full((batch, l, ldc), 7.0, dtype=torch.float32, device="cuda")
    rc = L.lq_test_wide_gemm(mode, l, big, K, xt.data_ptr(), ldx, at.data_ptr(), a.shape[2], ct2.data_ptr(), ldc, batch,
                             wgs or 0, part.data_ptr() if nfl else None, nfl, precision, None)
    assert rc == 0 and torch.equal(ct, ct2)


def up64(x):
    return (x + 63) // 64 * 64


# The products against an fp16 operand (the warm iterations' residual): ragged against the 256-column tiles and the
# 64-deep steps, cut and uncut reductions, fixed and data-derived scaling of X.  The reference multiplies the very same
# fp16 values in fp64, so what is left is the rounding (one plane) or the fp16 hi/lo split (two planes) of X and fp32
# accumulation.
F16_SHAPES = [
    (0, 32, 200, 160, 1, None), (0, 64, 768, 768, 1, 5), (0, 96, 130, 1040, 3, 7), (0, 96, 1000, 4096, 1, 0),
    (0, 96, 1500, 704, 5, 20), (0, 96, 1500, 704, 1, 1), (0, 96, 520, 4096, 1, 64), (0, 96, 300, 1000, 7, 6),
    (1, 32, 208, 150, 1, None), (1, 64, 768, 768, 1, 5), (1, 96, 1040, 131, 3, 7), (1, 96, 4096, 1000, 1, 0),
    (1, 96, 1500, 700, 5, 20), (1, 96, 520, 4096, 1, 64), (1, 96, 300, 1000, 7, 6), (1, 64, 96, 33, 1, None)]


# the byte plane (planes == 2) is read in NN layout (mode 1) only
@pytest.mark.parametrize("mode,l,big,K,batch,wgs,scaling,planes",
                         [sh + sp for sh in F16_SHAPES for sp in (("fixed", 1), ("lam", 1), ("fixed", 2))
                          if sp[1] == 1 or sh[0] == 1])
def test_wide_gemm_f16(env, mode, l, big, K, batch, wgs, scaling, planes):
    torch, lq, L = env
    rng = np.random.default_rng(l * 11 + big + mode)
    ldx = up64(K)
    x = np.zeros((batch, l, ldx), np.float32)
    x[:, :, :K] = rng.standard_normal((batch, l, K)) * (37.0 if scaling == "lam" else 0.02)
    a32 = (rng.standard_normal((batch, big, K) if mode == 0 else (batch, K, big)) * 3.0).astype(np.float32)
    a = a32.astype(np.float16)
    # planes == 2: the lo plane is one byte per element, the upper byte (round to nearest even) of the fp16 number
    # 2048 (a32 - a); the product is taken with a + alo, alo the value those bytes stand for
    lo_bits = ((a32 - a.astype(np.float32)) * 2048.0).astype(np.float16).view(np.uint16).astype(np.uint32)
    lo8 = ((lo_bits + 0x7F + ((lo_bits >> 8) & 1)) >> 8).astype(np.uint8)
    alo = (lo8.astype(np.uint16) << 8).view(np.float16).astype(np.float64) / 2048.0
    ldc = up32(big)
    xt, at, alt = torch.from_numpy(x).cuda(), torch.from_numpy(a).cuda(), torch.from_numpy(lo8).cuda()
    ct = torch.full((batch, l, ldc), 7.0, dtype=torch.float32, device="cuda")
    nfl = 0 if wgs is None else L.lq_test_wide_gemm_part_floats(l, wgs)
    part = torch.full((max(nfl, 1),), float("nan"), dtype=torch.float32, device="cuda")
    lam = torch.from_numpy(np.max(np.sum(x.astype(np.float64) ** 2, axis=2), axis=1)).cuda()     # per problem
    out_scale = 0.25

    def run(dst):
        rc = L.lq_test_wide_gemm_f16(mode, l, big, K, xt.data_ptr(), ldx, at.data_ptr(),
                                     alt.data_ptr() if planes == 2 else None, a.shape[2], dst.data_ptr(), ldc,
                                     batch, wgs or 0, part.data_ptr() if nfl else None, nfl, 64.0,
                                     lam.data_ptr() if scaling == "lam" else None, out_scale, None)
        assert rc == 0
        torch.cuda.synchronize()

    run(ct)
    got = ct.cpu().numpy()
    a64 = a.astype(np.float64) + (alo if planes == 2 else 0.0)
    ref = np.matmul(x[:, :, :K].astype(np.float64), a64.transpose(0, 2, 1) if mode == 0 else a64) * out_scale
    if scaling == "fixed":
        ref *= 64.0
    err = np.abs(got[:, :, :big] - ref)
    # two planes: X is split into fp16 hi + lo (2^-21); one plane: X is rounded to fp16 (2^-12 per entry, random sign)
    tol_max, tol_rms = (2e-5, 2e-6) if planes == 2 else (2e-3, 3e-4)
    assert err.max() < tol_max * np.abs(ref).max(), (err.max(), np.abs(ref).max())
    assert np.sqrt(np.mean(err ** 2)) < tol_rms * np.sqrt(np.mean(ref ** 2))
    assert np.all(got[:, :, big:] == 7.0)           # columns past the matrix are never written
    ct2 = torch.full((batch, l, ldc), 7.0, dtype=torch.float32, device="cuda")
    run(ct2)
    assert torch.equal(ct, ct2)


def test_wide_gemm_f16_rejects_byte_plane_in_nt_mode(env):
    torch, lq, L = env
    x = torch.zeros((32, 64), dtype=torch.float32, device="cuda")
    a = torch.zeros((64, 64), dtype=torch.float16, device="cuda")
    lo = torch.zeros((64, 64), dtype=torch.uint8, device="cuda")
    c = torch.zeros((32, 64), dtype=torch.float32, device="cuda")
    args = (32, 64, 64, x.data_ptr(), 64, a.data_ptr(), lo.data_ptr(), 64, c.data_ptr(), 64, 1, 0, None, 0, 1.0, None, 1.0, None)
    assert L.lq_test_wide_gemm_f16(0, *args) != 0
    assert L.lq_test_wide_gemm_f16(1, *args) == 0
    torch.cuda.synchronize()
    assert torch.count_nonzero(c) == 0


@pytest.mark.parametrize("use_alt", [True, False])
@pytest.mark.parametrize("l,m", [(32, 100), (64, 768), (96, 4096), (128, 1000), (256, 2048)])
def test_orthonormalize(env, l, m, use_alt):
    torch, lq, L = env
    rng = np.random.default_rng(l + m)
    ld = up32(m)
    x = np.zeros((l, ld), np.float32)
    # rows with a two-decade spread of singular values
    base = rng.standard_normal((l, m))
    u, _, vt = np.linalg.svd(base, full_matrices=False)
    x[:, :m] = (u * np.logspace(0, -2, min(l, m))) @ vt
    xt = torch.from_numpy(x).cuda()
    scratch = torch.empty(17 * l * l, dtype=torch.float64, device="cuda")
    alt = torch.zeros((l, ld), dtype=torch.float32, device="cuda")
    assert L.lq_test_orthonormalize(xt.data_ptr(), l, m, ld, scratch.data_ptr(), alt.data_ptr() if use_alt else None,
                                    None) == 0
    torch.cuda.synchronize()
    q = xt.cpu().numpy().astype(np.float64)
    if l <= m:
        assert np.max(np.abs(q @ q.T - np.eye(l))) < 5e-5
        # same row space, nested: row i of q lies in the span of the first i+1 rows of x
        coef = q[:, :m] @ np.linalg.pinv(x[:, :m].astype(np.float64))
        assert np.max(np.abs(np.triu(coef, 1))) < 1e-2 * np.max(np.abs(coef))
    assert np.all(q[:, m:] == 0)


@pytest.mark.parametrize("l", [96, 256])
def test_orthonormalize_rows_of_very_different_length(env, l):
    """Rows kept at unit length beside rows that a filter has amplified by many orders of magnitude (the cold start's
    locked and filtered rows): every row still gets its direction, none is taken for linearly dependent."""
    torch, lq, L = env
    rng = np.random.default_rng(7 * l)
    m = 1500
    ld = up32(m)
    q0, _ = np.linalg.qr(rng.standard_normal((m, l)))
    scale = np.ones(l)
    scale[4:] = 10.0 ** rng.uniform(5, 9, l - 4)          # rows 0..3 at unit length, the rest 1e5 .. 1e9 times longer
    mix = np.eye(l) + 1e-3 * np.tril(rng.standard_normal((l, l)), -1)      # and not quite orthogonal
    x = np.zeros((l, ld), np.float32)
    x[:, :m] = (scale[:, None] * (mix @ q0.T)).astype(np.float32)
    xt = torch.from_numpy(x).cuda()
    scratch = torch.empty(17 * l * l, dtype=torch.float64, device="cuda")
    alt = torch.zeros((l, ld), dtype=torch.float32, device="cuda")
    assert L.lq_test_orthonormalize(xt.data_ptr(), l, m, ld, scratch.data_ptr(), alt.data_ptr(), None) == 0
    torch.cuda.synchronize()
    q = xt.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(q @ q.T - np.eye(l))) < 5e-5
    assert np.max(np.abs(np.abs(np.sum(q[:, :m] * q0.T, axis=1)) - 1.0)) < 1e-4      # row i is +-(row i of q0^T), to the mixing


def test_filter_small_kernels(env):
    """lincomb3, deflate_rows and ritz_residual against numpy."""
    torch, lq, L = env
    rng = np.random.default_rng(99)
    l, m = 64, 1003
    ld = up32(m)
    def rows():
        a = np.zeros((l, ld), np.float32)
        a[:, :m] = rng.standard_normal((l, m))
        return a
    x, y, z = rows(), rows(), rows()
    for third in (True, False):
        xt = torch.from_numpy(x.copy()).cuda()
        yt, zt = torch.from_numpy(y).cuda(), torch.from_numpy(z).cuda()
        assert L.lq_test_lincomb3(xt.data_ptr(), C.c_float(0.75), yt.data_ptr(), C.c_float(-2.0),
                                  zt.data_ptr() if third else None, C.c_float(-1.0), l, ld, None) == 0
        torch.cuda.synchronize()
        ref = 0.75 * x.astype(np.float64) - 2.0 * y + (-1.0 * z if third else 0.0)
        assert np.max(np.abs(xt.cpu().numpy() - ref)) < 1e-5
    # deflation against 0, 5 and 16 orthonormal rows
    lock_rows = np.zeros((l, ld), np.float32)
    qq, _ = np.linalg.qr(rng.standard_normal((m, l)))
    lock_rows[:, :m] = qq.T
    lt = torch.from_numpy(lock_rows).cuda()
    for locked in (0, 5, 16):
        big = (x * np.float32(1e6)).astype(np.float32)
        xt = torch.from_numpy(big.copy()).cuda()
        assert L.lq_test_deflate_rows(xt.data_ptr(), lt.data_ptr(), l, locked, m, ld, None) == 0
        torch.cuda.synchronize()
        got = xt.cpu().numpy().astype(np.float64)
        u = lock_rows[:locked].astype(np.float64)
        ref = big.astype(np.float64) - (big.astype(np.float64) @ u.T) @ u
        ref[:locked] = u
        assert np.max(np.abs(got - ref)) < 2e-6 * np.max(np.abs(big))
        if locked:
            assert np.max(np.abs(got[locked:] @ u.T)) < 2e-6 * np.max(np.abs(big)) * np.sqrt(m)
            assert np.array_equal(got[:locked], u)
    assert L.lq_test_deflate_rows(xt.data_ptr(), lt.data_ptr(), l, 17, m, ld, None) != 0      # more than the kernel holds
    # residuals of Ritz pairs
    lam = rng.uniform(0.5, 2.0, l)
    g = (lam[:, None] * y.astype(np.float64) + 1e-3 * z).astype(np.float32)
    gt, yt = torch.from_numpy(g).cuda(), torch.from_numpy(y).cuda()
    lamt = torch.from_numpy(lam).cuda()
    res = torch.zeros(l, dtype=torch.float64, device="cuda")
    assert L.lq_test_ritz_residual(gt.data_ptr(), yt.data_ptr(), lamt.data_ptr(), 40, m, ld, res.data_ptr(), None) == 0
    torch.cuda.synchronize()
    ref = np.sum((g.astype(np.float64) - lam[:, None] * y.astype(np.float64))[:, :m] ** 2, axis=1)
    got = res.cpu().numpy()
    assert np.max(np.abs(got[:40] - ref[:40]) / ref[:40]) < 1e-10 and np.all(got[40:] == 0)


@pytest.mark.parametrize("l", [32, 64, 96, 128, 256])
def test_sym_eig(env, l):
    torch, lq, L = env
    rng = np.random.default_rng(l)
    b = rng.standard_normal((l, 3 * l)) * np.logspace(1, 0, l)[:, None]
    g = b @ b.T
    gt = torch.from_numpy(g.copy()).cuda()
    ut = torch.empty((l, l), dtype=torch.float32, device="cuda")
    lam = torch.empty(l, dtype=torch.float64, device="cuda")
    scratch = torch.empty(l * l, dtype=torch.float64, device="cuda")
    assert L.lq_test_sym_eig(gt.data_ptr(), l, ut.data_ptr(), lam.data_ptr(), scratch.data_ptr(), None) == 0
    torch.cuda.synchronize()
    lam_h, u = lam.cpu().numpy(), ut.cpu().numpy().astype(np.float64)
    ref = np.sort(np.linalg.eigvalsh(g))[::-1]
    assert np.all(np.diff(lam_h) <= 0)
    assert np.max(np.abs(lam_h - ref) / ref) < 1e-9
    assert np.max(np.abs(u @ u.T - np.eye(l))) < 1e-5
    assert np.max(np.abs(u @ g @ u.T - np.diag(lam_h))) < 1e-4 * lam_h[0]


@pytest.mark.parametrize("l", [32, 64, 96, 128])
@pytest.mark.parametrize("near_diagonal", [False, True])
def test_sym_eig_fast(env, l, near_diagonal):
    torch, lq, L = env
    rng = np.random.default_rng(l + 1000)
    if near_diagonal:      # the warm-started case: nearly orthogonal rows with a cluster of close values
        lam = np.concatenate([[900.0, 400.0], np.linspace(10.0, 9.0, l - 2)])
        pert = 1e-2 * rng.standard_normal((l, l))
        q, _ = np.linalg.qr(np.eye(l) + pert)
        g = (q * lam) @ q.T
    else:
        b = rng.standard_normal((l, 3 * l)) * np.logspace(1, 0, l)[:, None]
        g = b @ b.T
    g = (g + g.T) / 2
    gt = torch.from_numpy(g.copy()).cuda()
    ut = torch.empty((l, l), dtype=torch.float32, device="cuda")
    lam_d = torch.empty(l, dtype=torch.float64, device="cuda")
    assert L.lq_test_sym_eig_fast(gt.data_ptr(), l, ut.data_ptr(), lam_d.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert np.array_equal(gt.cpu().numpy(), g)
    u = ut.cpu().numpy().astype(np.float64)
    ref = np.sort(np.linalg.eigvalsh(g))[::-1]
    assert np.max(np.abs(u @ u.T - np.eye(l))) < 2e-5
    rq = np.einsum("ij,jk,ik->i", u, g, u)                      # Rayleigh quotients of the returned rows
    assert np.max(np.abs(rq - ref) / ref) < 5e-7                # second-order accurate eigenvalues
    off = u @ g @ u.T - np.diag(rq)
    assert np.max(np.abs(off)) < 2e-5 * ref[0]
    assert np.max(np.abs(lam_d.cpu().numpy() - ref) / ref) < 1e-4


def test_report_lds_limit(env):
    torch, lq, L = env
    lim = L.lq_test_lds_limit()
    print("LDS bytes per workgroup reported by the device:", lim)
    assert lim >= 65536
