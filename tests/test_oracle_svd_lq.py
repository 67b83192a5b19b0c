"""Pins for the oracle's SVD, Factorize (Algorithm 4), LQ loop (Algorithm 2) and error table
(Algorithm 3): LAPACK cross-checks, closed forms, Eckart-Young, and the invariants the
alternating scheme must satisfy."""
import numpy as np
import pytest

from paper_2311_12023_amd import gen


def test_jacobi_svd_closed_forms(oracle):
    u, s, vt = oracle.svd(np.diag([3.0, -5.0, 1.0]))
    assert np.allclose(s, [5, 3, 1], atol=1e-14)
    assert np.allclose((u * s) @ vt, np.diag([3.0, -5.0, 1.0]), atol=1e-14)
    a = np.outer([1.0, 2.0, 2.0], [3.0, 4.0])            # rank one: sigma = |x||y| = 3*5
    u, s, vt = oracle.svd(a)
    assert abs(s[0] - 15.0) < 1e-13 and abs(s[1]) < 1e-13
    a = np.array([[1.0, 2.0], [3.0, 4.0]])               # 2x2: sigma^2 = (30 +- sqrt(884))/2
    _, s, _ = oracle.svd(a)
    assert np.allclose(s ** 2, [(30 + np.sqrt(884)) / 2, (30 - np.sqrt(884)) / 2], rtol=1e-12)


@pytest.mark.parametrize("shape", [(40, 40), (33, 70), (70, 33), (5, 128), (128, 1)])
def test_jacobi_svd_against_lapack(oracle, shape):
    rng = np.random.default_rng(shape[0] * 1000 + shape[1])
    a = rng.standard_normal(shape)
    u, s, vt = oracle.svd(a)
    m = min(shape)
    assert np.all(np.diff(s) <= 0)
    assert np.max(np.abs(s - np.linalg.svd(a, compute_uv=False))) <= 1e-12 * s[0]
    assert np.linalg.norm((u * s) @ vt - a) <= 1e-12 * np.linalg.norm(a)
    assert np.max(np.abs(u.T @ u - np.eye(m))) < 1e-12
    assert np.max(np.abs(vt @ vt.T - np.eye(m))) < 1e-12


def test_jacobi_svd_planted_spectrum(oracle):
    rng = np.random.default_rng(3)
    uu, _ = np.linalg.qr(rng.standard_normal((50, 6)))
    vv, _ = np.linalg.qr(rng.standard_normal((80, 6)))
    sig = np.array([9.0, 4.0, 3.5, 3.4999, 1.0, 0.25])
    _, s, _ = oracle.svd((uu * sig) @ vv.T)
    assert np.allclose(s[:6], sig, rtol=1e-12) and np.all(s[6:] < 1e-13)


def test_factorize_eckart_young_and_balance(oracle):
    w = gen.weight_matrix(48, 80, 11, 6)
    r = 5
    l1, l2, sg = oracle.factorize(w, r)
    sv = np.linalg.svd(w.astype(np.float64), compute_uv=False)
    assert np.allclose(sg, sv[:r], rtol=1e-12)
    resid = w.astype(np.float64) - l1.astype(np.float64) @ l2.astype(np.float64)
    # rank-r error^2 equals the sum of the discarded sigma^2 (Eq. 2, the SVD step is the argmin)
    assert abs(np.sum(resid ** 2) - np.sum(sv[r:] ** 2)) < 1e-5 * np.sum(sv[r:] ** 2)
    # L1 = U sqrt(S), L2 = sqrt(S) Vt: both carry sqrt(sigma) per component
    assert np.allclose(np.linalg.norm(l1, axis=0) ** 2, sv[:r], rtol=1e-5)
    assert np.allclose(np.linalg.norm(l2, axis=1) ** 2, sv[:r], rtol=1e-5)
    assert np.allclose(l1.T.astype(np.float64) @ l1, np.diag(sv[:r]), atol=1e-5)


def test_factorize_weighted(oracle):
    d, k, r = 40, 56, 4
    w = gen.weight_matrix(d, k, 12, 6)
    rw = gen.positive_weights(d, 21)
    cw = gen.positive_weights(k, 22)
    l1, l2, sg = oracle.factorize(w, r, rw, cw)
    dr = np.sqrt(rw.astype(np.float64)); dc = np.sqrt(cw.astype(np.float64))
    sw = dr[:, None] * w.astype(np.float64) * dc[None, :]
    sv = np.linalg.svd(sw, compute_uv=False)
    assert np.allclose(sg, sv[:r], rtol=1e-12)
    resid = w.astype(np.float64) - l1.astype(np.float64) @ l2.astype(np.float64)
    werr = np.sum((dr[:, None] * resid * dc[None, :]) ** 2)
    # Eckart-Young on D_row W D_col  (Eq. 5)
    assert abs(werr - np.sum(sv[r:] ** 2)) < 1e-4 * np.sum(sv[r:] ** 2)
    # it is the weighted optimum for this rank-one weighting: random rank-r competitors are worse
    rng = np.random.default_rng(0)
    for _ in range(20):
        p1 = l1 + 1e-3 * rng.standard_normal(l1.shape).astype(np.float32)
        p2 = l2 + 1e-3 * rng.standard_normal(l2.shape).astype(np.float32)
        e = np.sum((dr[:, None] * (w.astype(np.float64) - p1.astype(np.float64) @ p2) * dc[None, :]) ** 2)
        assert e >= werr * (1 - 1e-9)
    # and the unweighted factorization is worse under the weighted norm
    u1, u2, _ = oracle.factorize(w, r)
    e_unw = np.sum((dr[:, None] * (w.astype(np.float64) - u1.astype(np.float64) @ u2) * dc[None, :]) ** 2)
    assert e_unw > werr
    # uniform weights reproduce the unweighted result bit for bit
    o1, o2, _ = oracle.factorize(w, r, np.ones(d, np.float32), np.ones(k, np.float32))
    assert np.array_equal(o1, u1) and np.array_equal(o2, u2)


def test_fisher_row_col_rank_one_is_exact(oracle):
    rng = np.random.default_rng(4)
    a = np.exp(rng.standard_normal(30)); b = np.exp(rng.standard_normal(50))
    f = np.outer(a, b) ** 2                       # sqrt(F) = a b^T
    rw, cw = oracle.fisher_row_col(f)
    assert np.allclose(np.outer(rw, cw), f, rtol=1e-5)
    # general F: D_row / D_col are the row / column means of sqrt(F) up to one constant
    f = gen.fisher_matrix(30, 50, 9)
    rw, cw = oracle.fisher_row_col(f)
    sf = np.sqrt(f)
    assert np.allclose(np.sqrt(rw), sf.mean(axis=1), rtol=1e-6)
    assert np.allclose(np.sqrt(cw) * sf.mean(), sf.mean(axis=0), rtol=1e-6)


def independent_first_step(oracle, w, r, cfg, rw=None, cw=None):
    """First LQ iteration rebuilt with LAPACK for the SVD: Q0 = 0, so Factorize sees W itself."""
    w64 = w.astype(np.float64)
    if rw is None:
        u, s, vt = np.linalg.svd(w64, full_matrices=False)
        l1 = (u[:, :r] * np.sqrt(s[:r])).astype(np.float32)
        l2 = (np.sqrt(s[:r])[:, None] * vt[:r]).astype(np.float32)
    else:
        dr = np.sqrt(rw.astype(np.float64)); dc = np.sqrt(cw.astype(np.float64))
        u, s, vt = np.linalg.svd(dr[:, None] * w64 * dc[None, :], full_matrices=False)
        l1 = ((u[:, :r] * np.sqrt(s[:r])) / dr[:, None]).astype(np.float32)
        l2 = ((np.sqrt(s[:r])[:, None] * vt[:r]) / dc[None, :]).astype(np.float32)
    low = l1.astype(np.float64) @ l2.astype(np.float64)
    t = (w64 - low).astype(np.float32)
    codes, sidx, v, _ = oracle.quantize(t.ravel(), cfg)
    q = oracle.dequantize(codes, sidx, v, cfg).reshape(w.shape)
    diff = w64 - low - q
    wt = 1.0 if rw is None else np.outer(rw.astype(np.float64), cw.astype(np.float64))
    return np.sqrt(np.sum(wt * diff ** 2)), q


def test_lq_first_iteration_against_lapack(oracle):
    w = gen.weight_matrix(64, 128, 31, 8)
    cfg = oracle.config(3, 16, 16)
    out = oracle.lq(w, 6, cfg, 1)
    eps, q = independent_first_step(oracle, w, 6, cfg)
    assert out["iters_done"] == 1
    assert abs(out["trace"][0] - eps) < 1e-6 * eps and out["err"] == out["trace"][0]
    assert np.mean(out["Q"] != q) < 1e-3          # sign/rounding of the two SVDs may flip a stray code
    # returned pieces are consistent with one another
    assert np.array_equal(oracle.dequantize(out["codes"], out["scale_idx"], out["v"], cfg).reshape(w.shape), out["Q"])
    resid = w.astype(np.float64) - out["Q"] - out["L1"].astype(np.float64) @ out["L2"].astype(np.float64)
    assert abs(np.linalg.norm(resid) - out["err"]) < 1e-9 * out["err"]


def test_lq_quantized_initialisation(oracle):
    """Q(0) = Quantize(W) (Section 3.1, footnote): the first Factorize sees W - Quantize(W); with one iteration this is
    the "SVD of the quantization residual" correction, built here from LAPACK and the separately pinned quantizer."""
    w = gen.weight_matrix(64, 128, 33, 8)
    cfg = oracle.config(3, 16, 16)
    r = 6
    out = oracle.lq(w, r, cfg, 1, init_quantized=True)
    c0, s0, v0, _ = oracle.quantize(w.ravel(), cfg)
    q0 = oracle.dequantize(c0, s0, v0, cfg).reshape(w.shape)
    u, sg, vt = np.linalg.svd((w - q0).astype(np.float64), full_matrices=False)
    low = (u[:, :r] * sg[:r]) @ vt[:r]
    assert np.allclose(out["sigma"], sg[:r], rtol=1e-9)
    assert np.allclose(out["L1"].astype(np.float64) @ out["L2"].astype(np.float64), low, atol=1e-6)
    c1, s1, v1, _ = oracle.quantize((w.astype(np.float64) - low).astype(np.float32).ravel(), cfg)
    q1 = oracle.dequantize(c1, s1, v1, cfg).reshape(w.shape)
    assert np.mean(out["Q"] != q1) < 1e-3
    eps = np.linalg.norm(w.astype(np.float64) - low - q1)
    assert abs(out["err"] - eps) < 1e-5 * eps
    # it is a different starting point, not a relabelling of Algorithm 2: the spectra of W and W - Quantize(W) differ
    plain = oracle.lq(w, r, cfg, 1)
    assert not np.allclose(plain["sigma"], out["sigma"], rtol=1e-3)
    # half-step optimality (Eckart-Young): the low-rank correction of the quantization residual cannot increase it
    assert np.linalg.norm(w.astype(np.float64) - q0 - low) <= np.linalg.norm(w.astype(np.float64) - q0)


def test_lq_weighted_first_iteration_and_error(oracle):
    w = gen.weight_matrix(48, 96, 32, 8)
    rw = gen.positive_weights(48, 1); cw = gen.positive_weights(96, 2)
    cfg = oracle.config(4, 32, 16)
    out = oracle.lq(w, 4, cfg, 3, row_w=rw, col_w=cw)
    eps, _ = independent_first_step(oracle, w, 4, cfg, rw, cw)
    assert abs(out["trace"][0] - eps) < 1e-6 * eps
    resid = w.astype(np.float64) - out["Q"] - out["L1"].astype(np.float64) @ out["L2"].astype(np.float64)
    werr = np.sqrt(np.sum(np.outer(rw.astype(np.float64), cw.astype(np.float64)) * resid ** 2))   # Eq. 4
    assert abs(werr - out["err"]) < 1e-9 * werr
    # uniform weights: identical to the unweighted run
    a = oracle.lq(w, 4, cfg, 2)
    b = oracle.lq(w, 4, cfg, 2, row_w=np.ones(48, np.float32), col_w=np.ones(96, np.float32))
    assert np.array_equal(a["codes"], b["codes"]) and a["err"] == b["err"]


def test_lq_invariants(oracle):
    w = gen.weight_matrix(96, 160, 33, 12)
    w64 = w.astype(np.float64)
    cfg = oracle.config(3, 32, 16)
    r = 8
    outs = [oracle.lq(w, r, cfg, t) for t in (1, 2, 3, 4)]
    # running fewer iterations is a prefix of running more
    for t, o in enumerate(outs):
        assert np.allclose(o["trace"][:t + 1], outs[-1]["trace"][:t + 1], rtol=0, atol=0)
    # half-step monotonicity: the SVD step cannot increase the error for the previous Q
    for t in range(1, 4):
        prev, cur = outs[t - 1], outs[t]
        half = np.linalg.norm(w64 - prev["Q"] - cur["L1"].astype(np.float64) @ cur["L2"].astype(np.float64))
        assert half <= prev["err"] * (1 + 1e-6)
    # the sigma returned are those of W - Q_prev
    sv = np.linalg.svd(w64 - outs[2]["Q"], compute_uv=False)
    assert np.allclose(outs[3]["sigma"], sv[:r], rtol=1e-10)
    # LQ beats plain NF quantization of W (Section 3.1, preliminary experiments) ...
    c, si, v, _ = oracle.quantize(w.ravel(), cfg)
    plain = np.linalg.norm(w64.ravel() - oracle.dequantize(c, si, v, cfg))
    assert outs[-1]["err"] < plain
    # ... and the error falls with the rank (Table 5)
    e4 = oracle.lq(w, 4, cfg, 3)["err"]; e16 = oracle.lq(w, 16, cfg, 3)["err"]
    assert e16 < outs[2]["err"] < e4
    # more bits, smaller error
    assert oracle.lq(w, r, oracle.config(8, 32, 16), 2)["err"] < 0.1 * oracle.lq(w, r, oracle.config(2, 32, 16), 2)["err"]


def test_lq_early_stop_semantics(oracle):
    """eps_0 = inf, so one iteration always runs; the loop stops at the first increase and returns
    that (worse) iterate, as Algorithm 2 prints it."""
    found = False
    for seed in range(40, 60):
        w = gen.weight_matrix(32, 64, seed, 2)
        cfg = oracle.config(2, 16, 16)
        free = oracle.lq(w, 2, cfg, 12, early_stop=False)
        stop = oracle.lq(w, 2, cfg, 12, early_stop=True)
        tr = free["trace"]
        inc = np.nonzero(np.diff(tr) > 0)[0]
        want = 12 if inc.size == 0 else inc[0] + 2
        assert stop["iters_done"] == want and stop["iters_done"] >= 1
        assert np.array_equal(stop["trace"][:want], tr[:want])
        assert stop["err"] == tr[want - 1]
        if inc.size:
            found = True
            assert np.all(np.isnan(stop["trace"][want:]))
    assert found, "no seed exercised the stopping rule"


def test_lq_keep_best_iterate(oracle):
    """early_stop == 2 (a variant of Algorithm 2's ending): same stopping rule, but the iterate before the increase is
    returned.  Its pieces must be exactly those of a run limited to that many iterations, and its error the smallest
    of the trace."""
    found = False
    for seed in range(40, 60):
        w = gen.weight_matrix(32, 64, seed, 2)
        cfg = oracle.config(2, 16, 16)
        stop = oracle.lq(w, 2, cfg, 12, early_stop=True)
        best = oracle.lq(w, 2, cfg, 12, early_stop=2)
        assert best["iters_done"] == stop["iters_done"]
        assert np.array_equal(best["trace"], stop["trace"], equal_nan=True)
        n = stop["iters_done"]
        stopped_by_rule = n >= 2 and stop["trace"][n - 1] > stop["trace"][n - 2]
        keep = n - 1 if stopped_by_rule else n
        ref = oracle.lq(w, 2, cfg, keep)
        for key in ("L1", "L2", "codes", "scale_idx", "v", "Q", "sigma"):
            assert np.array_equal(best[key], ref[key]), key
        assert best["err"] == ref["err"] == np.nanmin(best["trace"][:n])
        found |= stopped_by_rule
    assert found, "no seed exercised the stopping rule"


def test_error_table(oracle):
    w = gen.weight_matrix(48, 64, 35, 4)
    cfgs = [oracle.config(b, b0, 16) for b in (2, 4) for b0 in (16, 32)]
    e, s = oracle.error_table(w, 4, cfgs, 2)
    for i, c in enumerate(cfgs):
        assert e[i] == oracle.lq(w, 4, c, 2)["err"] ** 2           # E[i,c] = eps^2  (Algorithm 3)
        assert s[i] == w.size * (c.bits + 8 / c.block + 32 / (c.block * 16))
    assert e[2] < e[0] and e[0] < e[1]                              # more bits / smaller blocks help


def test_workload1_shape_and_statistics():
    w = gen.workload_matrix(1, 0)
    assert w.shape == (768, 768) and w.dtype == np.float32
    assert abs(w.std() - 0.02 * np.sqrt(5 / 3)) < 2e-3              # Student-t(5) std = sqrt(5/3)
    assert np.array_equal(w, gen.workload_matrix(1, 0))
