"""One-step anchoring of the LQ iteration (Algorithm 2) for the parity tests.

The iteration amplifies rounding-level differences from one pass to the next, so a whole trajectory of the GPU path and
of the oracle drift apart in individual codes.  A single pass does not: given the very same Q(t-1), Factorize and
Quantize of pass t agree to rounding.  The tests therefore take the GPU's own Q(t-1) (the path is deterministic, so
a run of t-1 iterations is the prefix of a run of t), let the CPU side do pass t from it, and compare eps_t and the
singular values of pass t at the tolerances of the benchmark spec (1e-3 and 1e-4 relative).

CPU side of a pass: the oracle's oq_lq_step (exact SVD by Jacobi) at small sizes; at sizes where Jacobi would take
hours, `lapack_step`, which takes the rank-r SVD from LAPACK and every other operation from the oracle (the CPU tests pin
it to oq_lq_step at small sizes).
"""
import numpy as np

SV_TOL = 1e-4
ERR_TOL = 1e-3


def top_svd(a, r):
    """Exact top-r singular triplets of the float64 matrix a: LAPACK's SVD, or (large matrices) LAPACK's symmetric
    eigen-solver on the Gram matrix of the shorter side, which gives the same subspace and values to ~1e-12 here."""
    d, k = a.shape
    if min(d, k) <= 1536:
        u, s, vt = np.linalg.svd(a, full_matrices=False)
        return u[:, :r], s[:r], vt[:r]
    import scipy.linalg as sl
    if d <= k:
        lam, u = sl.eigh(a @ a.T, subset_by_index=[d - r, d - 1])
        u, lam = u[:, ::-1], lam[::-1]
        s = np.sqrt(lam)
        return u, s, (u.T @ a) / s[:, None]
    lam, v = sl.eigh(a.T @ a, subset_by_index=[k - r, k - 1])
    v, lam = v[:, ::-1], lam[::-1]
    s = np.sqrt(lam)
    return (a @ v) / s[None, :], s, v.T


def lapack_step(oracle, w, q_prev, r, ocfg, row_w=None, col_w=None):
    """The loop body of Algorithm 2 from a given Q(t-1), with LAPACK's SVD standing in for the oracle's Jacobi and the
    oracle's quantizer / dequantizer on the full matrix.  Mirrors oq_lq_step operation by operation:
    Factorize(W - Q) (Algorithm 4; weighted: Eq. 5) with factors rounded to fp32, T = fl32(W - L1 L2) with the product in
    double, Quantize, Dequantize, eps = sqrt(sum w (W - L1 L2 - Q)^2) in double.  -> dict(err, sigma, Q, L1, L2)."""
    w64 = w.astype(np.float64)
    a = (w - q_prev).astype(np.float64)           # fp32 difference first, as the oracle forms A = W - Q in fp32
    if row_w is not None:
        dr, dc = np.sqrt(row_w.astype(np.float64)), np.sqrt(col_w.astype(np.float64))
        a = dr[:, None] * a * dc[None, :]
    u, s, vt = top_svd(a, r)
    l1 = u * np.sqrt(s)[None, :]
    l2 = np.sqrt(s)[:, None] * vt
    if row_w is not None:
        l1 = l1 / dr[:, None]
        l2 = l2 / dc[None, :]
    l1, l2 = l1.astype(np.float32), l2.astype(np.float32)
    t64 = w64 - l1.astype(np.float64) @ l2.astype(np.float64)
    codes, sidx, v, _ = oracle.quantize(t64.astype(np.float32).ravel(), ocfg)
    q = oracle.dequantize(codes, sidx, v, ocfg).reshape(w.shape)
    diff = t64 - q
    wt = 1.0 if row_w is None else np.outer(row_w.astype(np.float64), col_w.astype(np.float64))
    return dict(err=float(np.sqrt(np.sum(wt * diff * diff))), sigma=s, Q=q, L1=l1, L2=l2)


def cpu_step(oracle, w, q_prev, r, ocfg, row_w=None, col_w=None, exact="auto"):
    """Pass t on the CPU from Q(t-1): the oracle itself where its Jacobi SVD is affordable, lapack_step beyond."""
    if exact == "oracle" or (exact == "auto" and min(w.shape) <= 512 and max(w.shape) <= 1024):
        return oracle.lq_step(w, q_prev, r, ocfg, row_w, col_w)
    return lapack_step(oracle, w, q_prev, r, ocfg, row_w, col_w)


def check_anchored_decompose(oracle, lq, torch, w, rank, cfg_tuple, iters, seed, row_w=None, col_w=None, params=None,
                             which=None, label=""):
    """Every pass t in `which` (default: all of 1..iters) of lq_decompose against the CPU's pass t from the GPU's own
    Q(t-1).  Returns the run of `iters` iterations (dense Q included)."""
    wt = torch.from_numpy(w).cuda()
    grw = None if row_w is None else torch.from_numpy(row_w).cuda()
    gcw = None if col_w is None else torch.from_numpy(col_w).cuda()
    ocfg = oracle.config(*cfg_tuple)
    init_q = params is not None and params.init_quantized
    which = list(range(1, iters + 1)) if which is None else sorted(which)
    runs = {}
    for t in sorted(set(which) | {x - 1 for x in which if x > 1} | {iters}):
        runs[t] = lq.decompose(wt, rank, lq.config(*cfg_tuple), t, row_w=grw, col_w=gcw, seed=seed, params=params,
                               want_dense=True)
    full = runs[iters]
    for t in which:
        cur = runs[t]
        assert np.array_equal(cur["trace"][:t], full["trace"][:t])       # a shorter run is a prefix of the longer one
        if t > 1:
            q_prev = runs[t - 1]["Q"].cpu().numpy()
        elif init_q:
            c0, s0, v0, _ = oracle.quantize(w.ravel(), ocfg)
            q_prev = oracle.dequantize(c0, s0, v0, ocfg).reshape(w.shape)
        else:
            q_prev = np.zeros_like(w)
        ref = cpu_step(oracle, w, q_prev, rank, ocfg, row_w, col_w)
        rel_e = abs(cur["trace"][t - 1] - ref["err"]) / ref["err"]
        rel_s = np.max(np.abs(cur["sigma"] - ref["sigma"]) / ref["sigma"])
        print(f"{label} pass {t}: eps gpu {cur['trace'][t - 1]:.9g} cpu {ref['err']:.9g} rel {rel_e:.2e}; sigma rel {rel_s:.2e}")
        assert rel_e < ERR_TOL, (label, t, cur["trace"][t - 1], ref["err"])
        assert rel_s < SV_TOL, (label, t, rel_s)
    return full


def check_anchored_cell(oracle, w, rank, cfg_tuple, q_prev, eps_gpu, sigma_gpu, row_w=None, col_w=None, label=""):
    """A cell of the sweep: the CPU's pass from the captured Q(t-1) against the sweep's eps_t and sigma_t."""
    ref = cpu_step(oracle, w, q_prev, rank, oracle.config(*cfg_tuple), row_w, col_w)
    rel_e = abs(eps_gpu - ref["err"]) / ref["err"]
    rel_s = np.max(np.abs(sigma_gpu - ref["sigma"]) / ref["sigma"])
    print(f"{label} {cfg_tuple}: eps gpu {eps_gpu:.9g} cpu {ref['err']:.9g} rel {rel_e:.2e}; sigma rel {rel_s:.2e}")
    assert rel_e < ERR_TOL, (label, cfg_tuple, eps_gpu, ref["err"])
    assert rel_s < SV_TOL, (label, cfg_tuple, rel_s)
    return ref
