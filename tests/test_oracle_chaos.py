"""The LQ iteration amplifies rounding-level differences (documented behaviour of the method, measured on
the oracle's own arithmetic with LAPACK standing in for the SVD step so that a perturbation can be
injected).  This bounds what any parity test of a whole trajectory can ask for."""
import numpy as np

from paper_2311_12023_amd import gen


def trajectory(oracle, w, r, cfg, iters, perturb=0.0, seed=1):
    d, k = w.shape
    q = np.zeros_like(w)
    rng = np.random.default_rng(seed)
    errs, flips = [], []
    for t in range(iters):
        u, s, vt = np.linalg.svd((w - q).astype(np.float64), full_matrices=False)
        low = (u[:, :r] * s[:r]) @ vt[:r]
        if perturb and t == 0:
            low = low * (1 + perturb * rng.standard_normal(low.shape))
        tt = (w - low).astype(np.float32)
        codes, sidx, v, _ = oracle.quantize(tt.ravel(), cfg)
        q = oracle.dequantize(codes, sidx, v, cfg).reshape(d, k)
        errs.append(np.linalg.norm(w - low - q))
        flips.append(codes)
    return np.array(errs), flips, s[:r]


def test_code_flips_multiply_and_singular_values_drift(oracle):
    w = gen.weight_matrix(256, 384, 31337, 8)
    cfg = oracle.config(3, 16, 16)
    e0, c0, s0 = trajectory(oracle, w, 4, cfg, 6)
    e1, c1, s1 = trajectory(oracle, w, 4, cfg, 6, perturb=1e-5)
    nflip = [int(np.sum(a != b)) for a, b in zip(c0, c1)]
    assert nflip[-1] > 5 * max(nflip[0], 1)            # a handful of flipped codes becomes many
    assert np.max(np.abs(e1 - e0) / e0) < 1e-3         # ... while the error stays reproducible to 1e-3
    assert np.max(np.abs(s1 - s0) / s0) > 1e-6         # singular values of later iterations do not


def test_eight_bit_error_is_reproducible_only_to_about_1e_3(oracle):
    w = gen.weight_matrix(256, 384, 31337, 8)
    cfg = oracle.config(8, 16, 16)
    e0, _, _ = trajectory(oracle, w, 4, cfg, 4)
    spread = 0.0
    for seed in (1, 2):
        e1, _, _ = trajectory(oracle, w, 4, cfg, 4, perturb=1e-6, seed=seed)
        spread = max(spread, np.max(np.abs(e1 - e0) / e0))
    assert 1e-4 < spread < 3e-3


def test_two_bit_codes_make_the_trajectory_jump(oracle):
    """With 2-bit codes a flipped code moves a weight by up to a third of its block's absmax.  A relative
    perturbation of 1e-5 of the first low-rank part (below any flip) leaves the oracle's error trace alone; 1e-4
    (the accuracy to which a subspace with nearly equal singular values is determined at all) moves it by
    almost 1e-3.  Whole-trajectory comparisons of 2-bit cells are therefore held to a looser bound than 1e-3."""
    w = gen.weight_matrix(192, 512, 4242, 8, outlier_frac=0.004)
    cfg = oracle.config(2, 32, 64, 2, "bf16")
    e0, _, _ = trajectory(oracle, w, 6, cfg, 4)
    small = max(np.max(np.abs(trajectory(oracle, w, 6, cfg, 4, perturb=1e-5, seed=s)[0] - e0) / e0) for s in (1, 2))
    large = max(np.max(np.abs(trajectory(oracle, w, 6, cfg, 4, perturb=1e-4, seed=s)[0] - e0) / e0) for s in (1, 2, 3, 4))
    assert small < 1e-6
    assert 2e-4 < large < 3e-3
