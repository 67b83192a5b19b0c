"""Pins for the oracle's single pass of Algorithm 2 (oq_lq_step) and for the LAPACK-backed stand-in that the full-size
GPU tests use in its place (tests/anchor.py)."""
import numpy as np
import pytest

import anchor
from paper_2311_12023_amd import gen


@pytest.mark.parametrize("weighted", [False, True])
def test_chained_steps_reproduce_the_loop(oracle, weighted):
    """Algorithm 2 is its loop body applied T times from Q(0) = 0: chaining oq_lq_step gives the loop's trace, codes and
    factors bit for bit."""
    d, k, r = 96, 160, 4
    w = gen.weight_matrix(d, k, 515, 6, outlier_frac=0.01)
    rw = cw = None
    if weighted:
        rw, cw = gen.positive_weights(d, 1), gen.positive_weights(k, 2)
    cfg = oracle.config(3, 16, 16)
    ref = oracle.lq(w, r, cfg, 4, row_w=rw, col_w=cw)
    q = np.zeros_like(w)
    for t in range(4):
        st = oracle.lq_step(w, q, r, cfg, rw, cw)
        assert st["err"] == ref["trace"][t]
        q = st["Q"]
    for key in ("L1", "L2", "codes", "scale_idx", "v", "Q", "sigma"):
        assert np.array_equal(st[key], ref[key]), key


def test_step_from_quantized_start(oracle):
    """Q(0) = Quantize(W) (Section 3.1, footnote): the first pass of that variant is a step from Dequantize(Quantize(W))."""
    w = gen.weight_matrix(64, 128, 99, 4)
    cfg = oracle.config(4, 32, 16)
    c0, s0, v0, _ = oracle.quantize(w.ravel(), cfg)
    q0 = oracle.dequantize(c0, s0, v0, cfg).reshape(w.shape)
    ref = oracle.lq(w, 3, cfg, 1, init_quantized=True)
    st = oracle.lq_step(w, q0, 3, cfg)
    assert st["err"] == ref["err"] and np.array_equal(st["codes"], ref["codes"])


def test_step_pieces_are_consistent(oracle):
    """The step's outputs against their definitions, written out with numpy: Q is the dequantized codes, the codes are
    Quantize(fl32(W - L1 L2)), eps is the Frobenius norm of W - L1 L2 - Q, sigma are the singular values of W - Q(t-1)."""
    w = gen.weight_matrix(80, 96, 7, 5)
    qprev = (gen.weight_matrix(80, 96, 8, 0) * 0.5).astype(np.float32)
    cfg = oracle.config(2, 16, 16)
    st = oracle.lq_step(w, qprev, 5, cfg)
    assert np.allclose(st["sigma"], np.linalg.svd((w - qprev).astype(np.float64), compute_uv=False)[:5], rtol=1e-10)
    t = w.astype(np.float64) - st["L1"].astype(np.float64) @ st["L2"].astype(np.float64)
    codes, sidx, v, _ = oracle.quantize(t.astype(np.float32).ravel(), cfg)
    assert np.array_equal(codes, st["codes"]) and np.array_equal(sidx, st["scale_idx"]) and np.array_equal(v, st["v"])
    assert np.array_equal(oracle.dequantize(codes, sidx, v, cfg).reshape(w.shape), st["Q"])
    assert abs(np.sqrt(np.sum((t - st["Q"]) ** 2)) - st["err"]) < 1e-12 * st["err"]


@pytest.mark.parametrize("weighted,bits", [(False, 2), (False, 8), (True, 3)])
def test_lapack_step_matches_oracle_step(oracle, weighted, bits):
    """The stand-in used at sizes the Jacobi SVD cannot reach agrees with the oracle's own step where both run: the
    same eps and singular values to 1e-9 (the two SVD routines differ in the last bits of the factors, which flips a few
    codes at rounding boundaries and nothing else)."""
    d, k, r = 128, 192, 6
    w = gen.weight_matrix(d, k, 2718, 8, outlier_frac=0.01)
    rw = cw = None
    if weighted:
        rw, cw = gen.positive_weights(d, 3), gen.positive_weights(k, 4)
    cfg = oracle.config(bits, 32, 16)
    q = np.zeros_like(w)
    for _ in range(3):
        a = oracle.lq_step(w, q, r, cfg, rw, cw)
        b = anchor.lapack_step(oracle, w, q, r, cfg, rw, cw)
        assert abs(a["err"] - b["err"]) < 1e-6 * a["err"]
        assert np.max(np.abs(a["sigma"] - b["sigma"]) / a["sigma"]) < 1e-9
        assert np.mean(a["Q"] != b["Q"]) < 1e-3
        q = a["Q"]


def test_top_svd_gram_route_matches_full_svd():
    """Large matrices take the top singular triplets from the Gram matrix of the shorter side; same values and same
    rank-r product as the full SVD."""
    rng = np.random.default_rng(3)
    for shape in ((1600, 1700), (1700, 1600)):
        a = rng.standard_normal(shape) + 3.0 * np.outer(rng.standard_normal(shape[0]), rng.standard_normal(shape[1])) / 40
        u, s, vt = anchor.top_svd(a, 12)
        uf, sf, vtf = np.linalg.svd(a, full_matrices=False)
        assert np.max(np.abs(s - sf[:12]) / sf[:12]) < 1e-10
        assert np.max(np.abs((u * s) @ vt - (uf[:, :12] * sf[:12]) @ vtf[:12])) < 1e-8 * sf[0]
