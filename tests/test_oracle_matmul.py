"""Pins of the oracle's forward product Y = X (Q + L1 L2) (Section 3.2 "Implementation", Appendix A) against
things other than itself: selections that must return stored entries, a hand-computed case, and numpy's matmul on
the dense special cases."""
import numpy as np

from paper_2311_12023_amd import gen


def _quantized(oracle, d, k, cfg, seed):
    w = gen.weight_matrix(d, k, seed, 4)
    codes, sidx, v, _ = oracle.quantize(w.ravel(), cfg)
    return codes, sidx, v, oracle.dequantize(codes, sidx, v, cfg).reshape(d, k)


def test_identity_input_returns_the_dequantized_matrix(oracle):
    d, k = 32, 48
    cfg = oracle.config(3, 16, 4)
    codes, sidx, v, q = _quantized(oracle, d, k, cfg, 5)
    y = oracle.matmul(np.eye(d, dtype=np.float32), codes, sidx, v, cfg, k)
    assert np.array_equal(y, q.astype(np.float64))


def test_one_hot_rows_pick_rows_not_columns(oracle):
    """A transposed operand or swapped index would return a column of W (or fail on the shape)."""
    d, k, r = 32, 64, 3
    cfg = oracle.config(4, 16, 2)
    codes, sidx, v, q = _quantized(oracle, d, k, cfg, 6)
    l1, l2 = gen.low_rank_factors(d, k, r, 7, scale=0.5)
    x = np.zeros((2, d), np.float32)
    x[0, 5] = 1.0
    x[1, 31] = -2.0
    y = oracle.matmul(x, codes, sidx, v, cfg, k, l1, l2)
    w = q.astype(np.float64) + l1.astype(np.float64) @ l2.astype(np.float64)
    assert np.allclose(y[0], w[5], rtol=0, atol=1e-14)
    assert np.allclose(y[1], -2.0 * w[31], rtol=0, atol=1e-14)


def test_hand_computed_case(oracle):
    """Every code is the top code (value 1), one block, scale index = levels: Q is the constant v.  With
    X = [1 2 ... d], L1 = e_0 (column), L2 = row of 3s:  Y_j = v * d(d+1)/2 + 1 * 3."""
    d, k = 32, 16
    cfg = oracle.config(2, 16, 1)
    codes = np.full(d * k, 3, np.uint8)
    sidx = np.full(d * k // 16, 127, np.uint8)
    v = np.full(d * k // 16, 0.5, np.float32)
    x = np.arange(1, d + 1, dtype=np.float32)[None, :]
    l1 = np.zeros((d, 1), np.float32)
    l1[0, 0] = 1.0
    l2 = np.full((1, k), 3.0, np.float32)
    y, ya = oracle.matmul(x, codes, sidx, v, cfg, k, l1, l2, want_abs=True)
    sigma = np.float32(0.5) / np.float32(127)
    const = float(np.float32(127) * sigma)                 # reconstructed block scale, fp32
    assert np.allclose(y, const * d * (d + 1) / 2 + 3.0, rtol=1e-15, atol=0)
    assert np.allclose(ya, y)                                # all terms positive


def test_dense_special_cases_match_numpy(oracle):
    d, k, r, m = 64, 80, 5, 9
    cfg = oracle.config(8, 16, 16)
    codes, sidx, v, q = _quantized(oracle, d, k, cfg, 8)
    x = gen.activations(m, d, 9)
    l1, l2 = gen.low_rank_factors(d, k, r, 10)
    x64, q64 = x.astype(np.float64), q.astype(np.float64)
    # no low-rank part
    assert np.allclose(oracle.matmul(x, codes, sidx, v, cfg, k), x64 @ q64, rtol=1e-13, atol=1e-13)
    # codes of value zero everywhere: only the low-rank part is left, and (X L1) L2 = X (L1 L2)
    zero_code = np.full(d * k, 127, np.uint8)
    assert oracle.codebook(8)[127] == 0.0
    y = oracle.matmul(x, zero_code, sidx, v, cfg, k, l1, l2)
    assert np.allclose(y, (x64 @ l1.astype(np.float64)) @ l2.astype(np.float64), rtol=1e-12, atol=1e-13)
    # both parts, and the magnitude bound
    y, ya = oracle.matmul(x, codes, sidx, v, cfg, k, l1, l2, want_abs=True)
    assert np.allclose(y, x64 @ (q64 + l1.astype(np.float64) @ l2.astype(np.float64)), rtol=1e-12, atol=1e-13)
    assert np.allclose(ya, np.abs(x64) @ (np.abs(q64) + np.abs(l1).astype(np.float64) @ np.abs(l2).astype(np.float64)),
                       rtol=1e-12)
    assert np.all(ya >= np.abs(y) - 1e-12)
