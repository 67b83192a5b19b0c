"""Seeded synthetic inputs for the LQ decomposition path.

This module only draws random numbers and shapes them into test inputs; it holds none of the
method's arithmetic (no codebook, no quantizer, no SVD, no Fisher reduction).  Both the CPU
oracle's tests and the GPU parity tests / benchmark take their inputs from here so that the two
sides always see bit-identical fp32 arrays.

The matrices stand in for the pretrained weights the paper decomposes (RoBERTa-Large and
LLaMA-2 linear layers, Section 4), which are not available offline: heavy-tailed noise with the
kurtosis of trained weights, a planted low-rank part with a decaying spectrum, and a few
outlier columns.  Everything is generated on the host in float64 with numpy's counter-based
Philox generator and rounded once to float32.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 231112023

#: (d, k) of the seven linear layers of one LLaMA-2-7B block: q, k, v, o, gate, up, down.
LLAMA2_7B_LAYER = [(4096, 4096)] * 4 + [(4096, 11008)] * 2 + [(11008, 4096)]
#: one LLaMA-2-70B block (GQA k/v): q, o, k, v, gate, up, down.
LLAMA2_70B_LAYER = [(8192, 8192)] * 2 + [(8192, 1024)] * 2 + [(8192, 28672)] * 2 + [(28672, 8192)]
#: one RoBERTa-Large block: q, k, v, o, intermediate, output.
ROBERTA_LARGE_LAYER = [(1024, 1024)] * 4 + [(1024, 4096), (4096, 1024)]


def matrix_seed(config: int, index: int) -> int:
    """Seed of matrix `index` of workload `config` (1-based workload numbering)."""
    return BASE_SEED + 1000 * config + index


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def student_t_noise(rng: np.random.Generator, shape, nu: float = 5.0, scale: float = 0.02) -> np.ndarray:
    """scale * Student-t(nu), float64."""
    return rng.standard_t(nu, size=shape) * scale


def planted_low_rank(rng: np.random.Generator, d: int, k: int, rank: int,
                     top: float = 1.0, decay: float = 0.8) -> np.ndarray:
    """U diag(top * decay^i) V^T with U, V orthonormalised Gaussian draws, float64."""
    u, _ = np.linalg.qr(rng.standard_normal((d, rank)))
    v, _ = np.linalg.qr(rng.standard_normal((k, rank)))
    sig = top * decay ** np.arange(rank)
    return (u * sig) @ v.T


def weight_matrix(d: int, k: int, seed: int, planted_rank: int,
                  outlier_frac: float = 0.0, outlier_gain: float = 20.0) -> np.ndarray:
    """One synthetic weight matrix, float32, C-contiguous, shape (d, k).

    noise = 0.02 * Student-t(5); `round(outlier_frac * k)` columns (seeded permutation) have their
    noise multiplied by `outlier_gain`; the planted low-rank part is added afterwards.
    """
    rng = _rng(seed)
    w = student_t_noise(rng, (d, k))
    n_out = int(round(outlier_frac * k))
    if n_out > 0:
        cols = rng.permutation(k)[:n_out]
        w[:, cols] *= outlier_gain
    if planted_rank > 0:
        w += planted_low_rank(rng, d, k, planted_rank)
    return np.ascontiguousarray(w.astype(np.float32))


def workload_matrix(config: int, index: int = 0) -> np.ndarray:
    """Matrix `index` of one of the five benchmark workloads.

    1: one 768x768, planted rank 16.           2: RoBERTa-Large block shapes, planted rank 32.
    3: LLaMA-2-7B block shapes, planted rank 64, 0.1% outlier columns.
    4: one 4096x11008 from workload 3's generator.   5: LLaMA-2-70B block shapes, as 3.
    """
    seed = matrix_seed(config, index)
    if config == 1:
        return weight_matrix(768, 768, seed, 16)
    if config == 2:
        d, k = ROBERTA_LARGE_LAYER[index % len(ROBERTA_LARGE_LAYER)]
        return weight_matrix(d, k, seed, 32)
    if config == 3:
        d, k = LLAMA2_7B_LAYER[index]
        return weight_matrix(d, k, seed, 64, outlier_frac=0.001)
    if config == 4:
        return weight_matrix(4096, 11008, seed, 64, outlier_frac=0.001)
    if config == 5:
        d, k = LLAMA2_70B_LAYER[index]
        return weight_matrix(d, k, seed, 64, outlier_frac=0.001)
    raise ValueError(f"unknown workload {config}")


def fisher_matrix(d: int, k: int, seed: int, samples: int = 128, structured: bool = True) -> np.ndarray:
    """Synthetic diagonal Fisher information, float64, shape (d, k), strictly positive.

    Stands in for the mean over `samples` calibration gradients of g^2 (Section 3.3).  With
    g_ij = a_i * b_j * z_ij, z ~ N(0,1), the mean of `samples` squares is
    a_i^2 * b_j^2 * chi2(samples)/samples, which is drawn directly.  `structured=False` gives the
    literal iid case a = b = 1, for which the weighted path is close to the unweighted one.
    """
    rng = _rng(seed)
    if structured:
        a = np.exp(0.5 * rng.standard_normal(d))
        b = np.exp(0.5 * rng.standard_normal(k))
    else:
        a = np.ones(d)
        b = np.ones(k)
    chi = rng.chisquare(samples, size=(d, k)) / samples
    return (a * a)[:, None] * (b * b)[None, :] * chi


def positive_weights(n: int, seed: int, spread: float = 0.5) -> np.ndarray:
    """Log-normal positive weight vector, float32 (row or column Fisher weights for small tests)."""
    return np.exp(spread * _rng(seed).standard_normal(n)).astype(np.float32)


def activations(m: int, d: int, seed: int) -> np.ndarray:
    """Stand-in for a batch of layer inputs: unit normals with a few large feature columns, float32 (m, d)."""
    rng = _rng(seed)
    x = rng.standard_normal((m, d))
    cols = rng.permutation(d)[:max(1, d // 256)]
    x[:, cols] *= 8.0
    return np.ascontiguousarray(x.astype(np.float32))


def low_rank_factors(d: int, k: int, rank: int, seed: int, scale: float = 0.05):
    """Seeded dense factors L1 (d, rank), L2 (rank, k), float32: stand-ins for the low-rank pair of a decomposition."""
    rng = _rng(seed)
    l1 = rng.standard_normal((d, rank)) * scale
    l2 = rng.standard_normal((rank, k)) * scale
    return np.ascontiguousarray(l1.astype(np.float32)), np.ascontiguousarray(l2.astype(np.float32))


def paper_config_grid():
    """The 243 configurations (b0, B0, B1, b1, b2) of the paper's search space (Section 3.2, Table 1):
    b0, b1 in {2, 3, 4}, b2 in {bf16, fp16, fp32}, B0 in {16, 32, 64}, B1 in {16, 64, 256}."""
    return [(b0, blk, sblk, b1, b2) for b0 in (2, 3, 4) for b1 in (2, 3, 4) for b2 in ("bf16", "fp16", "fp32")
            for blk in (16, 32, 64) for sblk in (16, 64, 256)]


def config_grid(bits=(2, 3, 4, 8), blocks=(16, 32, 64), scale_blocks=(16, 64, 256)):
    """(bits, B0, B1) triples in a fixed order; the default is the 36-config sweep."""
    return [(b, b0, b1) for b in bits for b0 in blocks for b1 in scale_blocks]
