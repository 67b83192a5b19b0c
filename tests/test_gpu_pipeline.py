"""Algorithm 1 without the finetuning, end to end on the GPU path: error tables of several matrices (Algorithm 3),
the assignment under a bit budget (the integer program of Section 3.2), the final decomposition of every matrix with
its chosen configuration -- against the same pipeline run on the oracle (its error tables, brute force over all
assignments, its decomposition)."""
import numpy as np
import pytest

from paper_2311_12023_amd import gen
from test_gpu_decompose import ERR_TOL, ERR_TOL_CHAOTIC, check_decomposition_consistency

pytestmark = pytest.mark.gpu

SHAPES = [(96, 128), (128, 256), (64, 192)]
GRID = [(2, 16, 16), (2, 64, 16), (3, 16, 16), (3, 64, 16), (4, 16, 16), (4, 64, 16)]
RANK, ITERS = 4, 3


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    from paper_2311_12023_amd import lq
    return torch, lq


@pytest.mark.parametrize("bits_per_weight", [2.6, 3.3, 4.6])
def test_algorithm1_matches_oracle_pipeline(env, oracle, bits_per_weight):
    torch, lq = env
    # matrices of different difficulty: the later ones carry more heavy-tailed noise relative to their planted part
    ws = [gen.weight_matrix(d, k, 600 + i, 3, outlier_frac=0.01 * i) * (1.0 + i) for i, (d, k) in enumerate(SHAPES)]
    ocfgs = [oracle.config(*g) for g in GRID]
    oerr = np.zeros((len(ws), len(GRID)))
    osto = np.zeros((len(ws), len(GRID)))
    for i, w in enumerate(ws):
        oerr[i], osto[i] = oracle.error_table(w, RANK, ocfgs, ITERS)
    budget = bits_per_weight * sum(w.size for w in ws)
    want_choice, want = oracle.assign_bruteforce(oerr, osto, budget)
    assert want_choice is not None

    choice, outs, err, sto = lq.lq_lora_decompose([torch.from_numpy(w).cuda() for w in ws], RANK,
                                                  [lq.config(*g) for g in GRID], bits_per_weight, ITERS, seed=5)
    assert np.array_equal(sto, osto)
    for i in range(len(ws)):
        for c, g in enumerate(GRID):
            tol = ERR_TOL_CHAOTIC if g[0] == 2 else ERR_TOL
            assert abs(np.sqrt(err[i, c]) - np.sqrt(oerr[i, c])) < tol * np.sqrt(oerr[i, c]), (i, g)
    # the assignment found on the GPU's table is feasible and, priced on the oracle's table, optimal up to the
    # tolerance of the errors it was computed from
    assert sum(osto[i, choice[i]] for i in range(len(ws))) <= budget
    priced = sum(oerr[i, choice[i]] for i in range(len(ws)))
    assert priced <= want * (1 + 2 * ERR_TOL_CHAOTIC) + 1e-12
    # final decompositions: consistent pieces, errors equal to the table's cells
    for i, (w, out) in enumerate(zip(ws, outs)):
        check_decomposition_consistency(oracle, w, out, ocfgs[choice[i]], RANK)
        cell = np.sqrt(err[i, choice[i]])
        assert abs(out["err"] - cell) < ERR_TOL_CHAOTIC * cell
