"""ILPSolve of Algorithm 3 (the integer program of Section 3.2) on the host: the library's branch and bound against
the definition (brute force over all assignments, on tiny instances), a hand-worked instance, and properties that hold
at the paper's size (224 matrices x 243 configurations).  No GPU is touched."""
import ctypes as C
import os

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2311_12023_amd", "liblq_hip.so")


@pytest.fixture(scope="module")
def solve():
    if not os.path.exists(LIB):
        from paper_2311_12023_amd import build
        build.build()
    L = C.CDLL(LIB)
    vp = C.c_void_p
    L.lq_assign_configs.argtypes = [vp, vp, C.c_int, C.c_int, C.c_double, C.c_int64, vp, vp, vp, vp]

    def run(err, sto, budget, node_limit=0):
        err = np.ascontiguousarray(err, np.float64)
        sto = np.ascontiguousarray(sto, np.float64)
        n, c = err.shape
        choice = np.full(n, -1, np.int32)
        te, ts, lb = C.c_double(0), C.c_double(0), C.c_double(0)
        rc = L.lq_assign_configs(err.ctypes.data, sto.ctypes.data, n, c, float(budget), node_limit, choice.ctypes.data,
                                 C.addressof(te), C.addressof(ts), C.addressof(lb))
        return rc, choice, te.value, ts.value, lb.value
    return run


def test_bruteforce_oracle_on_a_hand_instance(oracle):
    """Two matrices, three configurations, worked by hand: with budget 9 the pairs that fit are
    (0,0) 4+4, (0,1) 4+5 and (1,0) 5+4; their errors are 10+8, 10+3 and 6+8: the best is (0,1) with 13."""
    err = [[10.0, 6.0, 1.0], [8.0, 3.0, 2.0]]
    sto = [[4.0, 5.0, 9.0], [4.0, 5.0, 7.0]]
    assert oracle.assign_bruteforce(err, sto, 9.0) == ([0, 1], 13.0)
    assert oracle.assign_bruteforce(err, sto, 7.9) == (None, float("inf"))
    assert oracle.assign_bruteforce(err, sto, 100.0) == ([2, 2], 3.0)
    # budget 13: (1,2) uses 5+7 = 12 bits for 6+2 = 8; (2,0) uses 13 for 1+8 = 9; (1,1) 10 bits for 9; (0,2) 11 bits for 12
    assert oracle.assign_bruteforce(err, sto, 13.0) == ([1, 2], 8.0)


def test_hand_instance(solve):
    err = [[10.0, 6.0, 1.0], [8.0, 3.0, 2.0]]
    sto = [[4.0, 5.0, 9.0], [4.0, 5.0, 7.0]]
    rc, choice, te, ts, lb = solve(err, sto, 9.0)
    assert rc == 0 and list(choice) == [0, 1] and te == 13.0 and ts == 9.0 and lb == 13.0
    assert solve(err, sto, 7.9)[0] == -8                                  # nothing fits
    rc, choice, te, ts, _ = solve(err, sto, 100.0)
    assert list(choice) == [2, 2] and te == 3.0 and ts == 16.0


@pytest.mark.parametrize("seed", range(40))
def test_matches_bruteforce(solve, oracle, seed):
    rng = np.random.Generator(np.random.Philox(1000 + seed))
    n, c = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    sto = rng.integers(1, 30, size=(n, c)).astype(np.float64)
    # errors loosely decreasing in storage, with noise, ties and dominated cells
    err = np.round(100.0 / sto + rng.uniform(0, 3, size=(n, c)), 1)
    lo, hi = sto.min(axis=1).sum(), sto.max(axis=1).sum()
    for budget in (lo, lo + 0.37 * (hi - lo), hi, lo - 1):
        want_choice, want = oracle.assign_bruteforce(err, sto, budget)
        rc, choice, te, ts, lb = solve(err, sto, budget)
        if want_choice is None:
            assert rc == -8
            continue
        assert rc == 0 and ts <= budget
        assert abs(te - want) < 1e-9 and abs(lb - te) < 1e-9
        assert abs(sum(err[i, choice[i]] for i in range(n)) - te) < 1e-9
        assert abs(sum(sto[i, choice[i]] for i in range(n)) - ts) < 1e-9


def test_paper_sized_instance(solve, oracle):
    """224 matrices x 243 configurations with the storage of Eq. 3 and errors that fall with the bit width: the search
    completes, respects the budget, is no worse than any uniform assignment that fits, and meets its own bound."""
    from paper_2311_12023_amd import gen
    grid = gen.paper_config_grid()
    assert len(grid) == 243
    shapes = (gen.LLAMA2_7B_LAYER * 32)[:224]
    rng = np.random.Generator(np.random.Philox(77))
    sto = np.array([[oracle.storage_bits(d * k, oracle.config(b0, B0, B1, b1, b2)) for (b0, B0, B1, b1, b2) in grid]
                    for d, k in shapes])
    hard = np.exp(rng.normal(0, 0.5, size=len(shapes)))                    # some matrices are harder to quantize
    bits = sto / np.array([d * k for d, k in shapes])[:, None]
    err = hard[:, None] * np.array([d * k for d, k in shapes])[:, None] * 4.0 ** (-bits) * \
        np.exp(rng.normal(0, 0.05, size=sto.shape))
    total = sum(d * k for d, k in shapes)
    for target in (2.5, 2.75, 3.25):
        rc, choice, te, ts, lb = solve(err, sto, target * total)
        assert rc == 0 and ts <= target * total
        assert lb <= te * (1 + 1e-12) and te - lb <= 1e-6 * te             # proven optimal
        for c in range(243):                                               # uniform assignments
            if sto[:, c].sum() <= target * total:
                assert te <= err[:, c].sum() * (1 + 1e-12)
        assert len(set(choice.tolist())) > 1                               # the budget is spent unevenly
    # a node limit returns a feasible assignment and a valid bound
    rc, choice, te2, ts2, lb2 = solve(err, sto, 2.75 * total, node_limit=3)
    assert rc == 0 and ts2 <= 2.75 * total and lb2 <= te2


def test_validation(solve):
    e = np.ones((2, 2))
    assert solve(e, e, -1.0)[0] == -8
    assert solve(np.array([[np.nan, 1.0]]), np.ones((1, 2)), 10.0)[0] == -8
    assert solve(-e, e, 10.0)[0] == -8
