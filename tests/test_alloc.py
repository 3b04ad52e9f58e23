"""Tag -> bitwidth allocation (Sec. 3.1.3, Eq. 3-4, Alg. 1): pins of the oracle, then the library against it."""
import ctypes as C
import os

import numpy as np
import pytest

from oracle import tkv_alloc_oracle as A
from paper_2605_17170_amd import tkv

GOLD = os.path.join(os.path.dirname(__file__), "golden", "alloc_worked.txt")


def _gold():
    d = {}
    for line in open(GOLD):
        if line.startswith("#") or "=" not in line:
            continue
        k, v = line.split("=")
        d[k.strip()] = [float(x) for x in v.split()]
    return d


def _knapsack_best_gain(N, D2, D4, limit):
    """Textbook 0/1 knapsack (dynamic programme over integer weights): the largest total gain of a set of
    upgrades whose cost 2 N_k fits in the budget.  Independent of the oracle's enumeration."""
    cap = int(np.floor(limit)) - 2 * sum(N)
    if cap < 0:
        return None
    best = [0.0] * (cap + 1)
    for k in range(len(N)):
        w, g = 2 * N[k], D2[k] - D4[k]
        if w == 0:
            if g > 0:
                best = [b + g for b in best]
            continue
        for c in range(cap, w - 1, -1):
            best[c] = max(best[c], best[c - w] + g)
    return best[cap]


# ------------------------------------------------------------------ oracle pins
def test_oracle_worked_example():
    g = _gold()
    N = [int(x) for x in g["N"]]
    assert A.allocate_greedy(N, g["D2"], g["D4"], g["B"][0]) == [int(x) for x in g["greedy"]]
    ex = A.allocate_exhaustive(N, g["D2"], g["D4"], g["B"][0])
    assert ex == [int(x) for x in g["exhaustive"]]
    assert abs(A.total_distortion(ex, g["D2"], g["D4"]) - g["distortion"][0]) < 1e-12
    N2 = [int(x) for x in g["N2"]]
    assert A.allocate_greedy(N2, g["D2_2"], g["D4_2"], g["B2"][0]) == [int(x) for x in g["greedy2"]]
    assert A.allocate_exhaustive(N2, g["D2_2"], g["D4_2"], g["B2"][0]) == [int(x) for x in g["exhaustive2"]]


def _random_instance(rng, n):
    N = [int(x) for x in rng.integers(0, 60, n)]
    if sum(N) == 0:
        N[0] = 5
    D4 = [float(x) for x in rng.uniform(0.0, 1.0, n)]
    D2 = [d + float(g) for d, g in zip(D4, rng.uniform(-0.2, 3.0, n))]
    B = float(rng.uniform(2.0, 4.0))
    return N, D2, D4, B


def test_oracle_exhaustive_equals_knapsack_optimum():
    rng = np.random.default_rng(70)
    for _ in range(150):
        n = int(rng.integers(1, 11))
        N, D2, D4, B = _random_instance(rng, n)
        bits = A.allocate_exhaustive(N, D2, D4, B)
        used = sum(n_ * b for n_, b in zip(N, bits))
        assert used <= A.budget_limit(N, B)
        gain = sum(D2[k] - D4[k] for k in range(n) if bits[k] == 4)
        assert abs(gain - _knapsack_best_gain(N, D2, D4, A.budget_limit(N, B))) < 1e-9


def test_oracle_greedy_invariants():
    rng = np.random.default_rng(71)
    for _ in range(200):
        n = int(rng.integers(1, 30))
        N, D2, D4, B = _random_instance(rng, n)
        bits = A.allocate_greedy(N, D2, D4, B)
        assert set(bits) <= {2, 4}
        assert sum(n_ * b for n_, b in zip(N, bits)) <= A.budget_limit(N, B)
        # the tag with the largest per-bit gain is upgraded whenever it fits on its own
        rho = [A._rho(N, D2, D4, k) for k in range(n)]
        top = max(range(n), key=lambda k: (rho[k], -k))
        if 2 * sum(N) + 2 * N[top] <= A.budget_limit(N, B):
            assert bits[top] == 4
        assert A.allocate_greedy(N, D2, D4, 2.0) == [4 if N[k] == 0 else 2 for k in range(n)]
        assert A.allocate_greedy(N, D2, D4, 4.0) == [4] * n


def test_oracle_greedy_is_optimal_for_equal_counts_and_positive_gains():
    rng = np.random.default_rng(72)
    for _ in range(100):
        n = int(rng.integers(2, 12))
        N = [7] * n
        D4 = [float(x) for x in rng.uniform(0, 1, n)]
        D2 = [d + float(g) for d, g in zip(D4, rng.uniform(0.01, 3, n))]
        B = float(rng.uniform(2.0, 4.0))
        g = A.allocate_greedy(N, D2, D4, B)
        e = A.allocate_exhaustive(N, D2, D4, B)
        assert abs(A.total_distortion(g, D2, D4) - A.total_distortion(e, D2, D4)) < 1e-12
# ------------------------------------------------------------------ library against the oracle
def _lib_alloc(fn, N, D2, D4, B):
    n = len(N)
    Na = (C.c_int64 * n)(*N)
    a2 = (C.c_double * n)(*D2)
    a4 = (C.c_double * n)(*D4)
    out = (C.c_uint8 * n)()
    rc = fn(n, Na, a2, a4, C.c_double(B), out)
    return rc, list(out)


def test_library_matches_oracle():
    L = tkv.lib()
    rng = np.random.default_rng(73)
    for i in range(300):
        n = int(rng.integers(1, 13))
        N, D2, D4, B = _random_instance(rng, n)
        if i % 7 == 0:                      # ties in rho and in the optimum
            D2 = [round(x, 1) for x in D2]
            D4 = [round(x, 1) for x in D4]
            N = [max(1, x // 10 * 10) for x in N]
        rc, bits = _lib_alloc(L.tkv_allocate_bits_greedy, N, D2, D4, B)
        assert rc == tkv.TKV_OK and bits == A.allocate_greedy(N, D2, D4, B)
        rc, bits = _lib_alloc(L.tkv_allocate_bits_exhaustive, N, D2, D4, B)
        assert rc == tkv.TKV_OK and bits == A.allocate_exhaustive(N, D2, D4, B)
    g = _gold()
    N = [int(x) for x in g["N"]]
    assert _lib_alloc(L.tkv_allocate_bits_greedy, N, g["D2"], g["D4"], g["B"][0])[1] == [int(x) for x in g["greedy"]]
    N2 = [int(x) for x in g["N2"]]
    assert _lib_alloc(L.tkv_allocate_bits_exhaustive, N2, g["D2_2"], g["D4_2"], g["B2"][0])[1] == [int(x) for x in g["exhaustive2"]]


def test_library_large_greedy_and_errors():
    L = tkv.lib()
    rng = np.random.default_rng(74)
    N, D2, D4, B = _random_instance(rng, 56)            # the paper's 56-tag space
    rc, bits = _lib_alloc(L.tkv_allocate_bits_greedy, N, D2, D4, B)
    assert rc == tkv.TKV_OK and bits == A.allocate_greedy(N, D2, D4, B)
    assert _lib_alloc(L.tkv_allocate_bits_exhaustive, N, D2, D4, B)[0] == tkv.TKV_ERR_INVALID_ARG   # > 22 tags
    assert _lib_alloc(L.tkv_allocate_bits_greedy, [1, 2], [1.0, 1.0], [0.5, 0.5], 1.5)[0] == tkv.TKV_ERR_INVALID_ARG
    assert _lib_alloc(L.tkv_allocate_bits_greedy, [1, -2], [1.0, 1.0], [0.5, 0.5], 3.0)[0] == tkv.TKV_ERR_INVALID_ARG
    assert _lib_alloc(L.tkv_allocate_bits_greedy, [1, 2], [1.0, float("nan")], [0.5, 0.5], 3.0)[0] == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_allocate_bits_greedy(0, None, None, None, C.c_double(3.0), None) == tkv.TKV_OK
