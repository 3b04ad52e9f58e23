"""CPU oracle of the tag -> bitwidth allocation (Sec. 3.1.3, Eq. 3-4, Alg. 1).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE: plain, slow, pure Python, used only by the tests.  It shares
no code with the library.

  allocate_exhaustive  the definition of Eq. 3 written out: every b in {2,4}^|S| that meets the budget
                       sum_k N_k b_k <= B sum_k N_k is visited and the one with the least sum_k D_k(b_k)
                       is returned (the paper uses this when |S| <= 22).
  allocate_greedy      Alg. 1 in the paper's order: per-bit gain rho_k = (D_k(2) - D_k(4)) / (2 N_k)
                       (Eq. 4), tags sorted by rho descending, remaining budget R = (B - 2) sum_k N_k, a tag
                       is upgraded to 4 bits whenever its extra cost 2 N_k fits in R.

Readings where the paper is silent: ties in rho keep tag order (stable sort); a tag without tokens (N_k = 0)
has rho = +inf / 0 / -inf by the sign of its gain; ties in the exhaustive minimum go to the allocation with
fewer total bits, then to the smaller bit mask (tag 0 = lowest bit, 1 = upgraded).  The budget is the
binary64 product T = B * sum_k N_k with a relative slack of 2^-40 (a decimal B such as 2.8 is not a binary64
number; without the slack an allocation that meets the budget exactly could be rejected); bits in use are
counted in exact integers, so "2 N_k fits in the remaining budget R" reads used + 2 N_k <= T (1 + 2^-40),
which is the paper's test R = (B - 2) sum N - (bits already spent) >= 2 N_k in exact arithmetic.

Pins (tests/test_alloc.py): a hand-worked example (tests/golden/alloc_worked.txt), the optimum against a
textbook 0/1-knapsack dynamic programme, budget feasibility, the closed cases B = 2 and B = 4, and the
equal-count case where the greedy walk is optimal.
"""
from __future__ import annotations

import itertools
import math


def _rho(N, D2, D4, k):
    gain = D2[k] - D4[k]
    if N[k] == 0:
        return math.inf if gain > 0 else (-math.inf if gain < 0 else 0.0)
    return gain / (2.0 * N[k])


def budget_limit(N, B):
    """Largest admissible number of cache bits: B * sum N with a relative slack of 2^-40."""
    t = B * float(sum(N))
    return t * (1.0 + 2.0 ** -40)


def allocate_greedy(N, D2, D4, B):
    n = len(N)
    rho = [_rho(N, D2, D4, k) for k in range(n)]
    order = sorted(range(n), key=lambda k: -rho[k])      # Python's sort is stable: ties keep tag order
    bits = [2] * n
    limit = budget_limit(N, B)
    used = 2 * sum(N)
    for k in order:
        if used + 2 * N[k] <= limit:
            bits[k] = 4
            used += 2 * N[k]
    return bits


def allocate_exhaustive(N, D2, D4, B):
    n = len(N)
    limit = budget_limit(N, B)
    best = None
    for mask in range(1 << n):
        bits = [4 if (mask >> k) & 1 else 2 for k in range(n)]
        if sum(N[k] * bits[k] for k in range(n)) > limit:
            continue
        cost = 0.0
        for k in range(n):
            cost = cost + (D4[k] if bits[k] == 4 else D2[k])
        key = (cost, sum(N[k] * bits[k] for k in range(n)), mask)
        if best is None or key < best[0]:
            best = (key, bits)
    return best[1]


def total_distortion(bits, D2, D4):
    cost = 0.0
    for k, b in enumerate(bits):
        cost = cost + (D4[k] if b == 4 else D2[k])
    return cost
