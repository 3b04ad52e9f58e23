"""Triaxial tagger and tag -> bitwidth lookup (Sec. 3.1, Sec. 3.2.3 "Tagging"): pins of the oracle, then the
library against it."""
import ctypes as C
import os

import numpy as np
import pytest

from oracle import tkv_tagger_oracle as T
from paper_2605_17170_amd import tkv
from paper_2605_17170_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "tagger_worked.txt")


def _gold():
    sem, mod, temporal, codes = [], [], [], []
    for line in open(GOLD):
        if not line.startswith("seg "):
            continue
        left, right = line[4:].split("->")
        s, m, n = (int(x) for x in left.split())
        tp, code = (int(x) for x in right.split())
        sem += [s] * n; mod += [m] * n; temporal += [tp] * n; codes += [code] * n
    return sem, mod, temporal, codes


def _random_chat(rng, n_seg):
    sem, mod = [], []
    for _ in range(n_seg):
        s = int(rng.integers(0, 7))
        m = int(rng.integers(0, 2)) if s == 5 else 0
        n = int(rng.integers(1, 9))
        sem += [s] * n; mod += [m] * n
    return sem, mod


# ------------------------------------------------------------------ the oracle against its pins
def test_oracle_worked_conversation():
    sem, mod, temporal, codes = _gold()
    assert len(sem) == 51
    tags = T.tag_tokens(sem, mod)
    assert tags == codes
    assert [k // 14 for k in tags] == temporal


def test_oracle_distance_is_the_number_of_later_user_messages():
    """Brute force over the definition: temporal depends only on how many user messages START after the token."""
    rng = np.random.default_rng(51)
    for _ in range(100):
        sem, mod = _random_chat(rng, int(rng.integers(1, 30)))
        n = len(sem)
        starts = [t for t in range(n) if sem[t] == 1 and (t == 0 or sem[t - 1] != 1)]
        tags = T.tag_tokens(sem, mod)
        for t in range(n):
            later = sum(1 for s in starts if s > t)
            want_temporal = {0: 3, 1: 2, 2: 1}.get(later, 0)
            tp, md, se = (int(x) for x in wl.tag_fields(tags[t]))      # the input generator's own field split
            assert (tp, md, se) == (want_temporal, mod[t], sem[t])
        tps = [k // 14 for k in tags]
        assert tps == sorted(tps) and tps[-1] == 3                    # ageing is monotone, the end is current


def test_oracle_closed_cases():
    assert T.tag_tokens([], []) == []
    assert T.tag_tokens([0, 0, 2], [0, 0, 0]) == [42, 42, 44]          # no user message: everything current
    assert T.tag_tokens([1, 1, 1], [0, 0, 0]) == [43, 43, 43]          # one message of three tokens, not three
    assert [k // 14 for k in T.tag_tokens([1, 6, 1, 6, 1, 6, 1], [0] * 7)] == [0, 0, 1, 1, 2, 2, 3]
    with pytest.raises(ValueError):
        T.tag_tokens([7], [0])
    table = [2] * 56
    table[43] = 4
    assert T.tags_to_bits([43, 0, 43], table) == [4, 2, 4]
    assert sum(T.tag_counts([43, 0, 43])) == 3 and T.tag_counts([43, 0, 43])[43] == 2


# ------------------------------------------------------------------ the library against the oracle
def test_library_matches_oracle():
    rng = np.random.default_rng(52)
    sem, mod, _, codes = _gold()
    assert tkv.tkv_tag_tokens(sem, mod).tolist() == codes
    for _ in range(200):
        sem, mod = _random_chat(rng, int(rng.integers(0, 40)))
        tags = tkv.tkv_tag_tokens(sem, mod)
        want = T.tag_tokens(sem, mod)
        assert tags.tolist() == want
        table = rng.choice([2, 4], 56).astype(np.uint8)
        assert tkv.tkv_tags_to_bits(tags, table).tolist() == T.tags_to_bits(want, table.tolist())
        assert tkv.tkv_tag_counts(tags).tolist() == T.tag_counts(want)


def test_library_rejects_bad_input():
    L = tkv.lib()
    sem = np.uint8([0, 7])
    mod = np.uint8([0, 0])
    out = np.full(2, 99, np.uint8)
    p = lambda a: C.c_void_p(a.ctypes.data)
    assert L.tkv_tag_tokens(p(sem), p(mod), 2, p(out)) == tkv.TKV_ERR_INVALID_ARG and out.tolist() == [99, 99]
    assert L.tkv_tag_tokens(p(np.uint8([0, 1])), p(np.uint8([0, 2])), 2, p(out)) == tkv.TKV_ERR_INVALID_ARG
    assert L.tkv_tag_tokens(None, None, 0, None) == tkv.TKV_OK
    table = np.full(56, 2, np.uint8)
    assert L.tkv_tags_to_bits(p(np.uint8([56])), 1, p(table), p(out)) == tkv.TKV_ERR_INVALID_ARG
    table[3] = 3
    assert L.tkv_tags_to_bits(p(np.uint8([0])), 1, p(table), p(out)) == tkv.TKV_ERR_BAD_BITS
    counts = np.zeros(56, np.int64)
    assert L.tkv_tag_counts(p(np.uint8([56])), 1, p(counts)) == tkv.TKV_ERR_INVALID_ARG and not counts.any()


def test_calibration_to_serving_chain():
    """Tag a conversation, count tokens per tag, allocate bitwidths under a budget, look the per-token widths up
    and route the residual: the host side of a request from template structure to tkv_plan_append's input."""
    rng = np.random.default_rng(53)
    sem, mod = _random_chat(rng, 200)
    tags = tkv.tkv_tag_tokens(sem, mod)
    N = tkv.tkv_tag_counts(tags)
    D4 = rng.random(56) * 0.1
    D2 = D4 + rng.random(56)
    table = np.uint8(tkv.tkv_allocate_bits_greedy(N.tolist(), D2.tolist(), D4.tolist(), 2.8))
    bits = tkv.tkv_tags_to_bits(tags, table)
    assert int(bits.astype(np.int64).sum()) <= 2.8 * len(sem) * (1 + 1e-9)      # Eq. 3's budget
    routed = tkv.tkv_route_residual(bits)
    assert int((routed == 2).sum()) % 32 == 0
