"""CPU oracle of the triaxial tagger and the tag -> bitwidth lookup (Sec. 3.1 "Tri-Axial Quantization" and
Sec. 3.2.3 "Tagging").

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE: plain, slow, pure Python, used only by the tests.  It shares
no code with the library.

A token's tag is a point of temporal x modal x semantic (4 x 2 x 7 = 56 tags):
  semantic  0 inst, 1 user, 2 assistant, 3 reasoning, 4 tool_call, 5 obs, 6 delim   (Table "Semantic axis")
  modal     0 text, 1 image
  temporal  0 older, 1 turn_m2, 2 turn_m1, 3 current: the distance, in turns, from the most recent turn;
            a turn runs from one user message up to, not including, the next.
The semantic role and the modality come from the chat template (here: given per token); the temporal value is
derived from the positions of the user messages.  Code = (temporal * 2 + modal) * 7 + semantic.

Readings where the paper is silent: a user message starts at a `user` token whose predecessor is not a `user`
token (template scaffolding in front of it belongs to the turn before); tokens in front of the first user
message (the system prompt) form turn 0 and age like any other turn; without any user message everything is
`current`.

Pins (tests/test_tagger.py): a hand-worked conversation (tests/golden/tagger_worked.txt), the suffix-count
definition of the distance by brute force, field round trips and monotonicity.
"""
from __future__ import annotations

N_SEMANTIC, N_MODAL, N_TEMPORAL = 7, 2, 4
USER = 1


def tag_tokens(semantic, modal):
    n = len(semantic)
    assert len(modal) == n
    turn = [0] * n
    cur = 0
    for t in range(n):
        if not (0 <= semantic[t] < N_SEMANTIC and 0 <= modal[t] < N_MODAL):
            raise ValueError("bad axis value at token %d" % t)
        if semantic[t] == USER and (t == 0 or semantic[t - 1] != USER):
            cur += 1                       # a user message begins: a new turn
        turn[t] = cur
    tags = []
    for t in range(n):
        back = cur - turn[t]               # 0 = the most recent turn
        temporal = 3 - back if back <= 2 else 0
        tags.append((temporal * N_MODAL + modal[t]) * N_SEMANTIC + semantic[t])
    return tags


def tags_to_bits(tags, table):
    assert len(table) == N_SEMANTIC * N_MODAL * N_TEMPORAL
    return [table[k] for k in tags]


def tag_counts(tags):
    counts = [0] * (N_SEMANTIC * N_MODAL * N_TEMPORAL)
    for k in tags:
        counts[k] += 1
    return counts
