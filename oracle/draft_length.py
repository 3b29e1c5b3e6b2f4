"""Oracle for the draft-length heuristic (Algorithm 1).  TEST INFRASTRUCTURE ONLY.

State is (l_draft, s).  After each speculative step, with x_1..x_b the numbers of
accepted draft tokens of the sequences in the batch:
  * if the largest x equals the current draft length (some sequence accepted every
    draft), grow by l_incre up to l_limit and clear s;
  * otherwise shrink by ceil(l_draft / l_mod) + s, but never below 1 nor below the
    largest x, and set s = 1 (so a consecutive shrink is one larger).
Constants of the paper: l0 = 7, l_incre = 2, l_mod = 10, l_limit = 32.
"""
from __future__ import annotations

L0, L_INCRE, L_MOD, L_LIMIT = 7, 2, 10, 32


def initial_state(l0: int = L0):
    return (l0, 0)


def next_draft_len(state, accepted, l_incre=L_INCRE, l_mod=L_MOD, l_limit=L_LIMIT):
    """One update of Algorithm 1: (l_draft, s), accepted counts -> new (l_draft, s)."""
    l_draft, s = state
    xs = [int(x) for x in accepted]
    if max(xs) == l_draft:
        return (min(l_draft + l_incre, l_limit), 0)
    ceil_div = -(-l_draft // l_mod)
    shrunk = l_draft - ceil_div - s
    return (max([1, shrunk] + xs), 1)
