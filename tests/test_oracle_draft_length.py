"""Pins for the draft-length heuristic oracle (Algorithm 1): hand traces worked from the
algorithm's text with the paper's constants, and the invariants the text states."""
import os

import numpy as np

from oracle import draft_length as dl


def test_constants_match_paper(golden_dir):
    gold = dict(line.split() for line in open(os.path.join(golden_dir, "draft_length_constants.txt"))
                if line.strip() and not line.startswith("#"))
    assert (dl.L0, dl.L_INCRE, dl.L_MOD, dl.L_LIMIT) == tuple(int(gold[k]) for k in ("l0", "l_incre", "l_mod", "l_limit"))
    assert dl.initial_state() == (7, 0)


def test_hand_traces():
    # some sequence accepted all 7 drafts: grow by 2, s cleared
    assert dl.next_draft_len((7, 0), [3, 7, 0]) == (9, 0)
    # nobody accepted everything: 7 - ceil(7/10) - 0 = 6, s becomes 1
    assert dl.next_draft_len((7, 0), [3, 2, 0]) == (6, 1)
    # consecutive decrease is one larger: 6 - ceil(6/10) - 1 = 4
    assert dl.next_draft_len((6, 1), [2, 1]) == (4, 1)
    # never below the largest accepted count: 6 - 1 - 1 = 4 but someone accepted 5
    assert dl.next_draft_len((6, 1), [5, 1]) == (5, 1)
    # larger lengths shrink faster: 25 - ceil(25/10) - 1 = 21
    assert dl.next_draft_len((25, 1), [0, 0]) == (21, 1)
    # floor at 1
    assert dl.next_draft_len((1, 1), [0]) == (1, 1)
    # cap at l_limit
    assert dl.next_draft_len((31, 0), [31]) == (32, 0)
    assert dl.next_draft_len((32, 0), [32, 1]) == (32, 0)


def test_invariants_random_walk():
    rng = np.random.default_rng(0)
    st = dl.initial_state()
    for _ in range(2000):
        l = st[0]
        x = rng.integers(0, l + 1, size=4)
        new = dl.next_draft_len(st, x)
        assert 1 <= new[0] <= dl.L_LIMIT
        if x.max() == l:
            assert new == (min(l + 2, 32), 0)
        else:
            assert new[1] == 1 and x.max() <= new[0] <= max(l, 1) and new[0] >= 1
        st = new
