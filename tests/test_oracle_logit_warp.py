"""Pins of the logits-front-end oracle (temperature + nucleus top-p + softmax) against closed
forms, library routines and an independently formulated nucleus filter."""
import numpy as np
import pytest
import torch
from scipy.special import softmax

from oracle.logit_warp import warp_probs, warp_row


def nucleus_by_removal(logits, T, top_p):
    """The same filter said the other way round, with torch's sort/cumsum: walk the tokens from the
    LEAST probable one up and drop a token while the mass of it and everything below it stays within
    the 1 - top_p that may be cut (the formulation common in sampling libraries)."""
    P = torch.softmax(torch.tensor(logits, dtype=torch.float64) / T, dim=-1)
    V = P.numel()
    # decreasing P, ties by increasing id == stable descending sort; reverse it for the ascending walk
    order = torch.sort(P, descending=True, stable=True).indices
    asc = torch.flip(order, dims=[0])
    tail = torch.cumsum(P[asc], 0)              # mass of a token and everything less probable
    total = tail[-1]
    drop = (total - tail) >= top_p              # what stays above it already reaches top_p
    drop[-1] = False
    keep = torch.zeros(V, dtype=torch.bool)
    keep[asc[~drop]] = True
    out = torch.where(keep, P, torch.zeros_like(P))
    return (out / out.sum()).numpy(), keep.numpy()


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("T,top_p", [(0.2, 0.95), (1.0, 0.9), (0.7, 0.5), (2.0, 0.999), (1.0, 0.05)])
def test_equals_the_removal_formulation(seed, T, top_p):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal(257) * 3).astype(np.float32)
    got, kept, _ = warp_row(logits, T, top_p)
    want, keep2 = nucleus_by_removal(logits, T, top_p)
    assert (kept == keep2).all()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)


def test_top_p_one_is_the_library_softmax():
    rng = np.random.default_rng(1)
    logits = rng.standard_normal((3, 5, 40)).astype(np.float32)
    np.testing.assert_allclose(warp_probs(logits, 0.5, 1.0), softmax(logits.astype(np.float64) / 0.5, axis=-1), rtol=1e-13)


def test_tiny_top_p_is_greedy():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((4, 33)).astype(np.float32)
    out = warp_probs(logits, 1.0, 1e-9)
    assert (out.argmax(-1) == logits.argmax(-1)).all()
    assert ((out == 0) | (out == 1)).all() and (out.sum(-1) == 1).all()


def test_uniform_logits_keep_the_lowest_ids():
    # ten equal tokens of 0.1: the cumulative sums in fp64 are 0.1, 0.2, 0.30000000000000004, 0.4 -> four
    # tokens reach 0.35, and equal probabilities are taken by increasing token id
    out = warp_probs(np.zeros(10, np.float32), 1.0, 0.35)
    np.testing.assert_allclose(out, [0.25] * 4 + [0.0] * 6)
    out = warp_probs(np.full(10, 7.0, np.float32), 0.3, 0.05)
    np.testing.assert_allclose(out, [1.0] + [0.0] * 9)


def test_two_level_distribution_closed_form():
    # logits ln 8, ln 4, ln 2, ln 1, ln 1 -> P = 8/16, 4/16, 2/16, 1/16, 1/16
    logits = np.log(np.array([2.0, 1.0, 8.0, 1.0, 4.0]))
    out = warp_probs(logits, 1.0, 0.8)                 # 0.5 + 0.25 = 0.75 < 0.8 <= 0.875
    np.testing.assert_allclose(out, np.array([2, 0, 8, 0, 4]) / 14.0, rtol=1e-13)
    out = warp_probs(logits, 1.0, 0.9)                 # needs one of the two 1/16 tokens: the lower id
    np.testing.assert_allclose(out, np.array([2, 1, 8, 0, 4]) / 15.0, rtol=1e-13)
    out = warp_probs(logits, 0.5, 0.8)                 # T = 0.5 squares the odds: 64, 16, 4, 1, 1 of 86
    np.testing.assert_allclose(out, np.array([0, 0, 64, 0, 16]) / 80.0, rtol=1e-13)


def test_temperature_is_a_division_of_the_logits_and_shifts_do_not_matter():
    rng = np.random.default_rng(3)
    logits = rng.standard_normal(100)
    a = warp_probs(logits, 0.25, 0.9)
    np.testing.assert_allclose(a, warp_probs(logits * 4.0, 1.0, 0.9), rtol=1e-12)
    np.testing.assert_allclose(a, warp_probs(logits + 123.0, 0.25, 0.9), rtol=1e-9)


@pytest.mark.parametrize("seed", range(4))
def test_nucleus_is_minimal_sufficient_and_a_top_set(seed):
    rng = np.random.default_rng(10 + seed)
    logits = rng.standard_normal(500) * 2
    for top_p in (0.1, 0.5, 0.9, 0.99):
        out, kept, P = warp_row(logits, 1.0, top_p)
        assert abs(out.sum() - 1) < 1e-12
        assert P[kept].sum() >= top_p                               # sufficient
        assert P[kept].sum() - P[kept].min() < top_p                # minimal: drop the smallest and it fails
        assert P[kept].min() >= P[~kept].max()                      # a set of most probable tokens
        np.testing.assert_allclose(out[kept] / out[kept].sum(), P[kept] / P[kept].sum(), rtol=1e-12)
    sizes = [warp_row(logits, 1.0, tp)[1].sum() for tp in (0.1, 0.3, 0.6, 0.9, 1.0)]
    assert sizes == sorted(sizes) and sizes[-1] == 500              # grows with top_p


def test_planted_mistakes_are_caught_by_the_pins():
    # a filter that drops the token that crosses top_p (a common off-by-one) fails the closed form
    logits = np.log(np.array([2.0, 1.0, 8.0, 1.0, 4.0]))
    P = softmax(logits)
    order = np.argsort(-P, kind="stable")
    csum = np.cumsum(P[order])
    wrong_keep = order[csum < 0.8]                                   # stops one token early
    wrong = np.zeros(5)
    wrong[wrong_keep] = P[wrong_keep]
    wrong /= wrong.sum()
    assert not np.allclose(wrong, warp_probs(logits, 1.0, 0.8))
