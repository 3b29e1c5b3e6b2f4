"""GPU parity of bass_warp_probs (temperature + nucleus top-p + softmax) against the fp64 oracle.

The kept set is an integer decision taken from floating-point masses: the library takes it on
fp32 values of 2^x (integer-rounded to 2^-40), the oracle in fp64.  Where the cumulative mass
passes top_p closer than the fp32 error, or two tokens near the cut differ by less than it, either
decision is right; the test then checks the properties that any right answer has (a set of most
probable tokens, sufficient, minimal, values normalised over it) instead of the oracle's particular one."""
import numpy as np
import pytest

import oracle.logit_warp as ow
import workloads as wl

pytestmark = pytest.mark.gpu

REL, ABS = 3e-5, 1e-9   # fp32 exp2 of arguments up to ~2^7 in magnitude: relative error ~ 2^-24 * 2^7 * ln 2
EDGE = 2e-5             # how close to top_p a cumulative mass may be for the decision to be open


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def check_rows(logits, T, top_p, got):
    logits = logits.reshape(-1, logits.shape[-1])
    got = got.reshape(logits.shape)
    open_rows = 0
    for r in range(logits.shape[0]):
        want, kept, P = ow.warp_row(logits[r], T, top_p)
        g = got[r].astype(np.float64)
        assert np.isfinite(g).all() and (g >= 0).all()
        assert abs(g.sum() - 1.0) < 1e-5
        gk = g > 0
        if (gk == kept).all():
            np.testing.assert_allclose(g, want, rtol=REL, atol=ABS)
            continue
        # decision differs: legitimate only at the edge of the nucleus, where fp32 values of 2^x may order
        # two nearly equal tokens the other way round or put the cumulative mass on the other side of top_p
        open_rows += 1
        sel = P * gk
        mass, p_least = sel.sum(), P[gk].min()
        if (~gk).any():
            assert P[~gk].max() <= p_least * (1 + 4 * REL)                   # still a set of most probable tokens
        assert mass >= top_p - EDGE                                          # that reaches top_p
        assert mass - p_least < top_p + EDGE                                 # and would not without its last token
        np.testing.assert_allclose(g, sel / mass, rtol=REL, atol=ABS)        # values right for the set chosen
    return open_rows


@pytest.mark.parametrize("T,top_p", [(0.2, 0.95), (1.0, 0.9), (0.7, 0.5), (1.0, 1.0), (2.0, 0.999), (1.0, 1e-6)])
def test_small_vocabularies(hip, T, top_p):
    rng = np.random.default_rng(3)
    for V in (1, 7, 64, 1000, 1025, 5000):
        logits = (rng.standard_normal((6, V)) * 3).astype(np.float32)
        got, status = hip.run_warp_probs(logits, T, top_p)
        assert status == 0
        # an open decision needs a cumulative mass within 2e-5 of top_p, or a near-tie at the cut: rare
        assert check_rows(logits, T, top_p, got) <= 1


@pytest.mark.parametrize("T,top_p", [(0.2, 0.95), (1.0, 0.9)])
def test_vocabularies_around_the_register_variants(hip, T, top_p):
    # rows of up to 32768 / 53248 / 65536 aligned logits are held in registers (8 / 13 / 16 groups of four per
    # thread); longer rows, and rows whose length is not a multiple of four, stream through the output row
    rng = np.random.default_rng(11)
    for V in (32764, 32768, 32772, 53248, 53252, 60000, 65536, 65540, 70001, 80000):
        logits = (rng.standard_normal((2, V)) * 2.5).astype(np.float32)
        got, status = hip.run_warp_probs(logits, T, top_p)
        assert status == 0
        assert check_rows(logits, T, top_p, got) <= 1


def test_full_step_shapes_and_determinism(hip):
    # the acceptance recipe's logits at the paper's sampling settings: 8 x 6 main rows, 8 x 5 draft rows of 50 000
    lt, ld = wl.make_logits(8, 5, 50000, 0, 3.0, 1.0)
    for logits in (lt, ld):
        got, status = hip.run_warp_probs(logits, 0.2, 0.95)
        assert status == 0
        assert check_rows(logits, 0.2, 0.95, got) <= 1
        again, _ = hip.run_warp_probs(logits, 0.2, 0.95)
        assert (got.view(np.uint32) == again.view(np.uint32)).all()      # integer masses: same bits every run
    # flat distribution at a high temperature: the nucleus holds most of the vocabulary
    got, _ = hip.run_warp_probs(lt[:2], 5.0, 0.9)
    assert check_rows(lt[:2], 5.0, 0.9, got) <= 1


def test_ties_are_taken_by_token_id(hip):
    # ten equal tokens, top_p 0.35: four are needed, the ones with the lowest ids
    got, _ = hip.run_warp_probs(np.zeros((1, 10), np.float32), 1.0, 0.35)
    np.testing.assert_allclose(got[0], [0.25] * 4 + [0.0] * 6, rtol=1e-6)
    # two levels with ties at the boundary, spread over many threads
    V = 4096
    logits = np.zeros((1, V), np.float32)
    logits[0, ::2] = np.log(3.0)                     # 2048 tokens of weight 3, 2048 of weight 1
    total = 3 * 2048 + 2048
    top_p = (3 * 2048 + 100.5) / total               # all heavy tokens and 101 light ones
    got, _ = hip.run_warp_probs(logits, 1.0, top_p)
    kept = got[0] > 0
    assert kept[::2].all()
    light = np.nonzero(kept[1::2])[0]
    assert len(light) == 101 and (light == np.arange(101)).all()
    assert abs(got[0].sum() - 1) < 1e-5


def test_degenerate_rows(hip):
    import paper_2404_15778_amd as bass
    logits = np.zeros((4, 300), np.float32)
    logits[0, :] = -np.inf                           # no finite logit: zeros + status
    logits[1, :] = -np.inf
    logits[1, 17] = 2.0                              # a single finite logit
    logits[2, 5] = np.nan                            # NaN gets probability 0
    logits[3, 9] = np.inf                            # +inf takes everything
    got, status = hip.run_warp_probs(logits, 1.0, 0.9)
    assert status & bass.STATUS_ZERO_MASS
    assert (got[0] == 0).all()
    assert got[1, 17] == 1.0 and got[1].sum() == 1.0
    assert got[2, 5] == 0 and abs(got[2].sum() - 1) < 1e-5
    assert got[3, 9] == 1.0 and got[3].sum() == 1.0


def test_warped_rows_feed_the_acceptance(hip):
    # p and q produced by the front end are valid inputs of bass_spec_accept: same result as the oracle's
    # acceptance on the same (library-made) rows
    import oracle
    lt, ld = wl.make_logits(4, 3, 2000, 5, 3.0, 1.0)
    p, _ = hip.run_warp_probs(lt, 0.2, 0.95)
    q, _ = hip.run_warp_probs(ld, 0.2, 0.95)
    rng = np.random.default_rng(9)
    tok = np.array([[int(rng.choice(2000, p=q[b, i].astype(np.float64) / q[b, i].astype(np.float64).sum()))
                     for i in range(3)] for b in range(4)], np.int32)
    a = wl.AcceptWorkload("warped", 4, 3, 2000, p, q, tok, np.full(4, 3, np.int32), rng.random((4, 4), dtype=np.float32))
    n_acc, nxt, status = hip.run_accept_workload(a)
    n_ref, t_ref, s_ref = oracle.spec_accept(a.p, a.q, a.draft_tok, a.n_draft, a.u)[:3]
    assert (n_acc == n_ref).all() and (nxt == t_ref).all() and status == s_ref


@pytest.mark.parametrize("V", [(1 << 19) - 1, 1 << 19])
def test_largest_vocabulary(hip, V):
    # the limit of the interface: rows of 2^19 logits stream through the output row (no register variant)
    rng = np.random.default_rng(V)
    logits = (rng.standard_normal((2, V)) * 3).astype(np.float32)
    for T, top_p in ((0.2, 0.95), (1.0, 0.9)):
        got, status = hip.run_warp_probs(logits, T, top_p)
        assert status == 0
        assert check_rows(logits, T, top_p, got) <= 1
