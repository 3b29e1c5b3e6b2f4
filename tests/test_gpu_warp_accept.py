"""GPU parity of bass_warp_accept (logits -> accepted prefix and next token in one call).

The call is defined as bass_warp_probs on the main- and the draft-model logits followed by bass_spec_accept on
the rows it made (Section 2.2; temperature and top-p of Section 4's table captions), without the rows being
stored.  Integer results, so the bar is equality:
  * with the two calls, on everything the call returns (n_accept, next_token, ctx_len, status bits);
  * with the ORACLE's acceptance run on the library-made probability rows (the rows themselves are checked
    against the oracle's warp in test_gpu_logit_warp.py);
  * with the oracle's own warp + acceptance, except where fp32 and fp64 values of 2^x put a decision on
    different sides (counted, and rare).
"""
import numpy as np
import pytest

import oracle
import oracle.logit_warp as ow
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def drafts_for(lt, ld, rng, greedy_share=0.5):
    """Draft tokens: the draft model's most likely token, or (for a share of them) one of its ten most likely."""
    B, kmax, V = ld.shape
    tok = np.zeros((B, kmax), np.int32)
    for b in range(B):
        for i in range(kmax):
            order = np.argsort(-ld[b, i], kind="stable")[:min(10, V)]
            tok[b, i] = order[0] if rng.random() < greedy_share else order[int(rng.integers(len(order)))]
    return tok


def both(hip, lt, ld, T, top_p, tok, nd, u, ctx=None):
    fused = hip.run_warp_accept(lt, ld, T, top_p, tok, nd, u, ctx)
    two = hip.run_warp_accept(lt, ld, T, top_p, tok, nd, u, ctx, two_calls=True)
    for a, b in zip(fused, two):
        np.testing.assert_array_equal(a, b)
    return fused


@pytest.mark.parametrize("T,top_p", [(0.2, 0.95), (1.0, 0.9), (1.0, 1.0), (0.7, 0.5)])
@pytest.mark.parametrize("V", [1, 7, 64, 1000, 1025, 4099, 5000])
def test_small_vocabularies_equal_the_two_calls(hip, V, T, top_p):
    rng = np.random.default_rng([V, int(T * 10)])
    B, kmax = 7, 3
    lt, ld = wl.make_logits(B, kmax, V, V, 3.0, 1.0)
    tok = drafts_for(lt, ld, rng)
    nd = np.array([3, 0, 1, 2, 3, 0, 3], np.int32)
    u = rng.random((B, kmax + 1), dtype=np.float32)
    both(hip, lt, ld, T, top_p, tok, nd, u, ctx=np.arange(B) * 10)


@pytest.mark.parametrize("V", [32768, 50000, 53252, 60000, 65540, 70001])
def test_vocabularies_of_every_row_variant(hip, V):
    # register variants of 8 / 13 / 16 groups per thread, the streaming variant, unaligned rows
    rng = np.random.default_rng(V)
    B, kmax = 3, 2
    lt, ld = wl.make_logits(B, kmax, V, V, 3.0, 1.0)
    tok = drafts_for(lt, ld, rng)
    u = rng.random((B, kmax + 1), dtype=np.float32)
    for T, top_p in ((0.2, 0.95), (1.0, 0.9)):
        both(hip, lt, ld, T, top_p, tok, np.array([2, 1, 2], np.int32), u)


def test_full_step_shape_against_the_oracle(hip):
    # B = 8, k = 5, V = 50 000 at the paper's sampling settings
    B, kmax, V, T, top_p = 8, 5, 50000, 0.2, 0.95
    open_decisions = 0
    for seed in range(3):
        rng = np.random.default_rng([seed, 5])
        lt, ld = wl.make_logits(B, kmax, V, seed, 3.0, 1.0)
        tok = drafts_for(lt, ld, rng)
        nd = np.full(B, kmax, np.int32)
        u = rng.random((B, kmax + 1), dtype=np.float32)
        n_acc, nxt, status = both(hip, lt, ld, T, top_p, tok, nd, u)
        assert status == 0
        assert 0 < n_acc.sum() < B * kmax            # the recipe exercises acceptances and rejections
        # the oracle's acceptance on the rows the library's front end makes: equal, always
        p, _ = hip.run_warp_probs(lt, T, top_p)
        q, _ = hip.run_warp_probs(ld, T, top_p)
        n_ref, t_ref, s_ref = oracle.spec_accept(p, q, tok, nd, u)[:3]
        np.testing.assert_array_equal(n_acc, n_ref)
        np.testing.assert_array_equal(nxt, t_ref)
        assert status == s_ref
        # the oracle's own warp (fp64) in front of its acceptance: equal unless a decision is open between
        # fp32 and fp64 values of 2^x
        po = np.stack([[ow.warp_row(lt[b, i], T, top_p)[0] for i in range(kmax + 1)] for b in range(B)]).astype(np.float32)
        qo = np.stack([[ow.warp_row(ld[b, i], T, top_p)[0] for i in range(kmax)] for b in range(B)]).astype(np.float32)
        n_o, t_o = oracle.spec_accept(po, qo, tok, nd, u)[:2]
        open_decisions += int(((n_o != n_acc) | (t_o != nxt)).sum())
    print(f"sequences whose result differs from the all-fp64 front end: {open_decisions} of {3 * B}", flush=True)
    assert open_decisions <= 2


def test_ties_at_the_threshold_are_judged_by_token_id(hip):
    # ten equal tokens, top_p 0.35: tokens 0..3 are kept with probability 1/4, 4..9 have probability 0 in both
    # models.  A draft among the kept ones is accepted (p = q), one outside is rejected (u q = 0 is not < 0).
    V = 10
    lt, ld = np.zeros((4, 2, V), np.float32), np.zeros((4, 1, V), np.float32)
    tok = np.array([[0], [3], [4], [9]], np.int32)
    u = np.full((4, 2), 0.5, np.float32)
    n_acc, nxt, status = both(hip, lt, ld, 1.0, 0.35, tok, np.ones(4, np.int32), u)
    np.testing.assert_array_equal(n_acc, [1, 1, 0, 0])
    assert (nxt < 4).all() and status == 0
    # two levels, the cut inside the lower one, spread over many threads (V = 4096: 2048 tokens of weight 3,
    # 2048 of weight 1, all heavy ones and the 101 light ones of lowest id are kept)
    V = 4096
    row = np.zeros(V, np.float32)
    row[::2] = np.log(3.0)
    top_p = (3 * 2048 + 100.5) / (3 * 2048 + 2048)
    lt, ld = np.tile(row, (3, 2, 1)), np.tile(row, (3, 1, 1))
    ld[:, :, :] += 0.25 * (np.arange(V) % 2 == 0)   # the draft model likes the heavy tokens a bit more
    tok = np.array([[1 + 2 * 100], [1 + 2 * 101], [2]], np.int32)  # last kept light token, first dropped one, a heavy one
    u = np.full((3, 2), 0.999, np.float32)
    both(hip, lt, ld, 1.0, top_p, tok, np.ones(3, np.int32), u)


def test_degenerate_rows_and_status_bits(hip):
    import paper_2404_15778_amd as bass
    B, kmax, V = 5, 2, 300
    lt, ld = wl.make_logits(B, kmax, V, 1, 3.0, 1.0)
    rng = np.random.default_rng(2)
    tok = drafts_for(lt, ld, rng)
    u = rng.random((B, kmax + 1), dtype=np.float32)
    ld[0] = lt[0, :kmax]                 # identical models and u = 1: rejected, the residual has no mass -> draw from p
    u[0, 0] = 1.0
    lt[1, 0] = -np.inf                   # a main-model row without any finite logit
    lt[2, 1, 5] = np.nan                 # NaN gets probability 0
    lt[2, 2, 9] = np.inf                 # +inf takes everything
    tok[3, 1] = 999                      # token id out of range -> clamped
    nd = np.array([2, 2, 2, 2, 7], np.int32)   # 7 > kmax -> clamped
    n_acc, nxt, status = both(hip, lt, ld, 1.0, 0.9, tok, nd, u)
    assert status & bass.STATUS_ZERO_MASS and status & bass.STATUS_TOKEN_CLAMPED and status & bass.STATUS_LEN_CLAMPED
    assert n_acc[0] == 0 and n_acc[1] == 0


def test_no_drafts_at_all_is_plain_sampling(hip):
    for V in (300, 50000):
        lt, _ = wl.make_logits(5, 0, V, 3, 3.0, 1.0)
        u = np.random.default_rng(V).random((5, 1), dtype=np.float32)
        n_acc, nxt, status = both(hip, lt, None, 0.2, 0.95, None, np.zeros(5, np.int32), u)
        assert status == 0 and (n_acc == 0).all()


@pytest.mark.parametrize("B", [1, 300])
def test_one_and_many_sequences(hip, B):
    # one sequence: its row pass is divided over as many workgroups as it has chunks; 300: one workgroup each
    V, kmax = 20000, 2
    rng = np.random.default_rng(B)
    lt, ld = wl.make_logits(B, kmax, V, B, 3.0, 1.0)
    tok = drafts_for(lt, ld, rng)
    u = rng.random((B, kmax + 1), dtype=np.float32)
    both(hip, lt, ld, 0.2, 0.95, tok, rng.integers(0, kmax + 1, B).astype(np.int32), u)


def test_more_drafts_than_the_kernel_stages(hip):
    # summaries of up to 33 rows per model are staged in LDS; longer drafts read the others from memory
    B, kmax, V = 3, 40, 600
    rng = np.random.default_rng(40)
    lt, ld = wl.make_logits(B, kmax, V, 40, 3.0, 0.3)
    tok = drafts_for(lt, ld, rng, greedy_share=1.0)
    u = rng.random((B, kmax + 1), dtype=np.float32) * 0.5     # mostly accepted: the prefix runs past row 33
    n_acc, _, _ = both(hip, lt, ld, 0.5, 0.95, tok, np.array([40, 37, 40], np.int32), u)
    print("accepted", n_acc.tolist(), flush=True)
    assert n_acc.max() > 33


@pytest.mark.parametrize("V", [(1 << 19) - 1, 1 << 19])
def test_largest_vocabulary(hip, V):
    rng = np.random.default_rng(V)
    lt, ld = wl.make_logits(2, 1, V, 7, 3.0, 1.0)
    tok = drafts_for(lt, ld, rng)
    u = rng.random((2, 2), dtype=np.float32)
    both(hip, lt, ld, 1.0, 0.9, tok, np.array([1, 0], np.int32), u)


def test_calls_in_a_row_on_one_workspace(hip):
    # the arrival counters and partial sums of a call must not leak into the next one (a smaller one here)
    import torch
    import paper_2404_15778_amd as bass
    dev = "cuda"
    ws = torch.empty(bass.bass_warp_accept_workspace_bytes(8, 3, 50000), dtype=torch.uint8, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    for rep, (B, kmax, V) in enumerate([(8, 3, 50000), (3, 1, 9000), (8, 3, 50000)]):
        rng = np.random.default_rng(rep)
        lt, ld = wl.make_logits(B, kmax, V, rep, 3.0, 1.0)
        tok = drafts_for(lt, ld, rng)
        u = rng.random((B, kmax + 1), dtype=np.float32)
        nd = np.full(B, kmax, np.int32)
        want = hip.run_warp_accept(lt, ld, 0.2, 0.95, tok, nd, u, two_calls=True)
        n_accept = torch.full((B,), -1, dtype=torch.int32, device=dev)
        next_token = torch.full((B,), -1, dtype=torch.int32, device=dev)
        for _ in range(3):
            bass.bass_warp_accept(hip.to_device(lt), hip.to_device(ld), 0.2, 0.95, hip.i32(tok), hip.i32(nd), hip.to_device(u),
                                  n_accept, next_token, ws, None, status)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(hip.to_host(n_accept), want[0])
        np.testing.assert_array_equal(hip.to_host(next_token), want[1])
    assert int(status.item()) == 0


def test_arguments_are_checked(hip):
    import torch
    import paper_2404_15778_amd as bass
    lt = torch.zeros((2, 2, 64), device="cuda")
    ld = torch.zeros((2, 1, 64), device="cuda")
    i32z = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    u = torch.zeros((2, 2), device="cuda")
    ws = torch.empty(bass.bass_warp_accept_workspace_bytes(2, 1, 64), dtype=torch.uint8, device="cuda")
    with pytest.raises(bass.BassError):   # workspace too small
        bass.bass_warp_accept(lt, ld, 1.0, 0.9, i32z(2, 1), i32z(2), u, i32z(2), i32z(2), ws[:256])
    with pytest.raises(bass.BassError):   # temperature must be positive
        bass.bass_warp_accept(lt, ld, 0.0, 0.9, i32z(2, 1), i32z(2), u, i32z(2), i32z(2), ws)
    assert bass.bass_warp_accept_workspace_bytes(2, 1, (1 << 19) + 1) == 0
