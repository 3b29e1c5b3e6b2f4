"""Pins for the speculative-sampling acceptance oracle (CPU only).

The rule is stochastic but fully specified; it is pinned against what the paper and
the mathematics fix: the emitted token is distributed exactly as the main model's p
(Section 2.2), the accepted-prefix law P(n >= i) = prod alpha_m, the paper's worked
numbers for the geometric model (Section 2.2.1, fixture), library inverse-CDF sampling
for the k = 0 special case, an exact rational-arithmetic brute force, and edge cases.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

import oracle
import workloads as wl

F32 = np.float32


def read_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def exact_rule_python(p, q, tok, k, u):
    """The same rule in exact rational arithmetic (Python ints / Fractions), one sequence."""
    kmax = q.shape[0]
    n = 0
    for i in range(k):
        x = int(tok[i])
        if Fraction(float(u[i])) * Fraction(float(q[i, x])) < Fraction(float(p[i, x])):
            n += 1
        else:
            break
    def weights(resid):
        W = []
        for j in range(p.shape[1]):
            w = F32(p[n, j]) - F32(q[n, j]) if resid else F32(p[n, j])   # fp32 subtraction
            w = Fraction(float(w))
            w = min(max(w, Fraction(0)), Fraction(1))
            W.append(int(w * 2**44))  # floor for non-negative rationals
        return W
    W = weights(n < k)
    if sum(W) == 0 and n < k:
        W = weights(False)
    S = sum(W)
    ur = min(max(Fraction(float(u[kmax])), Fraction(0)), Fraction(1) - Fraction(1, 2**24))
    T = (int(ur * 2**32) * S) >> 32
    c = 0
    for j, wj in enumerate(W):
        c += wj
        if c > T:
            return n, j
    return n, 0


@pytest.mark.parametrize("seed", range(3))
def test_matches_exact_rational_brute_force(seed):
    a = wl.make_accept("t", 6, 4, 16, seed, 2.0, 1.0, n_draft=[4, 3, 0, 4, 1, 2])
    n_acc, nxt, st = oracle.spec_accept(a.p, a.q, a.draft_tok, a.n_draft, a.u)
    assert st == 0
    for b in range(a.B):
        n, t = exact_rule_python(a.p[b], a.q[b], a.draft_tok[b], int(a.n_draft[b]), a.u[b])
        assert (int(n_acc[b]), int(nxt[b])) == (n, t)


def first_token_distribution(p_row, q_row, N=4096):
    """Deterministic quadrature over the two uniforms: distribution of the first emitted
    token when the draft x ~ q_row is judged against p_row (k = 1)."""
    V = p_row.shape[0]
    grid = ((np.arange(N) + 0.5) / N).astype(F32)
    dist = np.zeros(V)
    p = np.zeros((N, 2, V), F32)
    p[:, 0] = p_row
    p[:, 1] = p_row  # bonus row unused for the first token
    q = np.broadcast_to(q_row, (N, 1, V)).astype(F32)
    # resample distribution (needs a rejected draft): take u0 = largest grid value with a draft that rejects
    for x in range(V):
        if q_row[x] == 0:
            continue
        u = np.stack([grid, grid], axis=1)  # u0 sweeps the accept test
        n_acc, _, _ = oracle.spec_accept(p, q, np.full((N, 1), x), np.ones(N, np.int32), u)
        acc_frac = n_acc.mean()
        dist[x] += q_row[x] * acc_frac
        if acc_frac < 1.0:
            u = np.stack([np.full(N, 0.999999, F32), grid], axis=1)  # rejected: sweep the resample uniform
            n_acc, nxt, _ = oracle.spec_accept(p, q, np.full((N, 1), x), np.ones(N, np.int32), u)
            if (n_acc == 0).all():
                dist += q_row[x] * (1 - acc_frac) * np.bincount(nxt, minlength=V) / N
            else:  # ratio so close to 1 that u=0.999999 still accepts: rejection mass is negligible
                assert 1 - acc_frac < 1e-3
    return dist


def test_first_emitted_token_is_distributed_as_p_quadrature():
    # dyadic probabilities so that fp32 holds them exactly
    p_row = np.array([8, 1, 4, 3], F32) / 16
    q_row = np.array([2, 6, 4, 4], F32) / 16
    dist = first_token_distribution(p_row, q_row)
    np.testing.assert_allclose(dist, p_row, atol=2e-3)
    a = wl.make_accept("t", 1, 1, 8, 5, 2.0, None)
    dist = first_token_distribution(a.p[0, 0], a.q[0, 0])
    np.testing.assert_allclose(dist, a.p[0, 0], atol=2e-3)


@pytest.mark.parametrize("V", [4, 8, 64])
def test_chi_square_emitted_token_follows_target(V):
    rng = np.random.default_rng(100 + V)
    a = wl.make_accept("t", 1, 1, V, V, 2.0, None)
    p_row, q_row = a.p[0, 0], a.q[0, 0]
    N = 200_000
    x = rng.choice(V, size=N, p=q_row.astype(np.float64) / q_row.astype(np.float64).sum())
    p = np.broadcast_to(a.p[0], (N, 2, V))
    q = np.broadcast_to(a.q[0], (N, 1, V))
    u = rng.random((N, 2), dtype=F32)
    n_acc, nxt, st = oracle.spec_accept(p, q, x.reshape(N, 1), np.ones(N, np.int32), u)
    first = np.where(n_acc == 1, x, nxt)
    obs = np.bincount(first, minlength=V).astype(np.float64)
    exp = p_row.astype(np.float64) / p_row.astype(np.float64).sum() * N
    keep = exp >= 5
    chi2 = ((obs[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    assert stats.chi2.sf(chi2, keep.sum() - 1) > 1e-3
    # a planted mistake (residual taken as q-p) must be caught by the same statistic
    wrong = np.where(n_acc == 1, x, rng.choice(V, size=N, p=np.maximum(q_row - p_row, 0) / np.maximum(q_row - p_row, 0).sum()))
    obs_w = np.bincount(wrong, minlength=V).astype(np.float64)
    assert stats.chi2.sf(((obs_w[keep] - exp[keep]) ** 2 / exp[keep]).sum(), keep.sum() - 1) < 1e-6


def test_accepted_prefix_law_closed_form():
    # P(n >= i) = prod_{m<i} alpha_m with alpha_m = sum_j min(p_m[j], q_m[j]) when x_m ~ q_m
    k, V, N = 4, 16, 100_000
    a = wl.make_accept("t", 1, k, V, 21, 2.0, 1.0)
    rng = np.random.default_rng(22)
    q64 = a.q[0].astype(np.float64)
    tok = np.stack([rng.choice(V, size=N, p=q64[i] / q64[i].sum()) for i in range(k)], axis=1)
    p = np.broadcast_to(a.p[0], (N, k + 1, V))
    q = np.broadcast_to(a.q[0], (N, k, V))
    u = rng.random((N, k + 1), dtype=F32)
    n_acc, _, _ = oracle.spec_accept(p, q, tok, np.full(N, k, np.int32), u)
    alpha = np.minimum(a.p[0, :k].astype(np.float64), q64).sum(axis=1)
    surv = np.cumprod(alpha)
    for i in range(1, k + 1):
        emp = (n_acc >= i).mean()
        sd = np.sqrt(surv[i - 1] * (1 - surv[i - 1]) / N)
        assert abs(emp - surv[i - 1]) < 5 * sd + 1e-4, (i, emp, surv[i - 1])


def test_paper_worked_example_geometric_model(golden_dir):
    gold = read_golden(os.path.join(golden_dir, "naive_batched_sd_example.txt"))
    a_prob = gold["accept_prob"]
    # one-hot draft on token 0 with p(0) = 0.8: each draft is accepted with probability exactly min(1, .8/1)
    V, k, N = 2, 64, 40_000
    p_row = np.array([a_prob, 1 - a_prob], F32)
    q_row = np.array([1.0, 0.0], F32)
    p = np.broadcast_to(p_row, (N, k + 1, V))
    q = np.broadcast_to(q_row, (N, k, V))
    rng = np.random.default_rng(7)
    u = rng.random((N, k + 1), dtype=F32)
    n_acc, nxt, _ = oracle.spec_accept(p, q, np.zeros((N, k), np.int32), np.full(N, k, np.int32), u)
    tokens_per_draft = (n_acc + 1).mean()  # accepted drafts plus the corrected token
    assert abs(tokens_per_draft - gold["tokens_per_draft"]) < 0.08
    assert abs(tokens_per_draft - 1 / (1 - float(F32(a_prob)))) < 0.08
    # a rejected draft is always corrected to the only token with residual mass
    assert (nxt[n_acc < k] == 1).all()
    # naive batching: a batch of b sequences advances only to the first rejection anywhere in the batch
    b = int(gold["batch"])
    groups = n_acc[: (N // b) * b].reshape(-1, b)
    per_pos = (groups.min(axis=1) >= 1).mean()
    assert round(100 * a_prob**b) == gold["batch_accept_percent"]
    assert abs(100 * per_pos - gold["batch_accept_percent"]) < 1.5
    naive_tokens = (groups.min(axis=1) + 1).mean()
    assert abs(naive_tokens - gold["batch_tokens_per_draft"]) < 0.05


def test_no_drafts_reduces_to_library_inverse_cdf_sampling():
    a = wl.make_accept("t", 64, 0, 1000, 3, 3.0, None)
    n_acc, nxt, st = oracle.spec_accept(a.p, a.q, a.draft_tok, a.n_draft, a.u)
    assert (n_acc == 0).all() and st == 0
    for b in range(a.B):
        W = np.floor(a.p[b, 0].astype(np.float64) * 2.0**44).astype(np.uint64)
        cdf = np.cumsum(W)
        U = int(np.floor(float(a.u[b, 0]) * 2.0**32))
        T = (U * int(cdf[-1])) >> 32
        assert int(nxt[b]) == int(np.searchsorted(cdf, T, side="right"))
        # and agrees with plain floating inverse-CDF sampling except within rounding of a CDF step
    cdf64 = np.cumsum(a.p[:, 0].astype(np.float64), axis=1)
    plain = np.array([np.searchsorted(cdf64[b], float(a.u[b, 0]) * cdf64[b, -1], side="right") for b in range(a.B)])
    assert (plain == nxt).mean() > 0.95


def test_identical_models_accept_everything_and_draw_bonus_from_last_row():
    a = wl.make_accept("t", 16, 3, 32, 9, 2.0, None)
    q = a.p[:, :3].copy()
    n_acc, nxt, _ = oracle.spec_accept(a.p, q, a.draft_tok, a.n_draft, a.u)
    ok = np.take_along_axis(a.p[:, :3], a.draft_tok[:, :, None], axis=2)[:, :, 0] > 0
    assert (n_acc[ok.all(axis=1)] == 3).all()
    # bonus token = inverse CDF of row k with the dedicated uniform
    n0, nxt0, _ = oracle.spec_accept(a.p[:, 3:], np.zeros((16, 0, 32), F32), np.zeros((16, 0), np.int32),
                                     np.zeros(16, np.int32), a.u[:, 3:])
    np.testing.assert_array_equal(nxt[ok.all(axis=1)], nxt0[ok.all(axis=1)])


def test_rejected_draft_with_zero_target_mass_resamples_from_p():
    V = 8
    p_row = np.array([0, .25, .25, 0, .125, .125, .25, 0], F32)
    q_row = np.zeros(V, F32)
    q_row[0] = 1.0  # draft model is certain about a token the main model forbids
    N = 4096
    p = np.broadcast_to(p_row, (N, 2, V))
    q = np.broadcast_to(q_row, (N, 1, V))
    u = np.stack([np.zeros(N, F32), ((np.arange(N) + 0.5) / N).astype(F32)], axis=1)  # even u = 0 cannot accept p = 0
    n_acc, nxt, _ = oracle.spec_accept(p, q, np.zeros((N, 1), np.int32), np.ones(N, np.int32), u)
    assert (n_acc == 0).all()
    np.testing.assert_allclose(np.bincount(nxt, minlength=V) / N, p_row, atol=1e-3)  # residual = p exactly here
    assert not np.isin(nxt, [0, 3, 7]).any()  # zero-weight tokens are never emitted


def test_strict_comparison_and_edge_uniforms():
    V = 4
    p = np.array([[[.5, .5, 0, 0], [.25, .25, .25, .25]]], F32)
    q = np.array([[[.5, .25, .25, 0]]], F32)
    one = np.ones(1, np.int32)
    # ratio exactly 1: every u in [0,1) accepts
    assert oracle.spec_accept(p, q, [[0]], one, np.array([[0.99999994, 0.5]], F32))[0][0] == 1
    # ratio 2 (>1) accepts
    assert oracle.spec_accept(p, q, [[1]], one, np.array([[0.99999994, 0.5]], F32))[0][0] == 1
    # p = 0 is never accepted, not even with u = 0
    assert oracle.spec_accept(p, q, [[2]], one, np.array([[0.0, 0.5]], F32))[0][0] == 0
    # q = 0, p > 0 (cannot be drafted, but defined): accepted since u*0 < p
    q2 = np.array([[[0, .5, .5, 0]]], F32)
    assert oracle.spec_accept(p, q2, [[0]], one, np.array([[0.9, 0.5]], F32))[0][0] == 1
    # u exactly at the ratio is a rejection (strict '<'): p/q = .5 -> u = .5 rejects, just below accepts
    p3 = np.array([[[.25, .75, 0, 0], [1, 0, 0, 0]]], F32)
    q3 = np.array([[[.5, .5, 0, 0]]], F32)
    assert oracle.spec_accept(p3, q3, [[0]], one, np.array([[0.5, 0.5]], F32))[0][0] == 0
    assert oracle.spec_accept(p3, q3, [[0]], one, np.array([[0.49999997, 0.5]], F32))[0][0] == 1
    # after the rejection above the residual is max(p-q,0) = [0,.25,0,0] -> token 1 whatever the uniform
    for ur in [0.0, 0.3, 0.99999994, 1.0, 7.0]:
        assert oracle.spec_accept(p3, q3, [[0]], one, np.array([[0.5, ur]], F32))[1][0] == 1


def test_resample_boundaries_follow_cumulative_weights():
    # residual weights [0, .5, 0, .5] (after rejecting token 0): u < .5 -> token 1, u >= .5 -> token 3
    p = np.array([[[0, .5, 0, .5], [1, 0, 0, 0]]], F32)
    q = np.array([[[1, 0, 0, 0]]], F32)
    one = np.ones(1, np.int32)
    for ur, want in [(0.0, 1), (0.49999997, 1), (0.5, 3), (0.99999994, 3)]:
        n, t, _ = oracle.spec_accept(p, q, [[0]], one, np.array([[0.0, ur]], F32))
        assert (n[0], t[0]) == (0, want)


def test_stops_at_first_rejection_and_advances_lengths():
    V = 4
    p = np.tile(np.array([.5, .5, 0, 0], F32), (1, 5, 1))
    q = np.tile(np.array([.5, .5, 0, 0], F32), (1, 4, 1))
    p[0, 2] = [0, 0, .5, .5]  # draft 2 (token 0) has no target mass -> rejected; later drafts are not looked at
    tok = np.zeros((1, 4), np.int32)
    n, t, st, ctx = oracle.spec_accept(p, q, tok, [4], np.full((1, 5), 0.25, F32), ctx_len=[100])
    assert (n[0], st) == (2, 0) and t[0] == 2 and ctx[0] == 103  # 0.25 < 0.5 of residual [0,0,.5,.5]
    # n_draft limits how many drafts are judged
    n, t, st, ctx = oracle.spec_accept(p, q, tok, [1], np.full((1, 5), 0.25, F32), ctx_len=[100])
    assert n[0] == 1 and ctx[0] == 102 and t[0] == 0  # bonus row is p[1] = [.5,.5,0,0], u=.25 -> token 0


def test_degenerate_inputs_set_status_bits():
    V = 4
    p = np.tile(np.array([.25, .25, .25, .25], F32), (1, 3, 1))
    q = p[:, :2].copy()
    u = np.full((1, 3), 0.5, F32)
    _, _, st = oracle.spec_accept(p, q, [[1, 9]], [2], u)
    assert st & oracle.STATUS_TOKEN_CLAMPED
    n, _, st = oracle.spec_accept(p, q, [[1, 1]], [5], u)
    assert st & oracle.STATUS_LEN_CLAMPED and n[0] <= 2
    # residual without mass (p == q) after a forced rejection cannot happen (ratio 1 accepts); force p row of zeros
    pz = p.copy()
    pz[0, 0] = 0
    n, t, st = oracle.spec_accept(pz, q, [[1, 1]], [2], u)
    assert n[0] == 0 and t[0] == 0 and st & oracle.STATUS_ZERO_MASS
    # p <= q everywhere with a rejected draft: falls back to sampling p itself
    p2 = np.array([[[.25, .25, .5, 0], [1, 0, 0, 0]]], F32)
    q2 = np.array([[[.25, .25, .5, 0]]], F32)
    p2[0, 0, 0] = 0.125  # p(0) < q(0), nowhere p > q
    n, t, st = oracle.spec_accept(p2, q2, [[0]], [1], np.array([[0.75, 0.2]], F32))
    assert n[0] == 0 and st == 0 and t[0] == 1  # weights p = [.125,.25,.5,0]/.875: u=.2 -> cumulative .175 -> token 1
