"""Pins for the attention oracle (CPU only).

The oracle is the SPLIT-style definition (each sequence at its true length).  It is
pinned here against: a PAD-style dense masked formulation built from library routines
(numpy matmul + scipy softmax), closed forms, invariants and special cases.
"""
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
import workloads as wl


def pad_style_reference(w, Kf=None, Vf=None, Qf=None):
    """Dense BASS-PAD formulation: pad every sequence to the longest, give padded and
    not-yet-visible positions a score of -inf (probability exactly 0), library softmax."""
    f = (lambda a: wl.bf16_bits_to_f32(a).astype(np.float64)) if w.dtype == "bf16" else (lambda a: a.astype(np.float64))
    Q = f(w.Q) if Qf is None else Qf
    K = f(w.K) if Kf is None else Kf
    V = f(w.V) if Vf is None else Vf
    B, kmax, Hq, D = Q.shape
    Lmax = K.shape[1]
    g = Hq // w.Hkv
    Kh = np.repeat(K, g, axis=2)  # [B,L,Hq,D]
    Vh = np.repeat(V, g, axis=2)
    S = np.einsum("bihd,bjhd->bhij", Q, Kh) * w.scale  # [B,Hq,kmax,Lmax]
    j = np.arange(Lmax)[None, None, None, :]
    i = np.arange(kmax)[None, None, :, None]
    L = w.ctx_len[:, None, None, None]
    visible = j <= L + i
    S = np.where(visible, S, -np.inf)
    P = softmax(S, axis=-1)
    O = np.einsum("bhij,bjhd->bihd", P, Vh)
    lse = logsumexp(S, axis=-1).transpose(0, 2, 1)  # [B,kmax,Hq]
    rows = (np.arange(kmax)[None, :] < w.draft_len[:, None])
    O = O * rows[:, :, None, None]
    lse = lse * rows[:, :, None]
    return O, lse


def small(dtype, seed, B=3, Hq=4, Hkv=2, D=16, ctx=(5, 0, 33), nq=(3, 1, 4), kmax=None):
    return wl.make_attention("small", B, Hq, Hkv, D, dtype, list(ctx), list(nq), seed, kmax=kmax)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("seed", [0, 1])
def test_matches_pad_style_dense_reference(dtype, seed):
    w = small(dtype, seed, kmax=5)
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    Or, lser = pad_style_reference(w)
    np.testing.assert_allclose(O, Or, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lser, rtol=0, atol=1e-12)


def test_config1_matches_dense_reference():
    w = wl.config1()
    assert w.ctx_len.tolist() == [37, 90] and w.draft_len.tolist() == [4, 3]
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    Or, lser = pad_style_reference(w)
    np.testing.assert_allclose(O, Or, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lser, rtol=0, atol=1e-12)


def test_probability_rows_sum_to_one_and_mask_is_exact():
    w = small("fp32", 3)
    for b in range(w.B):
        for i in range(int(w.draft_len[b])):
            out, lse, probs = oracle.verify_attention_row(w.Q, w.K, w.V, b, i, 1, int(w.ctx_len[b]), w.scale,
                                                          want_probs=True)
            assert probs.shape == (int(w.ctx_len[b]) + i + 1,)  # nothing beyond ctx_len+i is visible
            assert abs(probs.sum() - 1.0) < 1e-14
            assert (probs > 0).all()


def test_row_function_equals_full_function():
    w = small("bf16", 4)
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    for b in range(w.B):
        for i in range(int(w.draft_len[b])):
            for h in range(w.Hq):
                out, l = oracle.verify_attention_row(w.Q, w.K, w.V, b, i, h, int(w.ctx_len[b]), w.scale)
                np.testing.assert_array_equal(out, O[b, i, h])
                assert l == lse[b, i, h]


def test_draft_len_one_is_ordinary_decode_attention():
    # one query per sequence over ctx_len+1 keys: the textbook single-token decode step
    w = wl.make_attention("decode", 2, 2, 2, 8, "fp32", [6, 11], [1, 1], 5)
    O, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    for b in range(2):
        n = int(w.ctx_len[b]) + 1
        for h in range(2):
            s = (w.K[b, :n, h].astype(np.float64) @ w.Q[b, 0, h].astype(np.float64)) * w.scale
            expect = softmax(s) @ w.V[b, :n, h].astype(np.float64)
            np.testing.assert_allclose(O[b, 0, h], expect, atol=1e-13)


def test_empty_context_first_query_returns_first_value_row():
    w = wl.make_attention("empty", 1, 2, 2, 8, "fp32", [0], [3], 6)
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    np.testing.assert_array_equal(O[0, 0], w.V[0, 0].astype(np.float64))  # softmax over one key is 1


def test_constant_values_give_that_value():
    w = small("fp32", 7)
    v = np.linspace(-1, 1, w.D).astype(np.float32)
    w.V[:] = v
    O, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    for b in range(w.B):
        nq = int(w.draft_len[b])
        np.testing.assert_allclose(O[b, :nq], np.broadcast_to(v, (nq, w.Hq, w.D)), atol=1e-14)
        assert (O[b, nq:] == 0).all()  # unused query slots are zero


def test_zero_keys_give_uniform_attention_closed_form():
    w = small("fp32", 8)
    w.K[:] = 0
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    g = w.Hq // w.Hkv
    for b in range(w.B):
        for i in range(int(w.draft_len[b])):
            n = int(w.ctx_len[b]) + i + 1
            for h in range(w.Hq):
                np.testing.assert_allclose(O[b, i, h], w.V[b, :n, h // g].astype(np.float64).mean(0), atol=1e-14)
                assert abs(lse[b, i, h] - math.log(n)) < 1e-14


def test_scale_is_applied_to_scores_once():
    # with one dominant key direction, doubling the scale must equal doubling Q
    w = small("fp32", 9)
    O2, l2 = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, 2 * w.scale)
    Oq, lq = oracle.verify_attention((2 * w.Q).astype(np.float32), w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    np.testing.assert_allclose(O2, Oq, atol=1e-13)
    np.testing.assert_allclose(l2, lq, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    w = small("fp32", 10, Hq=6, Hkv=2)
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    g = 3
    Om, lm = oracle.verify_attention(w.Q, np.repeat(w.K, g, axis=2), np.repeat(w.V, g, axis=2), w.ctx_len,
                                     w.draft_len, w.scale)
    np.testing.assert_array_equal(O, Om)
    np.testing.assert_array_equal(lse, lm)


def test_sequences_are_independent_and_permutable():
    w = small("bf16", 11)
    O, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    perm = [2, 0, 1]
    Op, _ = oracle.verify_attention(w.Q[perm], w.K[perm], w.V[perm], w.ctx_len[perm], w.draft_len[perm], w.scale)
    np.testing.assert_array_equal(Op, O[perm])
    K2 = w.K.copy()
    K2[2] ^= 0x8000  # flip the sign of every key of sequence 2
    O2, _ = oracle.verify_attention(w.Q, K2, w.V, w.ctx_len, w.draft_len, w.scale)
    np.testing.assert_array_equal(O2[[0, 1]], O[[0, 1]])
    assert not np.array_equal(O2[2], O[2])


def test_causal_among_drafts_and_blind_to_rows_beyond_valid():
    w = small("fp32", 12, ctx=(5, 2, 9), nq=(3, 2, 4), kmax=4)
    O, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    K2, V2 = w.K.copy(), w.V.copy()
    b = 2
    last = int(w.ctx_len[b]) + int(w.draft_len[b]) - 1  # the last draft token's own row
    K2[b, last] += 1.0
    V2[b, last] -= 3.0
    # rows beyond the valid range of other sequences hold garbage
    K2[0, int(w.ctx_len[0]) + int(w.draft_len[0]):] = np.nan
    V2[0, int(w.ctx_len[0]) + int(w.draft_len[0]):] = np.inf
    O2, _ = oracle.verify_attention(w.Q, K2, V2, w.ctx_len, w.draft_len, w.scale)
    nq = int(w.draft_len[b])
    np.testing.assert_array_equal(O2[b, : nq - 1], O[b, : nq - 1])  # earlier queries cannot see it
    assert not np.array_equal(O2[b, nq - 1], O[b, nq - 1])          # the last query sees itself
    np.testing.assert_array_equal(O2[0], O[0])
    assert np.isfinite(O2).all()


def test_dominant_key_selects_its_value_row():
    # a key aligned with the query with a huge score takes all the probability
    w = wl.make_attention("dom", 1, 1, 1, 8, "fp32", [20], [2], 13)
    w.K[0, :, 0] = 0
    w.Q[0, :, 0] = 0
    w.Q[0, :, 0, 0] = 1.0
    w.K[0, 7, 0, 0] = 1e4
    O, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    np.testing.assert_allclose(O[0, 0, 0], w.V[0, 7, 0], atol=1e-12)
    np.testing.assert_allclose(O[0, 1, 0], w.V[0, 7, 0], atol=1e-12)


def test_bf16_inputs_are_widened_exactly():
    w = small("bf16", 14)
    O, lse = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    # same numbers handed over as fp32 must give the identical fp64 result
    f = wl.bf16_bits_to_f32
    O32, lse32 = oracle.verify_attention(f(w.Q), f(w.K), f(w.V), w.ctx_len, w.draft_len, w.scale)
    np.testing.assert_array_equal(O, O32)
    np.testing.assert_array_equal(lse, lse32)
    # and the rounding helper is round-to-nearest-even (spot values)
    x = np.array([1.0, 1.00390625, 1.005859375, -2.0, 3.140625], np.float32)
    assert wl.to_bf16_bits(x).tolist() == [0x3F80, 0x3F80, 0x3F81, 0xC000, 0x4049]


def test_kv_append_oracle_is_a_row_copy():
    rng = np.random.default_rng(0)
    cache = np.zeros((2, 10, 2, 4), np.float32)
    rows = rng.standard_normal((2, 3, 2, 4)).astype(np.float32)
    oracle.kv_append(cache, rows, [4, 7], [2, 3])
    expect = np.zeros_like(cache)
    expect[0, 4:6] = rows[0, :2]
    expect[1, 7:10] = rows[1, :3]
    np.testing.assert_array_equal(cache, expect)
