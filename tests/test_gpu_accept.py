"""GPU parity: bass_spec_accept (through the C ABI) against the oracle, bit-exact."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def check(hip, a, ctx=None):
    ref = oracle.spec_accept(a.p, a.q, a.draft_tok, a.n_draft, a.u, ctx)
    got = hip.run_accept_workload(a, ctx)
    np.testing.assert_array_equal(got[0], ref[0])
    np.testing.assert_array_equal(got[1], ref[1])
    assert got[2] == ref[2]
    if ctx is not None:
        np.testing.assert_array_equal(got[3], ref[3])
    return got


def test_config1_accept_vocab64(hip):
    for seed in range(5):
        check(hip, wl.config1_accept(seed), ctx=[37, 90])


def test_config5_accept_vocab50k(hip):
    for seed in range(3):
        n_acc, nxt, st = check(hip, wl.config5_accept(seed))
        assert st == 0


@pytest.mark.parametrize("V", [1, 3, 4, 255, 256, 257, 1000, 4099])
def test_odd_vocab_sizes_and_ragged_draft_counts(hip, V):
    a = wl.make_accept("odd", 7, 3, V, V, 2.0, 1.0, n_draft=[3, 0, 1, 2, 3, 0, 3])
    check(hip, a, ctx=np.arange(7) * 10)


def test_many_random_rows_bit_exact(hip):
    # 4096 independent (p, q, u) rows in a few launches
    for seed in range(4):
        a = wl.make_accept("rows", 1024, 2, 64, 100 + seed, 2.0, None)
        check(hip, a)


def test_degenerate_rows_and_status_bits(hip):
    a = wl.make_accept("deg", 4, 2, 8, 1, 2.0, 1.0)
    a.q[0] = a.p[0, :2]                      # identical models
    a.p[1, 0] = 0                            # zero mass row -> status
    a.draft_tok[2, 1] = 99                   # token id out of range -> clamped
    a.n_draft = np.array([2, 2, 2, 5], np.int32)  # 5 > kmax -> clamped
    got = check(hip, a)
    assert got[2] & 7 == 7


@pytest.mark.parametrize("V", [(1 << 19) - 1, 1 << 19])
def test_largest_vocabulary(hip, V):
    # 2^19 entries is the limit of the interface (it keeps the integer weight sum below 2^63): 512 chunks of
    # 1024 entries in the kernel, the last one ragged for 2^19 - 1
    a = wl.make_accept("vmax", 3, 2, V, 5, 3.0, 1.0, n_draft=[2, 0, 1])
    check(hip, a)


def test_no_drafts_at_all_is_plain_sampling(hip):
    # kmax = 0: no draft model rows exist (q and draft_tok are empty); every sequence draws its token from p_0
    for V in (300, 50000):
        a = wl.make_accept("k0", 5, 0, V, 3, 2.0, 1.0)
        n_acc, nxt, st = check(hip, a)
        assert st == 0 and (n_acc == 0).all()
