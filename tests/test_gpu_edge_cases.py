"""GPU edge cases of the attention path: degenerate batches, exact-fit caches, clamped lengths,
more sequences than a wavefront has lanes, the largest query-row count."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "fp32": 1e-5}


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def check(hip, w, fused=False):
    O, lse, status, da = hip.run_attention_workload(w, poison=True, fused=fused)
    Or, lser = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    assert status == 0 and np.isfinite(O).all()
    assert np.abs(O - Or).max() <= TOL[w.dtype]
    assert np.abs(lse - lser).max() <= TOL[w.dtype]
    return O, da


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_all_sequences_inactive_gives_zeros(hip, dtype):
    w = wl.make_attention("inactive", 3, 4, 2, 64, dtype, [10, 0, 40], [0, 0, 0], 0, kmax=3, Lcap=64)
    O, lse, status, _ = hip.run_attention_workload(w, poison=True)
    assert status == 0 and (O == 0).all() and (lse == 0).all()


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("fused", [False, True])
def test_single_sequence_and_empty_contexts(hip, dtype, fused):
    check(hip, wl.make_attention("one", 1, 2, 2, 64, dtype, [0], [1], 1, kmax=1, Lcap=1), fused)
    check(hip, wl.make_attention("empty_ctx", 4, 4, 4, 64, dtype, [0, 0, 0, 0], [4, 1, 2, 3], 2, kmax=4, Lcap=40), fused)


@pytest.mark.parametrize("ctx", [31, 32, 33, 63, 64, 65])
def test_lengths_around_block_boundaries(hip, ctx):
    w = wl.make_attention("edge", 2, 2, 2, 128, "bf16", [ctx, ctx - 1], [1, 2], ctx, kmax=2, Lcap=96)
    check(hip, w, fused=True)


def test_cache_filled_to_capacity(hip):
    # the last draft row lands on the cache's last token, capacity a multiple of the block size and not
    for Lcap in (96, 100):
        w = wl.make_attention("full", 2, 4, 4, 128, "bf16", [Lcap - 4, Lcap - 1], [4, 1], Lcap, kmax=4, Lcap=Lcap)
        check(hip, w, fused=True)


@pytest.mark.parametrize("B", [70, 64, 65, 200])
def test_more_sequences_than_lanes(hip, B):
    # the schedule keeps 64 sequences at a time in a wavefront's lanes: exactly one chunk, one more sequence,
    # two chunks, and four with a ragged last one
    rng = np.random.default_rng(5 if B == 70 else B)
    ctx = rng.integers(0, 80, size=B)
    nq = rng.integers(0, 4, size=B)
    nq[[0, 63, B - 1]] = [2, 3, 1]
    for dtype in ("bf16", "fp32", "int8"):
        w = wl.make_attention(f"b{B}", B, 2, 2, 64, "bf16" if dtype == "int8" else dtype, ctx, nq, 6, kmax=3, Lcap=96)
        if dtype == "int8":
            import test_gpu_kv_int8 as i8
            i8.check(hip, w, two_step=False)
        else:
            check(hip, w, fused=(dtype == "bf16"))


def test_group_sizes_around_the_multiply_shift_division(hip):
    # a query row r of a kv head is token r / g, head r % g of the group; the kernels divide by g with a
    # host-prepared multiply-shift up to g = 64 and with a plain division beyond (fp32 only: the matrix-core
    # kernels stop at 64 rows per kv head)
    for Hq, Hkv in ((3, 1), (7, 1), (64, 1), (65, 1), (130, 2), (96, 1)):
        w = wl.make_attention(f"g{Hq // Hkv}", 2, Hq, Hkv, 64, "fp32", [45, 70], [3, 2], 19, kmax=3, Lcap=80)
        check(hip, w)
    for Hq, Hkv in ((3, 1), (6, 2), (7, 1), (63, 1)):
        w = wl.make_attention(f"g{Hq // Hkv}b", 2, Hq, Hkv, 64, "bf16", [45, 70], [1, 1], 23, kmax=1, Lcap=80)
        check(hip, w, fused=True)


def test_largest_row_count_bf16(hip):
    # kmax * (Hq / Hkv) = 64 query rows per kv head: four 16-row tiles
    w = wl.make_attention("rows64", 2, 16, 2, 128, "bf16", [100, 37], [8, 5], 7, kmax=8, Lcap=128)
    check(hip, w)
    w = wl.make_attention("rows64_d64", 2, 16, 2, 64, "bf16", [100, 37], [8, 5], 7, kmax=8, Lcap=128)
    check(hip, w, fused=True)


@pytest.mark.parametrize("D,kmax,Hq,Hkv", [(128, 12, 4, 4), (128, 16, 2, 2), (64, 32, 2, 2), (128, 20, 2, 2),
                                            (64, 24, 4, 2), (128, 9, 2, 1)])
@pytest.mark.parametrize("waves", [0, 64])
def test_fused_append_with_long_drafts(hip, D, kmax, Hq, Hkv, waves):
    # more than 8 new rows of 128 elements take several copies inside the launch; beyond
    # kmax * D = 2048 the append runs as a launch of its own: results and caches are the same
    import torch
    import paper_2404_15778_amd as bass
    ctx = [100, 37, 31, 0, 60]
    nq = [kmax, kmax - 3, 9, kmax, 1]
    w = wl.make_attention("long", 5, Hq, Hkv, D, "bf16", ctx, nq, 21, kmax=kmax, Lcap=160)
    bass.bass_set_attention_waves(waves)
    try:
        _, da = check(hip, w, fused=True)
    finally:
        bass.bass_set_attention_waves(0)
    total = w.ctx_len + w.draft_len
    K, V = da.gather(hip.i32(np.zeros(w.B)), hip.i32(total), int(total.max()))
    torch.cuda.synchronize()
    K, V = hip.to_host(K), hip.to_host(V)
    for b in range(w.B):
        t = int(total[b])
        np.testing.assert_array_equal(K[b, :t], w.K[b, :t])
        np.testing.assert_array_equal(V[b, :t], w.V[b, :t])


def test_lengths_outside_the_cache_are_clamped_and_reported(hip):
    import torch
    import paper_2404_15778_amd as bass
    w = wl.make_attention("clamp", 3, 2, 2, 128, "bf16", [50, 20, 30], [2, 2, 2], 8, kmax=2, Lcap=64)
    _, _, _, da = hip.run_attention_workload(w, poison=False)
    Q = hip.to_device(w.Q)
    bad_ctx = hip.i32([50, 63, -5])    # 63 + 2 > Lcap, negative length
    bad_nq = hip.i32([2, 2, 7])        # 7 > kmax
    da.status.zero_()
    O, _ = da.verify(Q, bad_ctx, bad_nq)
    torch.cuda.synchronize()
    assert int(da.status.item()) & bass.STATUS_LEN_CLAMPED
    assert np.isfinite(hip.to_host(O)).all()
    # the well-formed sequence is unaffected
    Or, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    assert np.abs(hip.to_host(O)[0] - Or[0]).max() <= TOL["bf16"]
    # append outside the cache: rows are dropped and reported
    da.status.zero_()
    Kn = torch.zeros((3, 2, 2, 128), dtype=torch.bfloat16, device="cuda")
    da.append(Kn, Kn, hip.i32([63, 0, 0]), hip.i32([2, 0, 5]))
    torch.cuda.synchronize()
    assert int(da.status.item()) & bass.STATUS_LEN_CLAMPED


def test_lse_is_optional(hip):
    import torch
    w = wl.make_attention("nolse", 2, 4, 4, 128, "bf16", [70, 10], [3, 2], 9, kmax=3, Lcap=80)
    _, _, _, da = hip.run_attention_workload(w, poison=True)
    Or, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    O, _ = da.verify(hip.to_device(w.Q), hip.i32(w.ctx_len), hip.i32(w.draft_len), want_lse=False)
    torch.cuda.synchronize()
    assert np.abs(hip.to_host(O) - Or).max() <= TOL["bf16"]


def test_gqa_equals_mha_with_repeated_kv_heads_on_gpu(hip):
    w = wl.make_attention("gqa", 2, 8, 2, 128, "bf16", [90, 45], [3, 2], 10, kmax=3, Lcap=100)
    O, _, _, _ = hip.run_attention_workload(w)
    m = wl.make_attention("mha", 2, 8, 8, 128, "bf16", [90, 45], [3, 2], 10, kmax=3, Lcap=100)
    m.Q, m.K, m.V = w.Q, np.repeat(w.K, 4, axis=2), np.repeat(w.V, 4, axis=2)
    Om, _, _, _ = hip.run_attention_workload(m)
    # same numbers, different work decomposition: equal up to the split-context rounding
    assert np.abs(O - Om).max() <= 1e-5


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("fp32", 64)])
def test_long_appends_at_unaligned_offsets_keep_their_neighbours(hip, dtype, D):
    # many rows at once (a prompt, a moved sequence) take the block-wise path of the bf16 cache: blocks that
    # the rows cover only partly keep their other tokens; rows beyond the cache are dropped and reported
    import torch
    import paper_2404_15778_amd as bass
    B, H, Lcap = 3, 2, 200
    first = [40, 0, 33]          # tokens already there
    more = [70, 100, 64]         # rows appended behind them in one call
    w = wl.make_attention("long_append", B, H, H, D, dtype, [a + b for a, b in zip(first, more)], [1, 1, 1], 3,
                          kmax=1, Lcap=Lcap)
    da = hip.DeviceAttention(B, 1, H, H, D, Lcap, dtype, w.scale, poison=True)
    K, V = w.K, w.V
    n1, n2 = max(first), max(more)
    A = np.zeros((B, n1, H, D), K.dtype)
    Av = np.zeros_like(A)
    Bk = np.zeros((B, n2, H, D), K.dtype)
    Bv = np.zeros_like(Bk)
    for b in range(B):
        A[b, :first[b]], Av[b, :first[b]] = K[b, :first[b]], V[b, :first[b]]
        Bk[b, :more[b]], Bv[b, :more[b]] = K[b, first[b]:first[b] + more[b]], V[b, first[b]:first[b] + more[b]]
    da.append(hip.to_device(A), hip.to_device(Av), hip.i32([0] * B), hip.i32(first))
    da.append(hip.to_device(Bk), hip.to_device(Bv), hip.i32(first), hip.i32(more))
    total = np.array(first) + np.array(more)
    Kg, Vg = da.gather(hip.i32([0] * B), hip.i32(total), int(total.max()))
    torch.cuda.synchronize()
    Kg, Vg = hip.to_host(Kg), hip.to_host(Vg)
    for b in range(B):
        np.testing.assert_array_equal(Kg[b, :total[b]], K[b, :total[b]])
        np.testing.assert_array_equal(Vg[b, :total[b]], V[b, :total[b]])
    assert int(da.status.item()) == 0
    # rows that would run past the capacity are dropped and reported, the ones inside are written
    da.append(hip.to_device(Bk), hip.to_device(Bv), hip.i32([Lcap - 10, 0, 0]), hip.i32([64, 0, 0]))
    torch.cuda.synchronize()
    assert int(da.status.item()) & bass.STATUS_LEN_CLAMPED
    Kg, _ = da.gather(hip.i32([Lcap - 10, 0, 0]), hip.i32([10, 0, 0]), 10)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(hip.to_host(Kg)[0, :10], Bk[0, :10])


@pytest.mark.parametrize("dtype,D,Lcap", [("bf16", 128, 70000), ("fp32", 64, 70000)])
@pytest.mark.parametrize("fused", [False, True])
def test_caches_beyond_four_gib(hip, dtype, D, Lcap, fused):
    # 10 sequences x 32 kv heads x 70 000 tokens of capacity: 5.7 GB per cache tensor, so that the last
    # sequences' rows lie beyond byte offset 2^32 (append, fetch and the fused append's stores all address
    # the cache with 64-bit offsets); the contexts themselves are short, so the oracle covers every row
    w = wl.make_attention("big_cache", 10, 32, 32, D, dtype, [300, 0, 17, 64, 1, 100, 33, 250, 5, 129],
                          [4, 1, 2, 3, 4, 1, 2, 3, 4, 1], 7, kmax=4, Lcap=Lcap)
    check(hip, w, fused)
