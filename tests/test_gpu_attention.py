"""GPU parity: bass_kv_append + bass_verify_attention (through the C ABI) against the fp64 oracle.

Bars (max-abs error of O): 2e-2 for bf16 inputs, 1e-5 for fp32 inputs.  lse is checked to
the same bars.  Caches are pre-filled with a NaN byte pattern, so any read beyond a
sequence's valid range shows up as a NaN in the output.
"""
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


def check_against_oracle(hip, w, waves=None, fused=False):
    import paper_2404_15778_amd as bass
    if waves is not None:
        bass.bass_set_attention_waves(waves)
    try:
        O, lse, status, _ = hip.run_attention_workload(w, poison=True, fused=fused)
    finally:
        bass.bass_set_attention_waves(0)
    Or, lser = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    assert status == 0
    assert np.isfinite(O).all() and np.isfinite(lse).all()
    err = np.abs(O - Or).max()
    lerr = np.abs(lse - lser).max()
    print(f"{w.name}: max|O-oracle|={err:.3e} max|lse-oracle|={lerr:.3e}", flush=True)
    assert err <= TOL[w.dtype], err
    assert lerr <= TOL[w.dtype], lerr
    for b in range(w.B):  # unused query slots are exactly zero
        assert (O[b, int(w.draft_len[b]):] == 0).all() and (lse[b, int(w.draft_len[b]):] == 0).all()
    return O, lse


def test_config1_tiny_fp32(hip):
    check_against_oracle(hip, wl.config1())


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("seed", [0, 1])
def test_small_ragged_bf16(hip, D, seed):
    # several 32-token blocks, ragged tails, an empty context, an inactive sequence
    w = wl.make_attention("small_bf16", 5, 4, 4, D, "bf16", [37, 90, 0, 200, 64], [4, 3, 2, 0, 6], seed, kmax=6,
                          Lcap=300)
    check_against_oracle(hip, w)


@pytest.mark.parametrize("waves", [64, 256, 8192])
def test_result_does_not_depend_on_the_work_spread(hip, waves):
    w = wl.make_attention("spread", 3, 4, 2, 128, "bf16", [300, 31, 1000], [5, 1, 3], 3, kmax=5, Lcap=1100)
    check_against_oracle(hip, w, waves=waves)


@pytest.mark.parametrize("g,kmax", [(2, 6), (4, 6), (8, 6), (8, 8)])
def test_grouped_query_heads_bf16(hip, g, kmax):
    nq = [kmax, 1, max(1, kmax - 2)]
    w = wl.make_attention("gqa", 3, 2 * g, 2, 128, "bf16", [150, 33, 257], nq, g, kmax=kmax, Lcap=300)
    check_against_oracle(hip, w)


def test_fp32_grouped_and_wide_heads(hip):
    w = wl.make_attention("fp32_gqa", 3, 6, 2, 128, "fp32", [70, 0, 130], [3, 2, 5], 5, kmax=5, Lcap=140)
    check_against_oracle(hip, w)
    w = wl.make_attention("fp32_many_rows", 2, 4, 1, 32, "fp32", [40, 9], [7, 3], 6, kmax=7, Lcap=64)
    check_against_oracle(hip, w)  # 28 query rows per kv head: more than one row chunk


def test_draft_len_one_is_decode_attention(hip):
    w = wl.make_attention("decode", 4, 8, 8, 128, "bf16", [511, 512, 513, 31], [1, 1, 1, 1], 7, kmax=1, Lcap=520)
    check_against_oracle(hip, w)


def test_kv_append_then_gather_is_bit_exact(hip):
    import torch
    for dtype in ("bf16", "fp32"):
        w = wl.make_attention("rt", 3, 4, 2, 64, dtype, [45, 0, 97], [3, 2, 4], 8, kmax=4, Lcap=128)
        _, _, status, da = hip.run_attention_workload(w)
        total = w.ctx_len + w.draft_len
        n = int(total.max())
        K, V = da.gather(hip.i32(np.zeros(w.B)), hip.i32(total), n)
        torch.cuda.synchronize()
        K, V = hip.to_host(K), hip.to_host(V)
        for b in range(w.B):
            t = int(total[b])
            np.testing.assert_array_equal(K[b, :t], w.K[b, :t])
            np.testing.assert_array_equal(V[b, :t], w.V[b, :t])
        assert status == 0


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("fp32", 64)])
@pytest.mark.parametrize("waves", [64, 1024])
def test_fused_append_verify_equals_separate_calls(hip, dtype, D, waves):
    import torch
    import paper_2404_15778_amd as bass
    # step rows straddle 32-token block boundaries (ctx 30, 63) and wavefront share boundaries
    w = wl.make_attention("fused", 5, 8, 4, D, dtype, [30, 63, 0, 500, 129], [6, 3, 2, 5, 0], 9, kmax=6, Lcap=520)
    check_against_oracle(hip, w, waves=waves, fused=True)
    bass.bass_set_attention_waves(waves)
    try:
        O1, lse1, st1, da1 = hip.run_attention_workload(w, poison=True, fused=False)
        O2, lse2, st2, da2 = hip.run_attention_workload(w, poison=True, fused=True)
    finally:
        bass.bass_set_attention_waves(0)
    # the fused launch splits the context at other points, so O agrees up to that rounding only
    split_tol = 5e-3 if dtype == "bf16" else 1e-5
    assert np.abs(O1 - O2).max() <= split_tol and np.abs(lse1 - lse2).max() <= split_tol
    assert st1 == 0 and st2 == 0
    total = w.ctx_len + w.draft_len
    n = int(total.max())
    for da in (da1, da2):
        K, V = da.gather(hip.i32(np.zeros(w.B)), hip.i32(total), n)
        torch.cuda.synchronize()
        K, V = hip.to_host(K), hip.to_host(V)
        for b in range(w.B):
            t = int(total[b])
            np.testing.assert_array_equal(K[b, :t], w.K[b, :t])
            np.testing.assert_array_equal(V[b, :t], w.V[b, :t])


def test_repeated_calls_share_one_workspace(hip):
    # the arrival counters must be left clean by every call: same workspace, different shapes / spreads
    import torch
    import paper_2404_15778_amd as bass
    w = wl.make_attention("rep", 4, 4, 4, 128, "bf16", [700, 90, 333, 1500], [3, 6, 1, 4], 11, kmax=6, Lcap=1600)
    Or, _ = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    _, _, _, da = hip.run_attention_workload(w, poison=True)
    Q = hip.to_device(w.Q)
    ctx, nq = hip.i32(w.ctx_len), hip.i32(w.draft_len)
    try:
        for waves in (64, 1024, 200, 8192, 64):
            bass.bass_set_attention_waves(waves)
            for _ in range(3):
                da.O.fill_(float("nan"))
                O, _ = da.verify(Q, ctx, nq)
                torch.cuda.synchronize()
                assert np.abs(hip.to_host(O) - Or).max() <= TOL["bf16"]
    finally:
        bass.bass_set_attention_waves(0)
    assert int(da.status.item()) == 0


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("fp32", 64)])
@pytest.mark.parametrize("variant", ["pad", "split"])
def test_pad_and_split_launch_variants_match_the_oracle(hip, dtype, D, variant):
    # Section 3.2: BASS-PAD (padded positions take part and get probability exactly 0) and BASS-SPLIT
    # (one launch per sequence) compute the same ragged attention; the caches are poisoned with NaN
    # beyond every sequence's valid range, which PAD reads
    import torch
    w = wl.make_attention("variants", 5, 8, 4, D, dtype, [30, 63, 0, 500, 129], [6, 3, 2, 5, 0], 13, kmax=6, Lcap=520)
    Or, lser = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    _, _, _, da = hip.run_attention_workload(w, poison=True)
    Q, ctx, nq = hip.to_device(w.Q), hip.i32(w.ctx_len), hip.i32(w.draft_len)
    longest = int((w.ctx_len + w.draft_len).max())
    for padded_len in ((longest, w.Lcap, 10) if variant == "pad" else (0,)):
        da.O.fill_(float("nan"))
        da.lse.fill_(float("nan"))
        O, lse = da.verify(Q, ctx, nq, variant=variant, padded_len=padded_len)
        torch.cuda.synchronize()
        O, lse = hip.to_host(O), hip.to_host(lse)
        assert int(da.status.item()) == 0
        assert np.isfinite(O).all() and np.isfinite(lse).all()
        assert np.abs(O - Or).max() <= TOL[dtype]
        assert np.abs(lse - lser).max() <= TOL[dtype]


@pytest.mark.parametrize("D,Hq,Hkv,kmax", [(128, 16, 2, 6), (64, 8, 1, 8), (128, 6, 2, 6), (128, 16, 4, 8)])
@pytest.mark.parametrize("waves", [0, 64, 200, 8192])
def test_grouped_query_shapes_over_work_spreads_and_variants(hip, D, Hq, Hkv, kmax, waves):
    # 48, 64, 18 and 32 query rows per kv head: the workgroup-level kernel (one 16-row tile per wavefront) with
    # few and many workgroups, units shorter than a workgroup's stretch and longer, and the PAD / SPLIT variants
    import torch
    import paper_2404_15778_amd as bass
    ctx = [700, 31, 0, 333, 64, 1]
    nq = [kmax, 1, 2, kmax - 1, 0, kmax]
    w = wl.make_attention("gqa_tiles", 6, Hq, Hkv, D, "bf16", ctx, nq, 29, kmax=kmax, Lcap=720)
    Or, lser = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
    _, _, _, da = hip.run_attention_workload(w, poison=True)
    Q, c, n = hip.to_device(w.Q), hip.i32(w.ctx_len), hip.i32(w.draft_len)
    longest = int((w.ctx_len + w.draft_len).max())
    bass.bass_set_attention_waves(waves)
    try:
        for variant in ("ragged", "pad", "split"):
            da.O.fill_(float("nan"))
            da.lse.fill_(float("nan"))
            O, lse = da.verify(Q, c, n, variant=variant, padded_len=longest)
            torch.cuda.synchronize()
            O, lse = hip.to_host(O), hip.to_host(lse)
            assert int(da.status.item()) == 0
            assert np.isfinite(O).all() and np.isfinite(lse).all()
            assert np.abs(O - Or).max() <= TOL["bf16"], variant
            assert np.abs(lse - lser).max() <= TOL["bf16"], variant
    finally:
        bass.bass_set_attention_waves(0)


@pytest.mark.parametrize("seed", range(6))
def test_random_lengths_and_work_spreads(hip, seed):
    # the even split of the block list, the units' virtual blocks (behind and in front of the last real
    # block) and the contributor ranges of the split-context merge, over random lengths and spreads: short
    # units, units of one block, stretches shorter and longer than a unit, inactive sequences
    rng = np.random.default_rng([seed, 0x5C4ED])
    for _ in range(5):
        B = int(rng.integers(1, 7))
        kmax = int(rng.integers(1, 7))
        ctx = rng.integers(0, 330, size=B)
        ctx[rng.random(B) < 0.3] = rng.integers(0, 40, size=int((rng.random(B) < 0.3).sum()) or 1)[0]
        nq = rng.integers(0, kmax + 1, size=B)
        if nq.max() == 0:
            nq[0] = 1
        Hkv = int(rng.choice([1, 2, 4]))
        D = int(rng.choice([64, 128]))
        waves = int(rng.choice([64, 68, 128, 192, 320, 512, 768, 1024]))
        w = wl.make_attention(f"rnd{seed}", B, Hkv, Hkv, D, "bf16", ctx, nq, int(rng.integers(1 << 30)), kmax=kmax,
                              Lcap=int(ctx.max()) + kmax + int(rng.integers(0, 40)))
        for fused in (False, True):
            check_against_oracle(hip, w, waves=waves, fused=fused)


@pytest.mark.parametrize("ctx", [1500, 1531, 290])
@pytest.mark.parametrize("fused", [False, True])
def test_one_unit_merged_from_dozens_of_partials(hip, ctx, fused):
    # a single sequence with one kv head spread over more wavefronts than it has blocks: every wavefront
    # delivers a partial of one block, and the merge goes through its rounds for the partials beyond the
    # eighth with full and with ragged last rounds (48, 49 and 10 contributors)
    w = wl.make_attention("one_unit", 1, 1, 1, 128, "bf16", [ctx], [3], ctx, kmax=3, Lcap=ctx + 40)
    check_against_oracle(hip, w, waves=256, fused=fused)


@pytest.mark.parametrize("dtype,tol", [("bf16", 5e-3), ("fp32", 1e-5)])
@pytest.mark.parametrize("waves", [768, 8192])
def test_alternating_inputs_on_one_workspace(hip, dtype, tol, waves):
    # The merging wavefront must see the partial results of THIS launch: a contributor's arrival may be counted
    # only after its partial stores have landed.  Two different batches alternate on the same caches' worth of
    # workspace, with short contexts spread over many wavefronts (every unit has several contributors), so that
    # a stale partial -- the other batch's values, left in the same slot by the previous launch -- would be an
    # error of the order of the outputs themselves, far above the bar used here (tighter than the contractual
    # one: at these short contexts |O| is 0.1 - 1).
    import torch
    import paper_2404_15778_amd as bass
    D = 128 if dtype == "bf16" else 64
    lens, nq = [400, 90, 257, 33, 480, 150], [4, 1, 3, 4, 2, 4]
    batches = [wl.make_attention(f"alt{s}", 6, 4, 4, D, dtype, lens, nq, 100 + s, kmax=4, Lcap=512) for s in (0, 1)]
    refs = [oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale) for w in batches]
    das, Qs = [], []
    for w in batches:
        _, _, _, da = hip.run_attention_workload(w, poison=True)
        das.append(da)
        Qs.append(hip.to_device(w.Q))
    ctx, n = hip.i32(lens), hip.i32(nq)
    shared = das[0].ws  # both batches' launches use this one workspace
    bass.bass_set_attention_waves(waves)
    try:
        for it in range(12):
            k = it % 2
            da = das[k]
            da.O.fill_(float("nan"))
            bass.bass_verify_attention(da.desc, Qs[k], da.Kc, da.Vc, ctx, n, da.O, da.lse, shared, da.status)
            torch.cuda.synchronize()
            assert np.abs(hip.to_host(da.O) - refs[k][0]).max() <= tol, (it, k)
            assert np.abs(hip.to_host(da.lse) - refs[k][1]).max() <= tol, (it, k)
    finally:
        bass.bass_set_attention_waves(0)
    assert int(das[0].status.item()) == 0 and int(das[1].status.item()) == 0
