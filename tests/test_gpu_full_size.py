"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times (default work spread, append fused into the attention launch).  The oracle cannot compute
every output row of these sizes in seconds, so rows are sampled (always including the extremes:
shortest / longest sequence, first / last query, first / last head) and checked one by one;
plus properties that hold at any size."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 2e-2  # bf16 inputs: the contractual bar
# Regression tripwires, about twice what the kernels measure on these inputs (O: the bf16 rounding of the
# probabilities; lse: fp32 sums of exact products).  |O| is about 0.05 at these context lengths, so the
# contractual bar alone would let a lost 32-token block pass; these and tests/test_gpu_exact_counts.py do not.
TRIP_O = 5e-3
TRIP_LSE = 2e-4


def softmax_mass(w, b, i, h, lse_gpu):
    """sum_j exp(s_j - lse) over the tokens row (b, i, h) may see, with the scores recomputed in fp64 from the
    inputs and lse as the GPU returned it: 1 if and only if the kernel's denominator counted every visible
    token once (a pin on the returned lse that needs no reference lse)."""
    g = w.Hq // w.Hkv
    n = int(w.ctx_len[b]) + i + 1
    q = wl.bf16_bits_to_f32(w.Q[b, i, h]).astype(np.float64)
    k = wl.bf16_bits_to_f32(w.K[b, :n, h // g]).astype(np.float64)
    return float(np.exp(k @ q * w.scale - float(lse_gpu)).sum())


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def sample_rows(w, rng, n):
    rows = set()
    order = np.argsort(w.ctx_len)
    for b in (int(order[0]), int(order[-1])):
        for i in (0, int(w.draft_len[b]) - 1):
            for h in (0, w.Hq - 1):
                rows.add((b, i, h))
    while len(rows) < n:
        b = int(rng.integers(w.B))
        rows.add((b, int(rng.integers(w.draft_len[b])), int(rng.integers(w.Hq))))
    return sorted(rows)


@pytest.mark.parametrize("make,nsample", [(wl.config2, 48), (wl.config4, 48), (wl.config3, 40)])
def test_full_size_sampled_rows(hip, make, nsample):
    w = make(0)
    print(f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} kv_bytes={w.kv_bytes}", flush=True)
    O, lse, status, da = hip.run_attention_workload(w, poison=True, fused=True)
    assert status == 0
    assert np.isfinite(O).all() and np.isfinite(lse).all()
    for b in range(w.B):
        assert (O[b, int(w.draft_len[b]):] == 0).all() and (lse[b, int(w.draft_len[b]):] == 0).all()
    worst = worst_l = 0.0
    for (b, i, h) in sample_rows(w, np.random.default_rng(1), nsample):
        ref, lref = oracle.verify_attention_row(w.Q, w.K, w.V, b, i, h, int(w.ctx_len[b]), w.scale)
        err = float(np.abs(O[b, i, h] - ref).max())
        worst = max(worst, err)
        assert err <= TOL, (b, i, h, err)
        assert err <= TRIP_O, (b, i, h, err)
        lerr = abs(float(lse[b, i, h]) - lref)
        worst_l = max(worst_l, lerr)
        assert lerr <= TRIP_LSE, (b, i, h, lerr)
        mass = softmax_mass(w, b, i, h, lse[b, i, h])
        assert abs(mass - 1.0) <= 2 * TRIP_LSE, (b, i, h, mass)
    print(f"{w.name}: worst sampled max-abs error {worst:.3e}, lse {worst_l:.3e}", flush=True)
    # launches on the same caches (rows already appended) are deterministic: two un-fused launches agree
    # bit for bit, and with the fused one up to the rounding of a different split of the context
    import torch
    Q, ctx, nq = hip.to_device(w.Q), hip.i32(w.ctx_len), hip.i32(w.draft_len)
    O2, lse2 = (hip.to_host(t) for t in da.verify(Q, ctx, nq))
    O3, lse3 = (hip.to_host(t) for t in da.verify(Q, ctx, nq))
    np.testing.assert_array_equal(O2, O3)
    np.testing.assert_array_equal(lse2, lse3)
    assert np.abs(O2 - O).max() <= 5e-3 and np.abs(lse2 - lse).max() <= 5e-3


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (16, 2)])
def test_one_very_long_context(hip, Hq, Hkv):
    # 100 000 cached tokens in one sequence next to a short one (3 126 blocks per kv head, spread over the
    # whole chip; dozens of partials per unit); one query tile per kv head and three (grouped queries)
    w = wl.make_attention("long_ctx", 2, Hq, Hkv, 128, "bf16", [100000, 40], [3, 2], 11, kmax=3, Lcap=100008)
    O, lse, status, _ = hip.run_attention_workload(w, poison=True, fused=True)
    assert status == 0 and np.isfinite(O).all() and np.isfinite(lse).all()
    worst = 0.0
    for b in range(w.B):
        for i in range(int(w.draft_len[b])):
            for h in sorted({0, Hq // 2, Hq - 1}):
                ref, lref = oracle.verify_attention_row(w.Q, w.K, w.V, b, i, h, int(w.ctx_len[b]), w.scale)
                worst = max(worst, float(np.abs(O[b, i, h] - ref).max()))
                assert abs(float(lse[b, i, h]) - lref) <= TRIP_LSE, (b, i, h)
                assert abs(softmax_mass(w, b, i, h, lse[b, i, h]) - 1.0) <= 2 * TRIP_LSE, (b, i, h)
    print(f"long context: worst max-abs error {worst:.3e}", flush=True)
    assert worst <= TOL and worst <= TRIP_O
