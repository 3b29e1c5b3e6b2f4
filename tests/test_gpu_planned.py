"""GPU: the step plan (bass_attention_plan) and the attention that consumes it (bass_verify_attention_planned).

The planning kernel must write, in every part a launch reads, exactly what the host planner writes (whose
invariants tests/test_attention_plan.py checks on the CPU); the planned attention must agree bit for bit
with the entry points that plan inside the call, and with the fp64 oracle to the usual bars; a launch that
is handed a plan made for something else must compute nothing and say so.
"""
import numpy as np
import pytest

import oracle
import workloads as wl
from test_attention_plan import parse_plan

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "fp32": 1e-5}


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def device_plan(hip, desc, ctx_len, draft_len, flags, padded_len=0):
    import torch
    import paper_2404_15778_amd as bass
    plan = bass.alloc_plan(desc)
    plan.fill_(0xA5)  # a plan buffer needs no clearing
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    bass.bass_attention_plan(desc, hip.i32(ctx_len), hip.i32(draft_len), flags, padded_len, plan, status)
    torch.cuda.synchronize()
    return plan, int(status.item())


def assert_same_plan(dev_bytes, host_bytes, B, Hkv):
    d, h = parse_plan(dev_bytes, B, Hkv), parse_plan(host_bytes, B, Hkv)
    np.testing.assert_array_equal(d["hdr"], h["hdr"])
    np.testing.assert_array_equal(d["records"], h["records"])
    for r in h["records"]:  # the overflow entries the records point at
        if int(r[16]) > 2:
            lo, hi = int(r[17]), int(r[17]) + int(r[16]) - 2
            np.testing.assert_array_equal(d["overflow"][lo:hi], h["overflow"][lo:hi])
    for part in ("seq_L", "seq_nq", "seq_inc", "owners"):
        np.testing.assert_array_equal(d[part], h[part])


@pytest.mark.parametrize("case", ["cfg2", "cfg3", "cfg4", "tiny_units", "clamped", "many_sequences", "padded"])
def test_device_plan_equals_host_plan(hip, case):
    import paper_2404_15778_amd as bass
    rng = np.random.default_rng(5)
    flags, padded, dtype = bass.PLAN_APPEND, 0, "bf16"
    if case in ("cfg2", "cfg3", "cfg4"):
        w = {"cfg2": wl.config2, "cfg3": wl.config3, "cfg4": wl.config4}[case](1, tensors=False)
        B, kmax, Hq, Hkv, Lcap, ctx, dl = w.B, w.kmax, w.Hq, w.Hkv, w.Lcap, w.ctx_len, w.draft_len
    elif case == "tiny_units":
        B, kmax, Hq, Hkv, Lcap = 70, 4, 8, 8, 300
        ctx, dl = rng.integers(0, 60, B), rng.integers(0, 5, B)
    elif case == "clamped":
        B, kmax, Hq, Hkv, Lcap = 5, 4, 4, 4, 200
        ctx, dl = np.array([500, -3, 199, 10, 0]), np.array([2, 9, 4, -1, 1])
    elif case == "many_sequences":  # more sequences than the planning workgroup has threads
        B, kmax, Hq, Hkv, Lcap, dtype = 2500, 2, 2, 1, 70, "fp32"
        ctx, dl = rng.integers(0, 69, B), rng.integers(0, 3, B)
    else:
        B, kmax, Hq, Hkv, Lcap, flags, padded = 6, 3, 4, 4, 1000, 0, 800
        ctx, dl = rng.integers(0, 900, B), rng.integers(0, 4, B)
    desc = bass.make_desc(B, kmax, Hq, Hkv, 128 if dtype == "bf16" else 64, Lcap, dtype, 1.0)
    plan, status = device_plan(hip, desc, ctx, dl, flags, padded)
    host, hstatus = bass.bass_attention_plan_host(desc, ctx, dl, flags, padded)
    assert status == hstatus
    assert_same_plan(plan.cpu().numpy(), host, B, Hkv)


def run_planned(hip, w, fused, waves=0, plan_flags=None, plan_bytes=None):
    """Context in the cache, then plan + planned attention.  Returns O, lse, status, DeviceAttention."""
    import torch
    import paper_2404_15778_amd as bass
    bass.bass_set_attention_waves(waves)
    try:
        da = hip.DeviceAttention(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, w.dtype, w.scale, poison=True)
        K, V = hip.to_device(w.K), hip.to_device(w.V)
        ctx, nq = hip.i32(w.ctx_len), hip.i32(w.draft_len)
        da.append(K, V, torch.zeros_like(ctx), ctx)
        Kn = np.zeros((w.B, w.kmax, w.Hkv, w.D), w.K.dtype)
        Vn = np.zeros_like(Kn)
        for b in range(w.B):
            L, n = int(w.ctx_len[b]), int(w.draft_len[b])
            Kn[b, :n] = w.K[b, L:L + n]
            Vn[b, :n] = w.V[b, L:L + n]
        Kn, Vn = hip.to_device(Kn), hip.to_device(Vn)
        if not fused:
            da.append(Kn, Vn, ctx, nq)
        plan = bass.alloc_plan(da.desc)
        if plan_bytes is not None:
            plan.copy_(torch.from_numpy(plan_bytes).to("cuda"))
        else:
            flags = (bass.PLAN_APPEND if fused else 0) if plan_flags is None else plan_flags
            bass.bass_attention_plan(da.desc, ctx, nq, flags, 0, plan, da.status)
        da.O.fill_(7.0)
        da.lse.fill_(7.0)
        bass.bass_verify_attention_planned(da.desc, hip.to_device(w.Q), Kn if fused else None, Vn if fused else None,
                                           da.Kc, da.Vc, plan, da.O, da.lse, da.ws, da.status)
        torch.cuda.synchronize()
        return hip.to_host(da.O), hip.to_host(da.lse), int(da.status.item()), da
    finally:
        bass.bass_set_attention_waves(0)


CASES = [
    ("bf16", 1, 128, False), ("bf16", 1, 128, True), ("bf16", 1, 64, True), ("bf16", 4, 128, False), ("bf16", 4, 128, True),
    ("int8kv", 1, 128, True), ("int8kv", 4, 128, False), ("fp32", 2, 64, True), ("fp32", 1, 32, False),
]


@pytest.mark.parametrize("dtype,g,D,fused", CASES)
@pytest.mark.parametrize("waves", [0, 64, 8192])
def test_planned_attention_matches_oracle_and_unplanned_call(hip, dtype, g, D, fused, waves):
    import paper_2404_15778_amd as bass
    gen = "bf16" if dtype == "int8kv" else dtype
    w = wl.make_attention("planned", 5, 2 * g, 2, D, gen, [37, 300, 0, 1000, 64], [4, 3, 2, 0, 6], 9, kmax=6, Lcap=1100)
    if dtype == "int8kv":
        w.dtype = "int8kv"
    O, lse, status, da = run_planned(hip, w, fused, waves)
    assert status == 0 and np.isfinite(O).all() and np.isfinite(lse).all()
    for b in range(w.B):
        assert (O[b, int(w.draft_len[b]):] == 0).all() and (lse[b, int(w.draft_len[b]):] == 0).all()
    if dtype != "int8kv":  # (INT8: the oracle comparison on represented values lives in test_gpu_kv_int8.py)
        Or, lser = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
        assert np.abs(O - Or).max() <= TOL[gen] and np.abs(lse - lser).max() <= TOL[gen]
    # the call that plans by itself, on the same caches (rows appended by now): same plan, same bits
    bass.bass_set_attention_waves(waves)
    try:
        if fused:
            Kn = np.zeros((w.B, w.kmax, w.Hkv, w.D), w.K.dtype)
            Vn = np.zeros_like(Kn)
            for b in range(w.B):
                L, n = int(w.ctx_len[b]), int(w.draft_len[b])
                Kn[b, :n], Vn[b, :n] = w.K[b, L:L + n], w.V[b, L:L + n]
            O2, lse2 = da.append_verify(hip.to_device(w.Q), hip.to_device(Kn), hip.to_device(Vn), hip.i32(w.ctx_len),
                                        hip.i32(w.draft_len))
        else:
            O2, lse2 = da.verify(hip.to_device(w.Q), hip.i32(w.ctx_len), hip.i32(w.draft_len))
        O2, lse2 = hip.to_host(O2), hip.to_host(lse2)
    finally:
        bass.bass_set_attention_waves(0)
    np.testing.assert_array_equal(O, O2)
    np.testing.assert_array_equal(lse, lse2)


def test_a_plan_serves_many_layers(hip):
    """One plan, several caches (layers) with different contents: every layer's result is its own."""
    import torch
    import paper_2404_15778_amd as bass
    ws = [wl.make_attention(f"layer{l}", 3, 4, 4, 128, "bf16", [200, 33, 700], [3, 1, 4], 20 + l, kmax=4, Lcap=720) for l in range(3)]
    desc = bass.make_desc(3, 4, 4, 4, 128, 720, "bf16", ws[0].scale)
    ctx, nq = hip.i32(ws[0].ctx_len), hip.i32(ws[0].draft_len)
    plan = bass.alloc_plan(desc)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    bass.bass_attention_plan(desc, ctx, nq, 0, 0, plan, status)
    workspace = bass.alloc_workspace(desc)
    for w in ws:
        da = hip.DeviceAttention(3, 4, 4, 4, 128, 720, "bf16", w.scale, poison=True)
        tot = hip.i32(w.ctx_len + w.draft_len)
        da.append(hip.to_device(w.K), hip.to_device(w.V), torch.zeros_like(tot), tot)
        bass.bass_verify_attention_planned(desc, hip.to_device(w.Q), None, None, da.Kc, da.Vc, plan, da.O, da.lse,
                                           workspace, status)
        torch.cuda.synchronize()
        Or, lser = oracle.verify_attention(w.Q, w.K, w.V, w.ctx_len, w.draft_len, w.scale)
        assert np.abs(hip.to_host(da.O) - Or).max() <= 2e-2 and np.abs(hip.to_host(da.lse) - lser).max() <= 2e-2
    assert int(status.item()) == 0


@pytest.mark.parametrize("what", ["append flag", "cleared buffer", "other work spread", "other batch"])
@pytest.mark.parametrize("dtype,g", [("bf16", 1), ("bf16", 4), ("fp32", 1)])
def test_foreign_plan_is_refused(hip, what, dtype, g):
    import paper_2404_15778_amd as bass
    w = wl.make_attention("refuse", 3, 2 * g, 2, 128 if dtype == "bf16" else 64, dtype, [100, 40, 7], [2, 1, 3], 4, kmax=3, Lcap=128)
    desc = bass.make_desc(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, dtype, w.scale)
    kw = {}
    if what == "append flag":
        kw["plan_flags"] = bass.PLAN_APPEND  # the launch brings no new rows
    elif what == "cleared buffer":
        kw["plan_bytes"] = np.zeros(bass.bass_attention_plan_bytes(desc), np.uint8)
    elif what == "other work spread":
        bass.bass_set_attention_waves(128)
        try:
            kw["plan_bytes"] = bass.bass_attention_plan_host(desc, w.ctx_len, w.draft_len, 0, 0)[0]
        finally:
            bass.bass_set_attention_waves(0)
    else:
        other = bass.make_desc(w.B + 1, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, dtype, w.scale)
        host = bass.bass_attention_plan_host(other, list(w.ctx_len) + [5], list(w.draft_len) + [1], 0, 0)[0]
        kw["plan_bytes"] = host[:bass.bass_attention_plan_bytes(desc)].copy()
    O, lse, status, _ = run_planned(hip, w, False, **kw)
    assert status == bass.STATUS_PLAN_MISMATCH
    assert (O == 7.0).all() and (lse == 7.0).all(), "a refused launch writes nothing"
