"""GPU parity of the INT8 KV cache: codes and scales bit for bit against the quantizer oracle, attention
over the INT8 cache against the fp64 attention oracle run on the represented values code * scale of the
quantized queries, keys and values."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle.kv_int8 import dequantize_rows, quantize_rows

pytestmark = pytest.mark.gpu

TOL = 2e-2   # same bar as the bf16 path: P is rounded to bf16 before the matrix cores in both


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def reference(w):
    """Oracle codes/scales of the whole logical cache and the attention over the represented values."""
    Kf, Vf = wl.bf16_bits_to_f32(w.K), wl.bf16_bits_to_f32(w.V)
    Kq, Ks = quantize_rows(Kf)
    Vq, Vs = quantize_rows(Vf)
    Qq, Qs = quantize_rows(wl.bf16_bits_to_f32(w.Q))   # the kernels quantize the query rows the same way
    O, lse = oracle.verify_attention(dequantize_rows(Qq, Qs), dequantize_rows(Kq, Ks), dequantize_rows(Vq, Vs),
                                     w.ctx_len, w.draft_len, w.scale)
    return (Kq, Ks, Vq, Vs), O, lse


def run(hip, w, two_step=True, variant="ragged", waves=0):
    """Fill an INT8 cache with the context, append the step's rows (separately or through
    bass_append_verify_attention), verify.  Returns O, lse, status, the DeviceAttention."""
    import torch
    import paper_2404_15778_amd as bass
    da = hip.DeviceAttention(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, "int8kv", w.scale, poison=True)
    ctx, nq = hip.i32(w.ctx_len), hip.i32(w.draft_len)
    da.append(hip.to_device(w.K), hip.to_device(w.V), torch.zeros_like(ctx), ctx)
    Kn = np.zeros((w.B, w.kmax, w.Hkv, w.D), np.uint16)
    Vn = np.zeros_like(Kn)
    for b in range(w.B):
        L, n = int(w.ctx_len[b]), int(w.draft_len[b])
        Kn[b, :n], Vn[b, :n] = w.K[b, L:L + n], w.V[b, L:L + n]
    Q = hip.to_device(w.Q)
    bass.bass_set_attention_waves(waves)
    try:
        if two_step:
            da.append(hip.to_device(Kn), hip.to_device(Vn), ctx, nq)
            O, lse = da.verify(Q, ctx, nq, variant=variant, padded_len=int((w.ctx_len + w.draft_len).max()))
        else:
            O, lse = da.append_verify(Q, hip.to_device(Kn), hip.to_device(Vn), ctx, nq)
        torch.cuda.synchronize()
    finally:
        bass.bass_set_attention_waves(0)
    return hip.to_host(O), hip.to_host(lse), int(da.status.item()), da


def check(hip, w, **kw):
    import torch
    (Kq, Ks, Vq, Vs), Or, lser = reference(w)
    O, lse, status, da = run(hip, w, **kw)
    assert status == 0 and np.isfinite(O).all() and np.isfinite(lse).all()
    assert np.abs(O - Or).max() <= TOL
    assert np.abs(lse - lser).max() <= TOL
    total = w.ctx_len + w.draft_len
    n = int(total.max())
    got = [hip.to_host(t) for t in da.gather_int8(hip.i32(np.zeros(w.B)), hip.i32(total), n)]
    torch.cuda.synchronize()
    for b in range(w.B):
        t = int(total[b])
        np.testing.assert_array_equal(got[0][b, :t], Kq[b, :t])       # codes bit for bit
        np.testing.assert_array_equal(got[1][b, :t], Vq[b, :t])
        np.testing.assert_array_equal(got[2][b, :t], Ks[b, :t])       # scales bit for bit
        np.testing.assert_array_equal(got[3][b, :t], Vs[b, :t])


@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("waves", [0, 64, 1024])
@pytest.mark.parametrize("two_step", [True, False])
def test_int8_cache_mha(hip, D, waves, two_step):
    # two_step False: bass_append_verify_attention quantizes and appends the step's rows inside the launch
    w = wl.make_attention("i8", 5, 8, 8, D, "bf16", [30, 63, 0, 500, 129], [6, 3, 2, 5, 0], 17, kmax=6, Lcap=520)
    check(hip, w, waves=waves, two_step=two_step)


@pytest.mark.parametrize("D,Hq,Hkv,kmax", [(128, 16, 4, 4), (128, 16, 2, 6), (64, 16, 2, 8), (128, 8, 1, 8)])
@pytest.mark.parametrize("two_step", [True, False])
def test_int8_cache_gqa_tiles(hip, D, Hq, Hkv, kmax, two_step):
    # 16, 48, 64 and 64 query rows per kv head: one to four tiles
    nq = [kmax, max(1, kmax - 2), 1]
    w = wl.make_attention("i8g", 3, Hq, Hkv, D, "bf16", [100, 37, 260], nq, 23, kmax=kmax, Lcap=300)
    check(hip, w, two_step=two_step)


@pytest.mark.parametrize("D,kmax,Hq,Hkv", [(128, 12, 4, 4), (128, 16, 2, 2), (64, 32, 2, 2), (128, 20, 2, 2), (64, 24, 4, 2)])
@pytest.mark.parametrize("waves", [0, 64])
def test_int8_fused_append_with_long_drafts(hip, D, kmax, Hq, Hkv, waves):
    # more than 8 rows of 128: several quantizing copies inside the launch; beyond kmax * D = 2048 the append
    # runs as a launch of its own
    w = wl.make_attention("i8long", 5, Hq, Hkv, D, "bf16", [100, 37, 31, 0, 60], [kmax, kmax - 3, 9, kmax, 1], 21,
                          kmax=kmax, Lcap=160)
    check(hip, w, two_step=False, waves=waves)


@pytest.mark.parametrize("ctx", [31, 32, 33, 64])
def test_int8_block_boundaries_and_the_one_call_entry_point(hip, ctx):
    w = wl.make_attention("i8e", 2, 4, 4, 128, "bf16", [ctx, ctx - 1], [1, 2], ctx, kmax=2, Lcap=96)
    check(hip, w, two_step=False)      # bass_append_verify_attention: quantizing append + attention


@pytest.mark.parametrize("variant", ["pad", "split"])
def test_int8_pad_and_split_variants(hip, variant):
    w = wl.make_attention("i8v", 4, 8, 4, 128, "bf16", [30, 200, 0, 77], [3, 2, 1, 4], 31, kmax=4, Lcap=220)
    check(hip, w, variant=variant)


def test_int8_rows_of_zeros_and_extreme_rows(hip):
    w = wl.make_attention("i8z", 2, 4, 4, 128, "bf16", [40, 20], [2, 1], 41, kmax=2, Lcap=64)
    w.K[0, 3] = 0                                                  # a key row of zeros: scale 0, codes 0
    w.V[1, 5] = 0
    w.V[0, 7] = wl.to_bf16_bits(np.full((4, 128), 3.0, np.float32))   # constant row: every code 127
    big = np.zeros((4, 128), np.float32)
    big[:, 0] = 1e4                                                # one huge element flattens the rest to 0
    w.K[1, 2] = wl.to_bf16_bits(big)
    check(hip, w)


def test_int8_query_rows_of_zeros_and_extreme_query_rows(hip):
    # the kernel quantizes each query row (token, query head) on the fly: scale 0 for a row of zeros (uniform
    # attention over the visible tokens), one dominant element, a constant row (every code 127)
    w = wl.make_attention("i8q", 2, 4, 2, 128, "bf16", [70, 33], [3, 2], 43, kmax=3, Lcap=96)
    w.Q[0, 1, 2] = 0
    one = np.zeros(128, np.float32)
    one[5] = 50.0
    w.Q[0, 0, 1] = wl.to_bf16_bits(one + 0.01)
    w.Q[1, 1, 3] = wl.to_bf16_bits(np.full(128, -0.75, np.float32))
    (_, _, _, _), Or, _ = reference(w)
    O, lse, status, _ = run(hip, w)
    assert status == 0 and np.isfinite(O).all()
    assert np.abs(O - Or).max() <= TOL
    # the row of zeros: plain mean of the represented V rows it may see
    Vq, Vs = quantize_rows(wl.bf16_bits_to_f32(w.V))
    Vhat = dequantize_rows(Vq, Vs).astype(np.float64)
    np.testing.assert_allclose(O[0, 1, 2], Vhat[0, :70 + 2, 1].mean(axis=0), atol=TOL)


def test_int8_deviation_from_the_unquantized_attention(hip):
    # What the INT8 cache costs in accuracy: the attention over it against the fp64 attention over the ORIGINAL
    # bf16 inputs (not over the represented values as in the parity checks above), at the benchmark shape, on
    # sampled rows.  N(0,1) keys and values, D = 128: a code step is about amax / 127 = 0.02 of a row's range,
    # so scores move by about 0.01 and outputs (|O| about 0.05 at these lengths) by about 1e-3.
    w = wl.config2(0)
    O, lse, status, _ = run(hip, w, two_step=False)
    assert status == 0
    rng = np.random.default_rng(8)
    worst_o = worst_l = 0.0
    rel = []
    for _ in range(32):
        b = int(rng.integers(w.B))
        i, h = int(rng.integers(w.draft_len[b])), int(rng.integers(w.Hq))
        ref, lref = oracle.verify_attention_row(w.Q, w.K, w.V, b, i, h, int(w.ctx_len[b]), w.scale)
        err = float(np.abs(O[b, i, h] - ref).max())
        worst_o, worst_l = max(worst_o, err), max(worst_l, abs(float(lse[b, i, h]) - lref))
        rel.append(float(np.linalg.norm(O[b, i, h] - ref) / np.linalg.norm(ref)))
    print(f"INT8 cache against unquantized inputs (cfg2, 32 rows): max |O - O_ref| = {worst_o:.2e}, "
          f"max |lse - lse_ref| = {worst_l:.2e}, relative L2 error of a row: median {np.median(rel):.2e}, "
          f"max {max(rel):.2e}", flush=True)
    assert worst_o <= 5e-3 and worst_l <= 2e-2 and max(rel) <= 5e-2


def test_int8_cache_is_about_half_the_bytes(hip):
    import paper_2404_15778_amd as bass
    a = bass.bass_kv_cache_bytes(bass.make_desc(8, 6, 32, 32, 128, 2056, "bf16", 1.0))
    b = bass.bass_kv_cache_bytes(bass.make_desc(8, 6, 32, 32, 128, 2056, "int8kv", 1.0))
    assert abs(b / a - (128 + 4) / 256) < 1e-9   # D + 4 bytes per token and head instead of 2 D


@pytest.mark.parametrize("two_step", [True, False])
def test_int8_cache_beyond_four_gib(hip, two_step):
    # 10 x 32 heads x 140 000 tokens of capacity: 5.9 GB per INT8 cache tensor; short contexts, every row checked
    w = wl.make_attention("i8big", 10, 32, 32, 128, "bf16", [300, 0, 17, 64, 1, 100, 33, 250, 5, 129],
                          [4, 1, 2, 3, 4, 1, 2, 3, 4, 1], 9, kmax=4, Lcap=140000)
    check(hip, w, two_step=two_step)
