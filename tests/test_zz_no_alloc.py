"""GPU: bass_verify_attention_noalloc (the entry point for callers that cannot allocate; its scratch is a static
device array inside the library) against bass_verify_attention on the same inputs: two calls in a row, the
second with a smaller input, then a larger one again; bit for bit (both run the same plan and the same
kernels; only where the partial results live differs).  Shapes beyond the static array are refused."""
import ctypes

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2404_15778_amd import harness
    return harness


def both(hip, w):
    """(O, lse) of bass_verify_attention and of bass_verify_attention_noalloc on the same caches."""
    import torch
    import paper_2404_15778_amd as bass
    O1, lse1, status, da = hip.run_attention_workload(w, poison=True)
    assert status == 0
    Q, ctx, nq = hip.to_device(w.Q), hip.i32(w.ctx_len), hip.i32(w.draft_len)
    O2 = torch.full_like(da.O, float("nan"))
    lse2 = torch.full_like(da.lse, float("nan"))
    bass.bass_verify_attention_noalloc(da.desc, Q, da.Kc, da.Vc, ctx, nq, O2, lse2, da.status)
    torch.cuda.synchronize()
    assert int(da.status.item()) == 0
    return (O1, lse1), (hip.to_host(O2), hip.to_host(lse2))


@pytest.mark.parametrize("dtype,g,D", [("bf16", 1, 128), ("bf16", 4, 128), ("fp32", 2, 64)])
def test_two_calls_in_a_row_second_one_smaller(hip, dtype, g, D):
    big = wl.make_attention("noalloc_big", 6, 4 * g, 4, D, dtype, [700, 90, 333, 1500, 0, 64], [3, 6, 1, 4, 2, 0], 31, kmax=6, Lcap=1600)
    small = wl.make_attention("noalloc_small", 2, 2 * g, 2, D, dtype, [40, 130], [2, 1], 32, kmax=2, Lcap=160)
    for w in (big, small, big):
        (O1, lse1), (O2, lse2) = both(hip, w)
        assert np.isfinite(O2).all() and np.isfinite(lse2).all()
        np.testing.assert_array_equal(O1, O2)
        np.testing.assert_array_equal(lse1, lse2)


def test_benchmark_shape_fits_and_oversized_shape_is_refused(hip):
    import paper_2404_15778_amd as bass
    w = wl.config2(0)
    (O1, lse1), (O2, lse2) = both(hip, w)
    np.testing.assert_array_equal(O1, O2)
    np.testing.assert_array_equal(lse1, lse2)
    # 2048 sequences x 32 heads x 16 rows of partial results per unit: far beyond 16 MiB
    d = bass.make_desc(2048, 16, 32, 32, 128, 64, "bf16", 0.1)
    one = ctypes.c_void_p(256)  # never dereferenced: the size check fails before any launch
    rc = bass.lib().bass_verify_attention_noalloc(ctypes.byref(d), one, one, one, one, one, one, None, None, None)
    assert rc == bass.ERR_WORKSPACE_TOO_SMALL
