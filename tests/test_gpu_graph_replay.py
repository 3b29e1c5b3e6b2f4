"""GPU: a verification step recorded into a HIP graph and replayed reproduces eager execution bit for bit,
on every replay, with eager launches on the same workspaces in between.  (The library's entry points only
enqueue kernels: no allocation, no synchronisation, no memset nodes.)"""
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


def test_a_step_replayed_as_a_graph_matches_eager(hip):
    import torch
    import paper_2404_15778_amd as bass

    # layers of four kinds: one query tile (merge inside the launch), grouped queries (tile kernel + reduction
    # launch), INT8 caches, fp32 caches; then the logits front end and the acceptance
    kinds = [("bf16", 4, 4, 128), ("bf16", 16, 2, 128), ("int8kv", 4, 4, 128), ("fp32", 4, 2, 64)]
    ctx_np, nq_np = np.array([70, 0, 333, 31]), np.array([3, 1, 4, 2])
    ctx, nq = hip.i32(ctx_np), hip.i32(nq_np)
    layers = []
    for dtype, Hq, Hkv, D in kinds:
        w = wl.make_attention("graph", 4, Hq, Hkv, D, "fp32" if dtype == "fp32" else "bf16", ctx_np, nq_np, 5, kmax=4, Lcap=400)
        da = hip.DeviceAttention(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, dtype, w.scale, poison=True)
        da.append(hip.to_device(w.K), hip.to_device(w.V), torch.zeros_like(ctx), ctx)
        Kn = np.zeros((w.B, w.kmax, w.Hkv, w.D), w.K.dtype)
        Vn = np.zeros_like(Kn)
        for b in range(w.B):
            L, n = int(ctx_np[b]), int(nq_np[b])
            Kn[b, :n], Vn[b, :n] = w.K[b, L:L + n], w.V[b, L:L + n]
        layers.append((da, hip.to_device(w.Q), hip.to_device(Kn), hip.to_device(Vn)))
    lt, ld = wl.make_logits(4, 3, 5000, 0, 3.0, 1.0)
    lt, ld = hip.to_device(lt), hip.to_device(ld)
    p, q = torch.empty_like(lt), torch.empty_like(ld)
    a = wl.make_accept("graph", 4, 3, 5000, 9, 3.0, 1.0)
    tok, ndr, u = hip.i32(a.draft_tok).reshape(4, 3), hip.i32(a.n_draft), hip.to_device(a.u)
    n_accept = torch.full((4,), -1, dtype=torch.int32, device="cuda")
    next_token = torch.full((4,), -1, dtype=torch.int32, device="cuda")
    ctx_next = torch.zeros_like(ctx)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")

    def step():
        for da, Q, Kn, Vn in layers:
            da.append_verify(Q, Kn, Vn, ctx, nq)
        da, Q, _, _ = layers[0]
        bass.bass_verify_attention_split(da.desc, Q, da.Kc, da.Vc, ctx, nq, da.O, da.lse, da.ws, da.status)
        bass.bass_warp_probs(lt, 0.2, 0.95, p, status)
        bass.bass_warp_probs(ld, 0.2, 0.95, q, status)
        ctx_next.copy_(ctx)
        bass.bass_spec_accept(p, q, tok, ndr, u, n_accept, next_token, ctx_next, status)

    def outputs():
        return [t.clone() for da, _, _, _ in layers for t in (da.O, da.lse)] + [p.clone(), q.clone(), n_accept.clone(),
                                                                                 next_token.clone(), ctx_next.clone()]

    def scribble():
        for da, _, _, _ in layers:
            da.O.fill_(7.0)
            da.lse.fill_(7.0)
        p.fill_(7.0)
        n_accept.fill_(-1)
        next_token.fill_(-1)

    step()
    torch.cuda.synchronize()
    want = outputs()
    assert int(status.item()) == 0 and all(int(da.status.item()) == 0 for da, _, _, _ in layers)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)

    other_nq = hip.i32(np.array([1, 4, 2, 0]))
    for replay in range(4):
        scribble()
        # eager launches with other lengths on the same workspaces between the replays
        for da, Q, _, _ in layers:
            da.verify(Q, ctx, other_nq)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (g, e) in enumerate(zip(outputs(), want)):
            assert torch.equal(g, e), (replay, i)
