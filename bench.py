#!/usr/bin/env python3
"""Benchmark of the BASS verification step on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input shaped like
the paper's 7.8B / batch-8 workload: for each of 32 attention layers, the append of the
step's K/V rows and the ragged verify attention (bass_append_verify_attention, one launch;
B=8, Hq=Hkv=32, D=128, bf16, ctx ~ U{512..2048}, drafts ~ U{1..6}), then one
bass_spec_accept over a 50k vocabulary (k=5).  Every layer has its own cache slab, so the KV reads of a step (~5 GB) cannot be
served from the 256 MB last-level cache.

Prints ONE JSON line.  `value` = algorithmic KV bytes of the step (every valid K and V row
once per layer) / wall time of the step, inputs resident in HBM.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=32, help="attention layers (independent cache slabs) per step")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0, help="override the attention work spread (0 = library default)")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from Python instead of replaying a HIP graph")
    ap.add_argument("--separate-append", action="store_true", help="bass_kv_append + bass_verify_attention as two launches")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run four 1 GiB device-to-device copies (a kernel of known traffic for counter scaling)")
    ap.add_argument("--kv-int8", action="store_true",
                    help="INT8 KV caches with per-token, per-head scales (not the headline configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def measured_traffic():
    """HBM bytes per attention launch from the rocprofv3 --pmc runs recorded under profiles/ (FETCH_SIZE
    and WRITE_SIZE, each scaled by a 1 GiB copy); None if that summary is not there."""
    path = os.path.join(ROOT, "profiles", "verify_attn_bf16_cfg2_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives are part of it); "
              f"--gpus {args.gpus} is not supported, use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    import paper_2404_15778_amd as bass
    from paper_2404_15778_amd import harness

    if not os.path.exists(bass.LIB_PATH):
        from paper_2404_15778_amd import build
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.waves:
        bass.bass_set_attention_waves(args.waves)

    # ---- synthetic inputs, resident in HBM ------------------------------------------------------
    w = wl.config2(args.seed, tensors=False)  # lengths only; tensors are drawn on the GPU below
    NL = args.layers
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234 + args.seed)
    desc = bass.make_desc(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, "int8kv" if args.kv_int8 else "bf16", w.scale)
    ctx, nq = harness.i32(w.ctx_len, dev), harness.i32(w.draft_len, dev)
    zero = torch.zeros_like(ctx)
    Lmax = int(w.ctx_len.max())
    fill_desc = desc.replace(kmax=Lmax)
    layers = []
    for _ in range(NL):
        Kc, Vc = bass.alloc_kv_cache(desc, dev, 0), bass.alloc_kv_cache(desc, dev, 0)
        Kctx = torch.randn((w.B, Lmax, w.Hkv, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        Vctx = torch.randn((w.B, Lmax, w.Hkv, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        bass.bass_kv_append(fill_desc, Kc, Vc, Kctx, Vctx, zero, ctx)  # the cached context
        del Kctx, Vctx
        shape_kv = (w.B, w.kmax, w.Hkv, w.D)
        layers.append(dict(
            Kc=Kc, Vc=Vc,
            Q=torch.randn((w.B, w.kmax, w.Hq, w.D), generator=gen, device=dev).to(torch.bfloat16),
            Kn=torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16),
            Vn=torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)))
    ws = bass.alloc_workspace(desc, dev)
    O = torch.empty((w.B, w.kmax, w.Hq, w.D), dtype=torch.float32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    acc = wl.config5_accept(args.seed)
    p, q, u = (harness.to_device(x, dev) for x in (acc.p, acc.q, acc.u))
    tok, ndr = harness.i32(acc.draft_tok, dev), harness.i32(acc.n_draft, dev)
    n_accept = torch.zeros(acc.B, dtype=torch.int32, device=dev)
    next_token = torch.zeros(acc.B, dtype=torch.int32, device=dev)
    # the length advance of the acceptance step runs on a scratch copy so that every timed step sees
    # the same ragged lengths
    ctx_scratch = ctx.clone()
    torch.cuda.synchronize()

    def step(events=None):
        # events (second pass only): [0] before the first attention launch, [1] after the last one,
        # [2] after the acceptance launch -- all on the stream the kernels are launched on
        if events is not None:
            events[0].record()
        for l in layers:
            if args.separate_append:
                bass.bass_kv_append(desc, l["Kc"], l["Vc"], l["Kn"], l["Vn"], ctx, nq, status)
                bass.bass_verify_attention(desc, l["Q"], l["Kc"], l["Vc"], ctx, nq, O, None, ws, status)
            else:  # append of the step's K/V rows fused into the attention launch
                bass.bass_append_verify_attention(desc, l["Q"], l["Kn"], l["Vn"], l["Kc"], l["Vc"], ctx, nq, O, None,
                                                  ws, status)
        if events is not None:
            events[1].record()
        bass.bass_spec_accept(p, q, tok, ndr, u, n_accept, next_token, ctx_scratch, status)
        if events is not None:
            events[2].record()

    # One step is 2 * layers + 1 launches of 3-40 us each; a serving loop replays them as a HIP graph so
    # that the CPU's launch cost does not pace the GPU.  (The library itself records no memset nodes.)
    run_step = step
    if not args.no_graph:
        step()  # eager reference for the replay check below
        torch.cuda.synchronize()
        O_ref, nacc_ref, tok_ref = O.clone(), n_accept.clone(), next_token.clone()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):  # every replay must reproduce the eager result bit for bit
            O.zero_()
            n_accept.fill_(-1)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(O, O_ref) and torch.equal(n_accept, nacc_ref) and torch.equal(next_token, tok_ref), \
                "graph replay differs from eager execution"
        run_step = graph.replay

    if args.calibration_copy:  # 1 GiB read + 1 GiB written per copy, by a plain elementwise copy kernel
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(status.item()) == 0, "device status word is not clean"
    ms_per_step = 1e3 * wall / args.steps

    # ---- second pass: HIP events around the step's run of attention launches and the acceptance ---
    # (eager launches on the current stream; the NL attention kernels run back to back, so
    # elapsed / NL is the average duration of one launch including the hand-over to the next)
    attn_ms, accept_ms = [], []
    for _ in range(args.steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        step(ev)
        torch.cuda.synchronize()
        attn_ms.append(ev[0].elapsed_time(ev[1]) / NL)
        accept_ms.append(ev[1].elapsed_time(ev[2]))
    attn_us = 1e3 * float(np.mean(attn_ms))
    accept_us = 1e3 * float(np.mean(accept_ms))

    # ---- side measurement (not part of the timed step): the logits front end that would make p and q ---
    # temperature 0.2, top-p 0.95 as in the paper's experiments; B*(k+1) main rows and B*k draft rows
    lt, ld = wl.make_logits(acc.B, acc.kmax, acc.V, args.seed, 3.0, 1.0)
    lt, ld = harness.to_device(lt, dev), harness.to_device(ld, dev)
    pw, qw = torch.empty_like(lt), torch.empty_like(ld)
    warp_ms = []
    reps = 10  # pairs per timed run, so that the launches queue up behind each other on the GPU
    for _ in range(2):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            bass.bass_warp_probs(lt, 0.2, 0.95, pw, status)
            bass.bass_warp_probs(ld, 0.2, 0.95, qw, status)
        e1.record()
        torch.cuda.synchronize()
        warp_ms.append(e0.elapsed_time(e1) / reps)
    warp_us = 1e3 * warp_ms[-1]
    del lt, ld, pw, qw

    kv_bytes = w.kv_bytes  # per layer
    if args.kv_int8:  # D codes + one fp32 scale per token and head instead of 2 D bytes
        kv_bytes = kv_bytes * (w.D + 4) // (2 * w.D)
    step_bytes = kv_bytes * NL
    value = step_bytes / (wall / args.steps) / 1e9
    n_acc_host = harness.to_host(n_accept)
    result = {
        "metric": "verify_attention_kv_read_GBps",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 (INT8 KV cache)" if args.kv_int8 else "bf16",
        "data": "synthetic",
        "config": {
            "workload": "cfg5 full verification step = cfg2 ragged MHA verify attention (B=8, Hq=Hkv=32, D=128, "
                        + ("bf16 Q, INT8 KV cache, " if args.kv_int8 else "bf16, ") +
                        f"ctx U[512,2048], drafts U[1,6]) x {NL} layers + spec_accept (V=50000, k=5)",
            "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "layers": NL, "seed": args.seed,
            "ctx_len": w.ctx_len.tolist(), "draft_len": w.draft_len.tolist(),
            "kv_bytes_per_layer": kv_bytes, "attention_waves": args.waves if args.waves else ("library default (1024)" if args.kv_int8 else bass.bass_set_attention_waves(0)),
            "launch": "eager" if args.no_graph else "hip_graph_replay",
            "append": "separate launch" if args.separate_append else "fused into the attention launch",
        },
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "verified_tokens_per_s": round(w.verified_tokens / (wall / args.steps), 1),
        "emitted_tokens_per_s": round(float((n_acc_host + 1).sum()) / (wall / args.steps), 1),
        "attention_call_us": round(attn_us, 2),
        "spec_accept_us": round(accept_us, 2),
        "logit_warp_us": round(warp_us, 2),
        "roofline": {
            "kernel": ("verify_attn_bf16<128,1,int8> (quantizing append + streaming + split-context reduction, one launch)"
                       if args.kv_int8 else
                       "verify_attn_bf16<128,1> (append + streaming + split-context reduction, one launch)"),
            "bound": "hbm",
            "achieved": round(kv_bytes / (attn_us * 1e-6) / 1e9, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(kv_bytes / (attn_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
            "traffic": None if args.kv_int8 else measured_traffic(),
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        wt = wl.config2(args.seed)  # one layer's tensors on the host
        reps_done, t_cpu = 0, 0.0
        layer_t = None
        while t_cpu < args.cpu_seconds and reps_done < 16 * NL:
            t1 = time.perf_counter()
            oracle.verify_attention(wt.Q, wt.K, wt.V, wt.ctx_len, wt.draft_len, wt.scale)
            layer_t = time.perf_counter() - t1
            t_cpu += layer_t
            reps_done += 1
        t1 = time.perf_counter()
        oracle.spec_accept(acc.p, acc.q, acc.draft_tok, acc.n_draft, acc.u)
        t_acc = time.perf_counter() - t1
        result["cpu_baseline"] = {
            "value": round(kv_bytes * reps_done / (t_cpu + t_acc * reps_done / NL) / 1e9, 3),
            "unit": "GB/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{reps_done} layer passes of cfg2 attention (one layer's tensors, every output row; a step has {NL}) "
                      f"+ the matching share of one V=50000 acceptance; {t_cpu:.1f} s of wall time",
            "attention_layer_ms": round(1e3 * t_cpu / reps_done, 2),
            "spec_accept_ms": round(1e3 * t_acc, 3),
        }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
