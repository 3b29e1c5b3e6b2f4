"""Calls of the library on the synthetic configurations, for timing under a profiler.

    python -m paper_2404_15778_amd.kernel_times attention --cfg 2 [--dtype bf16|int8kv] [--waves 0,1024]
                                                           [--slabs 16] [--fused] [--planned] [--reps 3]
    python -m paper_2404_15778_amd.kernel_times logits [--reps 5] [--temperature T --top-p P]
    python -m paper_2404_15778_amd.kernel_times summarize <kernel_trace.csv>

`attention` fills --slabs cache slabs of one attention configuration (workloads.config2/3/4, seed 0) with
bass_kv_append, so that consecutive calls cannot be served by the last-level cache, and calls
bass_verify_attention (or, with --fused, bass_append_verify_attention; with --planned, one
bass_attention_plan per sweep over the slabs and bass_verify_attention_planned per slab, as a verification
step does) over them --reps times per wavefront setting (0 = the library's default).  It prints the time per call seen by HIP events, which
includes the hand-over between launches; kernel durations come from running the same command under
`rocprofv3 --kernel-trace --output-format csv -d <dir> -o <name> -- python3 <repo>/paper_2404_15778_amd/kernel_times.py attention ...`
and passing `<dir>/<name>_kernel_trace.csv` to `summarize` (average, median and minimum of End - Start per
kernel, grid size and register count).

`logits` calls bass_warp_probs on the rows of one verification step (workloads.make_logits: 8 x 6 main-model
and 8 x 5 draft-model rows of 50 000 logits) at three settings: the paper's temperature 0.2 / top-p 0.95,
flat rows (1.0 / 0.9) and the plain softmax (1.0 / 1.0) -- or at the one setting given; then, at the first
setting, bass_spec_accept on the rows made and bass_warp_accept on the logits (drafts: the draft model's
most likely tokens).

Needs the GPU and the built library (except `summarize`).
"""
from __future__ import annotations

import argparse
import collections
import csv
import os
import sys

# the repository root (workloads.py, this package) must be importable when the file is run by path, as it
# is under a profiler started from another directory
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def attention(args):
    import torch

    import paper_2404_15778_amd as bass
    import workloads as wl
    from paper_2404_15778_amd import harness

    w = {2: wl.config2, 3: wl.config3, 4: wl.config4}[args.cfg](0, tensors=False)
    dev = "cuda:0"
    desc = bass.make_desc(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, args.dtype, w.scale)
    ctx, nq = harness.i32(w.ctx_len, dev), harness.i32(w.draft_len, dev)
    zero = torch.zeros_like(ctx)
    longest = int((w.ctx_len + w.draft_len).max())
    fill = desc.replace(kmax=longest)
    gen = torch.Generator(device=dev).manual_seed(1)
    K = torch.randn((w.B, longest, w.Hkv, w.D), device=dev, generator=gen).to(torch.bfloat16)
    V = torch.randn((w.B, longest, w.Hkv, w.D), device=dev, generator=gen).to(torch.bfloat16)
    slabs = []
    for _ in range(args.slabs):
        Kc, Vc = bass.alloc_kv_cache(desc, dev, 0), bass.alloc_kv_cache(desc, dev, 0)
        bass.bass_kv_append(fill, Kc, Vc, K, V, zero, ctx + nq)
        slabs.append((Kc, Vc))
    del K, V
    Q = torch.randn((w.B, w.kmax, w.Hq, w.D), device=dev, generator=gen).to(torch.bfloat16)
    Kn = torch.randn((w.B, w.kmax, w.Hkv, w.D), device=dev, generator=gen).to(torch.bfloat16)
    Vn = torch.randn((w.B, w.kmax, w.Hkv, w.D), device=dev, generator=gen).to(torch.bfloat16)
    ws = bass.alloc_workspace(desc, dev)
    O = torch.empty((w.B, w.kmax, w.Hq, w.D), dtype=torch.float32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    plan = bass.alloc_plan(desc, dev)
    print(f"cfg{args.cfg} {args.dtype}: kv_bytes (bf16-equivalent) {w.kv_bytes}", flush=True)
    try:
        for waves in args.waves:
            in_effect = bass.bass_set_attention_waves(waves)
            for _ in range(args.reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                if args.planned:
                    bass.bass_attention_plan(desc, ctx, nq, bass.PLAN_APPEND if args.fused else 0, 0, plan, status)
                e0.record()
                for Kc, Vc in slabs:
                    if args.planned:
                        bass.bass_verify_attention_planned(desc, Q, Kn if args.fused else None, Vn if args.fused else None,
                                                           Kc, Vc, plan, O, None, ws, status)
                    elif args.fused:
                        bass.bass_append_verify_attention(desc, Q, Kn, Vn, Kc, Vc, ctx, nq, O, None, ws, status)
                    else:
                        bass.bass_verify_attention(desc, Q, Kc, Vc, ctx, nq, O, None, ws, status)
                e1.record()
                torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / len(slabs)
            label = waves if waves else f"default ({in_effect} for one-tile bf16 shapes)"
            print(f"wavefronts {label}: {us:.2f} us per call, {w.kv_bytes / us / 1e3:.0f} GB/s of bf16-equivalent KV bytes",
                  flush=True)
    finally:
        bass.bass_set_attention_waves(0)
    assert int(status.item()) == 0


def logits(args):
    import torch

    import paper_2404_15778_amd as bass
    import workloads as wl
    from paper_2404_15778_amd import harness

    lt, ld = wl.make_logits(8, 5, 50000, 0, 3.0, 1.0)
    lt, ld = harness.to_device(lt), harness.to_device(ld)
    pw, qw = torch.empty_like(lt), torch.empty_like(ld)
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    settings = ((0.2, 0.95), (1.0, 0.9), (1.0, 1.0)) if args.temperature is None else ((args.temperature, args.top_p),)
    for T, top_p in settings:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(args.reps + 1):  # the first pair warms up
            if i == 1:
                e0.record()
            bass.bass_warp_probs(lt, T, top_p, pw, status)
            bass.bass_warp_probs(ld, T, top_p, qw, status)
        e1.record()
        torch.cuda.synchronize()
        print(f"T={T} top_p={top_p}: {e0.elapsed_time(e1) * 1e3 / args.reps:.1f} us per pair of launches (48 + 40 rows)",
              flush=True)
    # the acceptance on the rows made last, and the call that goes from the logits to the acceptance without them
    T, top_p = settings[0]
    tok = lt[:, :5].argmax(dim=-1).to(torch.int32).contiguous()
    nd = torch.full((8,), 5, dtype=torch.int32, device="cuda:0")
    u = torch.rand((8, 6), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(3))
    n_acc, nxt = torch.zeros_like(nd), torch.zeros_like(nd)
    ws = torch.empty(bass.bass_warp_accept_workspace_bytes(8, 5, 50000), dtype=torch.uint8, device="cuda:0")
    bass.bass_warp_probs(lt, T, top_p, pw, status)
    bass.bass_warp_probs(ld, T, top_p, qw, status)
    for _ in range(args.reps + 1):
        bass.bass_spec_accept(pw, qw, tok, nd, u, n_acc, nxt, None, status)
    two = (n_acc.clone(), nxt.clone())
    for _ in range(args.reps + 1):
        bass.bass_warp_accept(lt, ld, T, top_p, tok, nd, u, n_acc, nxt, ws, None, status)
    torch.cuda.synchronize()
    assert torch.equal(n_acc, two[0]) and torch.equal(nxt, two[1])
    print(f"bass_warp_accept at T={T} top_p={top_p}: accepted {n_acc.tolist()}, same as the two calls", flush=True)


def summarize(args):
    rows = list(csv.DictReader(open(args.trace)))
    agg = collections.defaultdict(list)
    for r in rows:
        name = r["Kernel_Name"]
        if "bass::" not in name and "bass" not in name:
            continue
        key = (name.split("(")[0].replace("void ", ""), r.get("Grid_Size_X") or r.get("Grid_Size"),
               r.get("VGPR_Count") or r.get("Arch_VGPR_Count"))
        agg[key].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    for (name, grid, vgpr), v in agg.items():
        v = sorted(v)
        print(f"{name}  grid {grid}  vgpr {vgpr}:  n={len(v)}  avg {sum(v) / len(v) / 1e3:.2f} us  "
              f"median {v[len(v) // 2] / 1e3:.2f} us  min {v[0] / 1e3:.2f} us")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("attention")
    a.add_argument("--cfg", type=int, choices=(2, 3, 4), default=2)
    a.add_argument("--dtype", choices=("bf16", "int8kv"), default="bf16")
    a.add_argument("--waves", type=lambda s: [int(x) for x in s.split(",")], default=[0])
    a.add_argument("--slabs", type=int, default=16)
    a.add_argument("--reps", type=int, default=3)
    a.add_argument("--fused", action="store_true")
    a.add_argument("--planned", action="store_true")
    a.set_defaults(run=attention)
    g = sub.add_parser("logits")
    g.add_argument("--reps", type=int, default=5)
    g.add_argument("--temperature", type=float, default=None)
    g.add_argument("--top-p", type=float, default=0.95)
    g.set_defaults(run=logits)
    s = sub.add_parser("summarize")
    s.add_argument("trace")
    s.set_defaults(run=summarize)
    args = ap.parse_args()
    if args.what != "summarize":
        import torch
        if not torch.cuda.is_available():
            raise SystemExit("needs a GPU")
    args.run(args)


if __name__ == "__main__":
    main()
