"""BASS-PAD vs BASS-SPLIT vs the single ragged launch (paper Section 3.2 and its ablation in Section 4.6).

The paper's kernel-level finding: padding to the longest sequence wins when the lengths of a batch
are close to each other, per-sequence launches win when they differ by a large margin.  This script
times the three launch variants of the same attention kernel on synthetic batches whose lengths are
close, moderately spread (the cfg2 recipe) and widely spread (the cfg3 recipe), bf16, 32 heads of 128.

    python -m paper_2404_15778_amd.ablation [--layers 16] [--reps 5] [--seed 0]

One JSON line per (scenario, variant): microseconds per layer call, useful KV bytes per second, and
the bytes the variant actually has to read.  "ragged", "pad" and "split" are the entry points that take the
lengths (every call plans its own work division: one small launch in front of each attention launch);
"ragged, one plan" and "pad, one plan" make the division once for all layers, as a verification step does.  Needs the GPU and the built library.
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

import paper_2404_15778_amd as bass
from paper_2404_15778_amd import harness

H, D, KMAX = 32, 128, 8


def scenarios(seed):
    rng = np.random.default_rng(seed)
    out = []
    out.append(("close: B=8, ctx U[1900,2048]", rng.integers(1900, 2049, size=8), rng.integers(1, 7, size=8)))
    out.append(("cfg2: B=8, ctx U[512,2048]", rng.integers(512, 2049, size=8), rng.integers(1, 7, size=8)))
    wide = np.rint(np.exp(rng.uniform(np.log(128), np.log(8192), size=8))).astype(np.int64)
    wide[0] = 8000  # one long prompt among short ones
    out.append(("wide: B=8, ctx logU[128,8192], one of 8000", wide, rng.integers(1, 9, size=8)))
    wide32 = np.rint(np.exp(rng.uniform(np.log(128), np.log(8192), size=32))).astype(np.int64)
    out.append(("cfg3: B=32, ctx logU[128,8192]", wide32, rng.integers(1, 9, size=32)))
    return out


def run(name, ctx_len, draft_len, layers, reps, dev):
    B = len(ctx_len)
    total = ctx_len + draft_len
    longest = int(total.max())
    Lcap = longest + 8
    desc = bass.make_desc(B, KMAX, H, H, D, Lcap, "bf16", 1.0 / np.sqrt(D))
    ctx, nq = harness.i32(ctx_len, dev), harness.i32(draft_len, dev)
    zero = torch.zeros_like(ctx)
    gen = torch.Generator(device=dev).manual_seed(1)
    fill = desc.replace(kmax=longest)
    rows = torch.randn((B, longest, H, D), device=dev, generator=gen).to(torch.bfloat16)
    slabs = []
    for _ in range(layers):
        Kc, Vc = bass.alloc_kv_cache(desc, dev, 0), bass.alloc_kv_cache(desc, dev, 0)
        bass.bass_kv_append(fill, Kc, Vc, rows, rows, zero, ctx + nq)
        slabs.append((Kc, Vc))
    del rows
    Q = torch.randn((B, KMAX, H, D), device=dev, generator=gen).to(torch.bfloat16)
    ws = bass.alloc_workspace(desc, dev)
    O = torch.empty((B, KMAX, H, D), dtype=torch.float32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    row_bytes = 2 * H * D * 2  # K and V of one token, all heads
    useful = int(total.sum()) * row_bytes
    blocks = lambda n: -(-int(n) // 32) * 32
    read = {"ragged": sum(blocks(t) for t in total) * row_bytes, "split": sum(blocks(t) for t in total) * row_bytes,
            "pad": B * blocks(longest) * row_bytes}
    # the work division of a step made once for all its layers (ragged and padded), as a verification step does
    plan_r, plan_p = bass.alloc_plan(desc, dev), bass.alloc_plan(desc, dev)
    bass.bass_attention_plan(desc, ctx, nq, 0, 0, plan_r, status)
    bass.bass_attention_plan(desc, ctx, nq, 0, longest, plan_p, status)
    read["ragged, one plan"], read["pad, one plan"] = read["ragged"], read["pad"]
    calls = {
        "ragged": lambda Kc, Vc: bass.bass_verify_attention(desc, Q, Kc, Vc, ctx, nq, O, None, ws, status),
        "pad": lambda Kc, Vc: bass.bass_verify_attention_pad(desc, Q, Kc, Vc, ctx, nq, longest, O, None, ws, status),
        "split": lambda Kc, Vc: bass.bass_verify_attention_split(desc, Q, Kc, Vc, ctx, nq, O, None, ws, status),
        "ragged, one plan": lambda Kc, Vc: bass.bass_verify_attention_planned(desc, Q, None, None, Kc, Vc, plan_r, O, None, ws, status),
        "pad, one plan": lambda Kc, Vc: bass.bass_verify_attention_planned(desc, Q, None, None, Kc, Vc, plan_p, O, None, ws, status),
    }
    ref = None
    for variant, call in calls.items():
        best = float("inf")
        for _ in range(reps + 1):  # first repetition warms up
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for Kc, Vc in slabs:
                call(Kc, Vc)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / layers)
        out = O.clone()
        if ref is None:
            ref = out
        # the variants cut the context at different points: equal up to that rounding
        assert float((out - ref).abs().max()) <= 5e-3, (name, variant)
        print(json.dumps({"scenario": name, "variant": variant, "us_per_layer": round(best, 2),
                          "useful_kv_GBps": round(useful / best / 1e3, 1), "useful_kv_bytes": useful,
                          "bytes_read": read[variant], "launches_per_layer": B if variant == "split" else 1,
                          "plan_launches_per_layer": 0 if "one plan" in variant else (B if variant == "split" else 1),
                          "ctx_min": int(ctx_len.min()), "ctx_max": int(ctx_len.max())}), flush=True)
    assert int(status.item()) == 0


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--layers", type=int, default=16, help="independent cache slabs cycled through (defeats the last-level cache)")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("the ablation needs a GPU")
    for name, ctx_len, draft_len in scenarios(args.seed):
        run(name, np.asarray(ctx_len, np.int64), np.asarray(draft_len, np.int64), args.layers, args.reps, "cuda:0")
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
