#!/usr/bin/env python3
"""Benchmark of the BASS verification step on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input shaped like the paper's
7.8B / batch-8 workload: one bass_attention_plan (all layers of a step see the same lengths), then for
each of 32 attention layers the append of the step's K/V rows and the ragged verify attention
(bass_verify_attention_planned, one launch; B=8, Hq=Hkv=32, D=128, bf16, ctx ~ U{512..2048}, drafts ~
U{1..6}), then one bass_spec_accept over a 50k vocabulary (k=5).  Every layer has its own cache slab, so
the KV reads of a step (~5 GB) cannot be served from the 256 MB last-level cache.

Prints ONE JSON line.  `value` = algorithmic KV bytes of the step (every valid K and V row once per
layer) / wall time of the step, inputs resident in HBM, for seed 0 of the input recipe.  The same line
carries the per-launch roofline figures of seeds 0-2, the plain streaming-read ceiling measured on the
same cache slabs, the attention launches of the other benchmark configurations (cfg3: 32 long ragged
sequences, cfg4: grouped-query heads), and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
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
    ap.add_argument("--seed", type=int, default=0, help="seed of the headline run (`value`)")
    ap.add_argument("--waves", type=int, default=0, help="override the attention work spread (0 = library default)")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from Python instead of replaying a HIP graph")
    ap.add_argument("--unplanned", action="store_true",
                    help="bass_append_verify_attention per layer (a plan inside every call) instead of one plan per step")
    ap.add_argument("--separate-append", action="store_true", help="bass_kv_append + bass_verify_attention as two launches")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run four 1 GiB device-to-device copies (a kernel of known traffic for counter scaling)")
    ap.add_argument("--kv-int8", action="store_true",
                    help="INT8 KV caches with per-token, per-head scales (not the headline configuration)")
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the other seeds, the other configurations and the side measurements (profiling runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def measured_traffic(version):
    """HBM bytes per attention launch from the rocprofv3 --pmc runs recorded under profiles/ (FETCH_SIZE
    and WRITE_SIZE, each scaled by a 1 GiB copy), if that summary was made with this library version."""
    path = os.path.join(ROOT, "profiles", "verify_attn_bf16_cfg2_hbm_traffic.txt")
    traffic, at_version = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
            if line.startswith("bass_version:"):
                at_version = int(line.split(":")[1])
    except (OSError, ValueError):
        return None
    return traffic if at_version == version else None


class Step:
    """Device state of one verification step of `NL` layers for a fixed shape; lengths and contents can be
    redrawn in place (the graph of the step reads the lengths from device memory)."""

    def __init__(self, args, bass, harness, torch, w, NL, dev, with_accept, acc=None):
        self.args, self.bass, self.harness, self.torch, self.w, self.NL, self.dev = args, bass, harness, torch, w, NL, dev
        dtype = "int8kv" if args.kv_int8 else "bf16"
        self.desc = bass.make_desc(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, dtype, w.scale)
        self.ctx, self.nq = harness.i32(w.ctx_len, dev), harness.i32(w.draft_len, dev)
        self.layers = []
        for _ in range(NL):
            self.layers.append(dict(Kc=bass.alloc_kv_cache(self.desc, dev, 0), Vc=bass.alloc_kv_cache(self.desc, dev, 0),
                                    Q=None, Kn=None, Vn=None))
        self.ws = bass.alloc_workspace(self.desc, dev)
        self.plan = bass.alloc_plan(self.desc, dev)
        self.O = torch.empty((w.B, w.kmax, w.Hq, w.D), dtype=torch.float32, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        self.with_accept = with_accept
        if with_accept:
            self.p, self.q, self.u = (harness.to_device(x, dev) for x in (acc.p, acc.q, acc.u))
            self.tok, self.ndr = harness.i32(acc.draft_tok, dev), harness.i32(acc.n_draft, dev)
            self.n_accept = torch.zeros(acc.B, dtype=torch.int32, device=dev)
            self.next_token = torch.zeros(acc.B, dtype=torch.int32, device=dev)
            # the length advance of the acceptance step runs on a scratch copy so that every timed step
            # sees the same ragged lengths
            self.ctx_scratch = self.ctx.clone()
        self.graph = None

    def fill(self, w, seed, acc=None):
        """Draws the cached context and the step's Q / new rows on the GPU (seeded) for the lengths of `w`."""
        torch, bass, dev = self.torch, self.bass, self.dev
        self.w = w
        self.ctx.copy_(self.harness.i32(w.ctx_len, dev))
        self.nq.copy_(self.harness.i32(w.draft_len, dev))
        gen = torch.Generator(device=dev)
        gen.manual_seed(1234 + seed)
        zero = torch.zeros_like(self.ctx)
        for l in self.layers:
            for b in range(w.B):  # one sequence at a time: the fp32 draw of a whole long batch would not be small
                L = int(w.ctx_len[b])
                if L == 0:
                    continue
                d1 = self.desc.replace(B=1, kmax=L)
                Kctx = torch.randn((1, L, w.Hkv, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
                Vctx = torch.randn((1, L, w.Hkv, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
                per_seq = bass.bass_kv_cache_bytes(self.desc) // w.B
                bass.bass_kv_append(d1, l["Kc"][b * per_seq:(b + 1) * per_seq], l["Vc"][b * per_seq:(b + 1) * per_seq],
                                    Kctx, Vctx, zero[:1], self.ctx[b:b + 1])
            shape_kv = (w.B, w.kmax, w.Hkv, w.D)
            l["Q"] = torch.randn((w.B, w.kmax, w.Hq, w.D), generator=gen, device=dev).to(torch.bfloat16)
            l["Kn"] = torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)
            l["Vn"] = torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)
        if self.with_accept and acc is not None:
            for dst, src in ((self.p, acc.p), (self.q, acc.q), (self.u, acc.u)):
                dst.copy_(self.harness.to_device(src, dev))
            self.tok.copy_(self.harness.i32(acc.draft_tok, dev).reshape(self.tok.shape))
            self.ndr.copy_(self.harness.i32(acc.n_draft, dev))
        if self.with_accept:
            self.ctx_scratch.copy_(self.ctx)
        torch.cuda.synchronize()

    def run(self, events=None):
        """Enqueues one step.  events (optional): [0] before the plan, [1] before the first attention launch,
        [2] after the last one, [3] after the acceptance launch -- on the stream the kernels are launched on."""
        args, bass = self.args, self.bass
        rec = (lambda i: events[i].record()) if events is not None else (lambda i: None)
        rec(0)
        planned = not (args.unplanned or args.separate_append)
        if planned:
            self.launch_plan()
        rec(1)
        for l in self.layers:
            if args.separate_append:
                bass.bass_kv_append(self.desc, l["Kc"], l["Vc"], l["Kn"], l["Vn"], self.ctx, self.nq, self.status)
                bass.bass_verify_attention(self.desc, l["Q"], l["Kc"], l["Vc"], self.ctx, self.nq, self.O, None, self.ws,
                                           self.status)
            elif args.unplanned:
                bass.bass_append_verify_attention(self.desc, l["Q"], l["Kn"], l["Vn"], l["Kc"], l["Vc"], self.ctx, self.nq,
                                                  self.O, None, self.ws, self.status)
            else:  # append of the step's K/V rows fused into the attention launch, work division from the step's plan
                bass.bass_verify_attention_planned(self.desc, l["Q"], l["Kn"], l["Vn"], l["Kc"], l["Vc"], self.plan, self.O,
                                                   None, self.ws, self.status)
        rec(2)
        if self.with_accept:
            self.launch_accept()
        rec(3)

    def capture(self):
        """The step as a HIP graph (the library records no memset nodes); every replay is checked against
        eager execution."""
        torch = self.torch
        self.run()
        torch.cuda.synchronize()
        O_ref = self.O.clone()
        refs = (self.n_accept.clone(), self.next_token.clone()) if self.with_accept else None
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                self.run()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):
            self.O.zero_()
            if self.with_accept:
                self.n_accept.fill_(-1)
            graph.replay()
            torch.cuda.synchronize()
            same = torch.equal(self.O, O_ref)
            if self.with_accept:
                same = same and torch.equal(self.n_accept, refs[0]) and torch.equal(self.next_token, refs[1])
            assert same, "graph replay differs from eager execution"
        self.graph = graph

    def time_steps(self, steps, warmup):
        """Wall time of `steps` steps after `warmup` untimed ones, synchronised on both sides; seconds."""
        torch = self.torch
        go = self.graph.replay if self.graph is not None else self.run
        for _ in range(warmup):
            go()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            go()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        assert int(self.status.item()) == 0, "device status word is not clean"
        return wall

    def launch_times(self, sweeps):
        """HIP events around the step's run of attention launches, the plan and the acceptance (eager launches
        on the current stream; the NL attention kernels run back to back, so elapsed / NL is the average
        duration of one launch including the hand-over to the next).  Returns microseconds."""
        import numpy as np
        torch = self.torch
        plan_ms, attn_ms, accept_ms = [], [], []
        self.run()  # untimed: the first eager step after a replay
        for _ in range(sweeps):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            self.run(ev)
            torch.cuda.synchronize()
            plan_ms.append(ev[0].elapsed_time(ev[1]))
            attn_ms.append(ev[1].elapsed_time(ev[2]) / self.NL)
            accept_ms.append(ev[2].elapsed_time(ev[3]))
        # a single launch between two events mostly shows the events: the plan and the acceptance are timed
        # as runs of back-to-back launches instead (both are idempotent on these inputs)
        planned = not (self.args.unplanned or self.args.separate_append)
        plan_us = self.repeated(self.launch_plan) if planned else 1e3 * float(np.mean(plan_ms))
        accept_us = self.repeated(self.launch_accept) if self.with_accept else 1e3 * float(np.mean(accept_ms))
        return plan_us, 1e3 * float(np.mean(attn_ms)), accept_us

    def repeated(self, launch, n=16, sweeps=3):
        """Microseconds per launch of n back-to-back launches (HIP events around the run), last of `sweeps` runs."""
        torch = self.torch
        for _ in range(sweeps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                launch()
            e1.record()
            torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / n

    def launch_plan(self):
        self.bass.bass_attention_plan(self.desc, self.ctx, self.nq, self.bass.PLAN_APPEND, 0, self.plan, self.status)

    def launch_accept(self):
        self.bass.bass_spec_accept(self.p, self.q, self.tok, self.ndr, self.u, self.n_accept, self.next_token,
                                   self.ctx_scratch, self.status)

    def kv_bytes(self):
        kv = self.w.kv_bytes  # per layer
        if self.args.kv_int8:  # D codes + one fp32 scale per token and head instead of 2 D bytes
            kv = kv * (self.w.D + 4) // (2 * self.w.D)
        return kv

    def ceiling(self, sweeps, waves):
        """Plain streaming read of as many bytes as one attention launch reads, from every layer's K and V
        slabs in turn (bass_bench_stream_read).  Returns (microseconds per launch, bytes per launch)."""
        import numpy as np
        torch, bass = self.torch, self.bass
        each = self.kv_bytes() // 2
        sink = torch.zeros(8192, dtype=torch.int32, device=self.dev)
        ms, nbytes = [], 0
        for it in range(sweeps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for l in self.layers:
                nbytes = bass.bass_bench_stream_read(l["Kc"], l["Vc"], each, waves, sink)
            e1.record()
            torch.cuda.synchronize()
            if it:
                ms.append(e0.elapsed_time(e1) / self.NL)
        return 1e3 * float(np.mean(ms)), nbytes


def oracle_baseline(args, wl, w_host, acc, kv_bytes, NL):
    """The CPU oracle as it stands on a bounded sample of the workload: repeated passes over one layer's
    tensors with all host threads until the time budget is used, best of 5 passes with all threads and with
    one, one acceptance."""
    import oracle
    try:
        affinity = len(os.sched_getaffinity(0))
    except AttributeError:
        affinity = os.cpu_count()
    threads = oracle.num_threads()

    def one_pass():
        t1 = time.perf_counter()
        oracle.verify_attention(w_host.Q, w_host.K, w_host.V, w_host.ctx_len, w_host.draft_len, w_host.scale)
        return time.perf_counter() - t1

    reps_done, t_cpu, best_all = 0, 0.0, float("inf")
    while (t_cpu < args.cpu_seconds and reps_done < 16 * NL) or reps_done < 5:
        t = one_pass()
        best_all = min(best_all, t)
        t_cpu += t
        reps_done += 1
    best_one = None
    try:  # the same passes on one thread (OpenMP's own switch; the oracle is not touched)
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        best_one = min(one_pass() for _ in range(5 if best_all < 0.5 else 2))
        gomp.omp_set_num_threads(threads)
    except OSError:
        pass
    t1 = time.perf_counter()
    oracle.spec_accept(acc.p, acc.q, acc.draft_tok, acc.n_draft, acc.u)
    t_acc = time.perf_counter() - t1
    out = {
        "value": round(kv_bytes * reps_done / (t_cpu + t_acc * reps_done / NL) / 1e9, 3),
        "unit": "GB/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"{reps_done} layer passes of cfg2 attention (one layer's tensors, every output row; a step has {NL}) "
                  f"+ the matching share of one V=50000 acceptance; {t_cpu:.1f} s of wall time with {threads} threads, "
                  f"then passes on one thread",
        "affinity_cores": affinity,
        "attention_layer_ms": round(1e3 * t_cpu / reps_done, 2),
        "attention_layer_ms_best_all_threads": round(1e3 * best_all, 2),
        "attention_layer_ms_best_one_thread": None if best_one is None else round(1e3 * best_one, 2),
        "value_one_thread": None if best_one is None else round(kv_bytes / best_one / 1e9, 3),
        "spec_accept_ms": round(1e3 * t_acc, 3),
    }
    return out


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
    NL = args.layers

    # ---- headline: cfg5 step (cfg2 attention x NL layers + acceptance), inputs resident in HBM ----------
    w = wl.config2(args.seed, tensors=False)  # lengths only; tensors are drawn on the GPU
    acc = wl.config5_accept(args.seed)
    step = Step(args, bass, harness, torch, w, NL, dev, True, acc)
    step.fill(w, args.seed)
    if not args.no_graph:
        step.capture()

    if args.calibration_copy:  # 1 GiB read + 1 GiB written per copy, by a plain elementwise copy kernel
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    wall = step.time_steps(args.steps, args.warmup)
    ms_per_step = 1e3 * wall / args.steps
    plan_us, attn_us, accept_us = step.launch_times(args.steps)
    kv_bytes = step.kv_bytes()
    value = kv_bytes * NL / (wall / args.steps) / 1e9
    n_acc_host = harness.to_host(step.n_accept)
    waves_in_effect = args.waves if args.waves else bass.bass_set_attention_waves(0)

    def frac_of(kvb, us):
        return kvb / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS

    seeds = [{"seed": args.seed, "kv_bytes_per_layer": kv_bytes, "ms_per_step": round(ms_per_step, 4),
              "GBps": round(value, 1), "attention_call_us": round(attn_us, 2), "frac": round(frac_of(kv_bytes, attn_us), 4)}]
    ceiling_us = ceiling_bytes = None
    others = {}
    warp_us = two_us = fused_us = None
    if not args.only_headline:
        ceiling_us, ceiling_bytes = step.ceiling(6, 768)
        # ---- the other draws of the same recipe: same slabs, same graph, lengths and contents redrawn ----
        for s in [x for x in (0, 1, 2) if x != args.seed]:
            ws_, acc_s = wl.config2(s, tensors=False), wl.config5_accept(s)
            step.fill(ws_, s, acc_s)
            wall_s = step.time_steps(args.steps, args.warmup)
            _, attn_s, _ = step.launch_times(args.steps)
            kvb = step.kv_bytes()
            seeds.append({"seed": s, "kv_bytes_per_layer": kvb, "ms_per_step": round(1e3 * wall_s / args.steps, 4),
                          "GBps": round(kvb * NL / (wall_s / args.steps) / 1e9, 1), "attention_call_us": round(attn_s, 2),
                          "frac": round(frac_of(kvb, attn_s), 4)})
        seeds.sort(key=lambda r: r["seed"])

        # ---- side measurement: the logits front end that would make p and q ---------------------------
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
                bass.bass_warp_probs(lt, 0.2, 0.95, pw, step.status)
                bass.bass_warp_probs(ld, 0.2, 0.95, qw, step.status)
            e1.record()
            torch.cuda.synchronize()
            warp_ms.append(e0.elapsed_time(e1) / reps)
        warp_us = 1e3 * warp_ms[-1]
        # ... and the call that goes from the logits to the acceptance without storing p and q
        wa_ws = torch.empty(bass.bass_warp_accept_workspace_bytes(acc.B, acc.kmax, acc.V), dtype=torch.uint8, device=dev)
        n_acc2, nxt2 = torch.zeros_like(step.n_accept), torch.zeros_like(step.next_token)
        two_us = step.repeated(lambda: (bass.bass_warp_probs(lt, 0.2, 0.95, pw, step.status),
                                        bass.bass_warp_probs(ld, 0.2, 0.95, qw, step.status),
                                        bass.bass_spec_accept(pw, qw, step.tok, step.ndr, step.u, n_acc2, nxt2, None, step.status)),
                               n=reps)
        want = (n_acc2.clone(), nxt2.clone())
        fused_us = step.repeated(lambda: bass.bass_warp_accept(lt, ld, 0.2, 0.95, step.tok, step.ndr, step.u, n_acc2, nxt2,
                                                               wa_ws, None, step.status), n=reps)
        assert torch.equal(n_acc2, want[0]) and torch.equal(nxt2, want[1]), "bass_warp_accept differs from the two calls"
        del lt, ld, pw, qw, wa_ws

    del step
    torch.cuda.empty_cache()

    if not args.only_headline:
        # ---- the attention launches of the other configurations (append fused, one plan per sweep) --------
        for name, make, nl in (("cfg3", wl.config3, 8), ("cfg4", wl.config4, NL)):
            wo = make(0, tensors=False)
            so = Step(args, bass, harness, torch, wo, nl, dev, False)
            so.fill(wo, 0)
            so.run()
            torch.cuda.synchronize()
            p_us, a_us, _ = so.launch_times(max(4, args.steps // 2))
            c_us, c_bytes = so.ceiling(3, 768)
            kvb = so.kv_bytes()
            rows = wo.kmax * (wo.Hq // wo.Hkv)
            others[name] = {
                "workload": f"B={wo.B}, Hq={wo.Hq}, Hkv={wo.Hkv}, D={wo.D}, {nl} cache slabs in turn, seed 0",
                "kv_bytes_per_call": kvb, "attention_call_us": round(a_us, 2), "plan_us": round(p_us, 2),
                "GBps": round(kvb / (a_us * 1e-6) / 1e9, 1), "frac": round(frac_of(kvb, a_us), 4),
                "launches_per_call": 1 if rows <= 16 else 2,
                "ceiling_GBps": round(c_bytes / (c_us * 1e-6) / 1e9, 1),
                "frac_of_ceiling": round((kvb / a_us) / (c_bytes / c_us), 4),
            }
            assert int(so.status.item()) == 0
            del so
            torch.cuda.empty_cache()

    version = bass.bass_version()
    fracs = sorted(r["frac"] for r in seeds)
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
            "workload": "cfg5 full verification step = one plan + cfg2 ragged MHA verify attention (B=8, Hq=Hkv=32, D=128, "
                        + ("bf16 Q, INT8 KV cache, " if args.kv_int8 else "bf16, ") +
                        f"ctx U[512,2048], drafts U[1,6]) x {NL} layers + spec_accept (V=50000, k=5)",
            "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "layers": NL, "seed": args.seed,
            "ctx_len": w.ctx_len.tolist(), "draft_len": w.draft_len.tolist(),
            "kv_bytes_per_layer": kv_bytes, "attention_waves": waves_in_effect,
            "launch": "eager" if args.no_graph else "hip_graph_replay",
            "append": "separate launch" if args.separate_append else "fused into the attention launch",
            "plan": "inside every call" if (args.unplanned or args.separate_append) else "one bass_attention_plan per step",
            "bass_version": version,
        },
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "verified_tokens_per_s": round(w.verified_tokens / (wall / args.steps), 1),
        "emitted_tokens_per_s": round(float((n_acc_host + 1).sum()) / (wall / args.steps), 1),
        "attention_call_us": round(attn_us, 2),
        "attention_plan_us": round(plan_us, 2),
        "spec_accept_us": round(accept_us, 2),
        "logit_warp_us": None if warp_us is None else round(warp_us, 2),
        "logits_to_acceptance_us": None if fused_us is None else {
            "bass_warp_probs x 2 + bass_spec_accept": round(two_us, 2), "bass_warp_accept": round(fused_us, 2)},
        "roofline": {
            "kernel": ("verify_attn_bf16<128,1,int8> (quantizing append + streaming + split-context reduction, one launch)"
                       if args.kv_int8 else
                       "verify_attn_bf16<128,1> (append + streaming + split-context reduction, one launch)"),
            "bound": "hbm",
            "achieved": round(kv_bytes / (attn_us * 1e-6) / 1e9, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(frac_of(kv_bytes, attn_us), 4),
            "traffic": None if args.kv_int8 else measured_traffic(version),
            "ceiling_GBps": None if ceiling_us is None else round(ceiling_bytes / (ceiling_us * 1e-6) / 1e9, 1),
            "ceiling_us": None if ceiling_us is None else round(ceiling_us, 2),
            "frac_of_ceiling": None if ceiling_us is None else round((kv_bytes / attn_us) / (ceiling_bytes / ceiling_us), 4),
            "ceiling_kernel": "bass_bench_stream_read: plain non-temporal read of the same number of bytes from the same slabs, 768 wavefronts",
        },
        "seeds": seeds,
        "roofline_frac_median_of_seeds": fracs[len(fracs) // 2],
        "roofline_frac_min_of_seeds": fracs[0],
        "other_configs": others,
    }

    if not args.no_cpu_baseline:
        wt = wl.config2(args.seed)  # one layer's tensors on the host
        kvb_host = wt.kv_bytes
        result["cpu_baseline"] = oracle_baseline(args, wl, wt, acc, kvb_host, NL)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
