"""The work plan of the attention launches, checked on the CPU (no GPU needed).

1. bass_attention_plan_host (the library's host planner, through the C ABI) on random ragged batches:
   every real 32-token block of every (sequence, kv head) unit belongs to exactly one share's segments;
   inactive sequences get none; the contributors of a unit are exactly the shares w_lo..w_hi its
   segments name; partial slots never collide; every offset a launch derives stays inside the cache,
   the overflow list and the workspace.  The block counts come from the paper's statement of the
   problem (Section 3.2: every sequence is processed over its own length, padded positions only in the
   PAD scheme), written out here independently of the library.
2. The same arithmetic (attn_plan.h, bass_layout.h) compiled with g++ under AddressSanitizer and
   UndefinedBehaviorSanitizer and swept over shapes, lengths and spreads (tests/host/plan_sanitize.cpp).
3. The CPU oracle compiled under the same sanitizers and run once on small inputs
   (tests/host/oracle_sanitize.c).
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

import paper_2404_15778_amd as bass

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2404_15778_amd", "csrc")
HOST = os.path.join(ROOT, "tests", "host")

HEADER_WORDS = 16  # magic, B, kmax, Hkv, Lcap, nshares, pad, pad_before, span, flags, total, any_inactive, any_clamped
SEG_WORDS = 8      # b, kvh, L, nq, first, n, owners, flags
REC_WORDS = 20     # two segments, nseg, overflow, signature, reserved
MAGIC = 0x42415331


def parse_plan(plan: np.ndarray, B: int, Hkv: int):
    """Splits the bytes of a plan into its parts (the layout include/bass.h leaves opaque; the test knows it)."""
    w = plan.view(np.int32)
    hdr = w[:HEADER_WORDS]
    nshares = int(hdr[5])
    a16 = lambda words: (words + 3) // 4 * 4
    at = HEADER_WORDS
    records = w[at:at + nshares * REC_WORDS].reshape(nshares, REC_WORDS)
    at += nshares * REC_WORDS
    n_over = nshares + B * Hkv
    overflow = w[at:at + n_over * SEG_WORDS].reshape(n_over, SEG_WORDS)
    at += n_over * SEG_WORDS
    seq_L = w[at:at + B]
    at = a16(at + B)
    seq_nq = w[at:at + B]
    at = a16(at + B)
    seq_inc = w[at:at + B]
    at = a16(at + B)
    owners = w[at:at + B * Hkv]
    at = a16(at + B * Hkv)
    return dict(hdr=hdr, nshares=nshares, records=records, overflow=overflow, seq_L=seq_L, seq_nq=seq_nq,
                seq_inc=seq_inc, owners=owners, words=at)


def clamp(L, nq, kmax, Lcap):
    """The clamping include/bass.h promises for out-of-range lengths."""
    nq = min(max(nq, 0), kmax, Lcap)
    L = max(L, 0)
    if L + nq > Lcap:
        L = Lcap - nq
    return L, nq


def segments_of(plan, w):
    rec = plan["records"][w]
    nseg, over = int(rec[16]), int(rec[17])
    out = []
    for i in range(nseg):
        seg = rec[8 * i:8 * i + 8] if i < 2 else plan["overflow"][over + i - 2]
        out.append(tuple(int(x) for x in seg))
    return out


def check_plan(desc, ctx_len, draft_len, flags, padded_len, expect_shares=None):
    plan_bytes, status = bass.bass_attention_plan_host(desc, ctx_len, draft_len, flags, padded_len)
    B, Hkv, kmax, Lcap = desc.B, desc.Hkv, desc.kmax, desc.Lcap
    plan = parse_plan(plan_bytes, B, Hkv)
    hdr = plan["hdr"]
    assert int(hdr[0]) == MAGIC and tuple(int(x) for x in hdr[1:5]) == (B, kmax, Hkv, Lcap)
    nshares = plan["nshares"]
    if expect_shares is not None:
        assert nshares == expect_shares
    assert plan["words"] * 4 <= bass.bass_attention_plan_bytes(desc)
    span = int(hdr[8])
    assert span == padded_len
    nblk_cap = (Lcap + 31) // 32
    clamped = [clamp(int(l), int(n), kmax, Lcap) for l, n in zip(ctx_len, draft_len)]
    assert [int(x) for x in plan["seq_L"]] == [c[0] for c in clamped]
    assert [int(x) for x in plan["seq_nq"]] == [c[1] for c in clamped]
    any_clamped = any(c != (int(l), int(n)) for c, l, n in zip(clamped, ctx_len, draft_len))
    assert bool(hdr[12]) == any_clamped and bool(status & bass.STATUS_LEN_CLAMPED) == any_clamped
    assert bool(hdr[11]) == any(c[1] == 0 for c in clamped)
    # blocks of a unit, from the problem statement: the sequence's own length, or the padded length
    nblk = [0 if nq == 0 else (max(L + nq, min(span, Lcap)) + 31) // 32 for L, nq in clamped]
    cover = {(b, h): np.zeros(nblk[b], np.int32) for b in range(B) for h in range(Hkv)}
    holders = {}
    slots = set()
    real_per_share = []
    seen_overflow = 0
    for w in range(nshares):
        segs = segments_of(plan, w)
        rec = plan["records"][w]
        if len(segs) > 2:  # a share's run of overflow entries: behind the runs of the shares before it, inside the list
            assert int(rec[17]) >= seen_overflow
            seen_overflow = int(rec[17]) + len(segs) - 2
        assert seen_overflow <= nshares + B * Hkv
        prev = -1
        real = 0
        for (b, h, L, nq, first, n, owners, sflags) in segs:
            assert 0 <= b < B and 0 <= h < Hkv
            assert (L, nq) == clamped[b] and nq > 0
            assert n >= 1 and first >= 0 and first + n <= nblk[b] <= nblk_cap
            assert bool(sflags & 1) == (first + n == nblk[b])
            unit = b * Hkv + h
            assert unit > prev, "the units of a share come in list order"
            prev = unit
            cover[(b, h)][first:first + n] += 1
            holders.setdefault(unit, []).append(w)
            assert owners == int(plan["owners"][unit])
            slot = w + unit
            assert slot not in slots and slot < nshares + B * Hkv
            slots.add(slot)
            real += n
        real_per_share.append(real)
    for (b, h), c in cover.items():
        assert (c == 1).all(), f"unit ({b},{h}): blocks covered {c.tolist()}"
        unit = b * Hkv + h
        if nblk[b] == 0:
            assert unit not in holders
            continue
        lo, hi = int(plan["owners"][unit]) & 0xFFFF, (int(plan["owners"][unit]) >> 16) & 0xFFFF
        assert holders[unit] == list(range(lo, hi + 1)), f"unit {unit}: holders {holders[unit]} vs {lo}..{hi}"
    # balance: the shares that hold work differ by at most one entry (real blocks plus a unit's `pad` virtual
    # ones), except the last one, which takes what is left
    total_real = sum(nblk) * Hkv
    assert sum(real_per_share) == total_real
    pad = int(hdr[6])
    if total_real:
        entries = total_real + pad * sum(1 for x in nblk if x) * Hkv
        assert int(hdr[10]) == entries
        busy = [r for r in real_per_share if r]
        assert max(busy) <= -(-entries // min(len(busy), nshares)) + 1
    return plan


def mk(B, kmax, Hq, Hkv, D, Lcap, dtype="bf16"):
    return bass.make_desc(B, kmax, Hq, Hkv, D, Lcap, dtype, 1.0)


def test_paper_shaped_batches():
    import workloads as wl
    for seed in range(3):
        w = wl.config2(seed, tensors=False)
        d = mk(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap)
        for flags in (0, bass.PLAN_APPEND):
            plan = check_plan(d, w.ctx_len, w.draft_len, flags, 0, expect_shares=768)
            assert int(plan["hdr"][6]) == (3 if flags else 2)
    w = wl.config3(0, tensors=False)
    check_plan(mk(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap), w.ctx_len, w.draft_len, 0, 0, expect_shares=768)
    w = wl.config4(0, tensors=False)  # grouped-query: one stretch per workgroup
    check_plan(mk(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap), w.ctx_len, w.draft_len, 0, 0, expect_shares=256)
    check_plan(mk(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, "int8kv"), w.ctx_len, w.draft_len, bass.PLAN_APPEND, 0,
               expect_shares=1024)
    w = wl.config2(0, tensors=False)  # INT8 caches with one query tile per kv head: the bf16 default
    check_plan(mk(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, "int8kv"), w.ctx_len, w.draft_len, bass.PLAN_APPEND, 0,
               expect_shares=768)


@pytest.mark.parametrize("seed", range(40))
def test_random_batches(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 80)) if seed % 5 == 0 else int(rng.integers(1, 10))
    Hkv = int(rng.choice([1, 2, 3, 8, 32]))
    g = int(rng.choice([1, 2, 4, 8]))
    kmax = int(rng.integers(1, 9))
    Lcap = int(rng.choice([33, 200, 2056, 8200]))
    dtype = ["bf16", "fp32", "int8kv"][seed % 3]
    if dtype != "fp32" and kmax * g > 64:
        g = 1
    d = mk(B, kmax, Hkv * g, Hkv, 128 if dtype != "fp32" else 64, Lcap, dtype)
    ctx = rng.integers(0, Lcap + 1, B)
    dl = rng.integers(0, kmax + 1, B)
    if seed % 4 == 0:  # out-of-range lengths are clamped
        ctx[0] = Lcap + 7
        dl[-1] = kmax + 3
    if seed % 7 == 0:
        ctx[:] = rng.integers(0, 40, B)  # many tiny units: shares span several of them
    waves = [0, 64, 100, 1020, 8192][seed % 5]
    try:
        bass.bass_set_attention_waves(waves)
        for flags, padded in ((0, 0), (bass.PLAN_APPEND, 0), (0, int(rng.integers(1, Lcap + 30)))):
            check_plan(d, ctx, dl, flags, padded)
    finally:
        bass.bass_set_attention_waves(0)


def test_empty_batch_and_single_block():
    d = mk(3, 4, 8, 8, 128, 100)
    plan = check_plan(d, [5, 9, 0], [0, 0, 0], 0, 0)
    assert int(plan["hdr"][10]) == 0 and all(int(r[16]) == 0 for r in plan["records"])
    check_plan(d, [0, 0, 0], [1, 0, 1], bass.PLAN_APPEND, 0)  # one-token sequences: one block per unit


def test_bad_arguments():
    d = mk(2, 4, 8, 8, 128, 100)
    lib = bass.lib()
    import ctypes
    buf = np.zeros(bass.bass_attention_plan_bytes(d), np.uint8)
    ctx = np.zeros(2, np.int32)
    args = lambda flags, padded, n: (ctypes.byref(d), ctypes.c_void_p(ctx.ctypes.data), ctypes.c_void_p(ctx.ctypes.data),
                                    flags, padded, ctypes.c_void_p(buf.ctypes.data), n, None)
    assert lib.bass_attention_plan_host(*args(0, 0, 16)) == bass.ERR_WORKSPACE_TOO_SMALL
    assert lib.bass_attention_plan_host(*args(2, 0, buf.size)) == bass.ERR_INVALID_ARG
    assert lib.bass_attention_plan_host(*args(0, -1, buf.size)) == bass.ERR_INVALID_ARG
    assert lib.bass_attention_plan_host(*args(bass.PLAN_APPEND, 64, buf.size)) == bass.ERR_INVALID_ARG
    assert bass.bass_attention_plan_bytes(mk(2, 4, 8, 3, 128, 100)) == 0  # Hq % Hkv != 0


def _sanitized(compiler, src, extra, args=()):
    exe = os.path.join(ROOT, "tests", "host", "_build_" + os.path.splitext(os.path.basename(src))[0])
    cmd = [compiler, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-I", CSRC, *extra,
           "-o", exe, src, "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    try:
        return subprocess.run([exe, *args], capture_output=True, text=True, timeout=300)
    finally:
        os.remove(exe)


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_plan_arithmetic_under_sanitizers():
    r = _sanitized("g++", os.path.join(HOST, "plan_sanitize.cpp"), ["-std=c++17"], ["4000"])
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout + r.stderr


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host compiler")
def test_oracle_under_sanitizers():
    r = _sanitized("gcc", os.path.join(HOST, "oracle_sanitize.c"), ["-std=c11", "-fopenmp"])
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr
