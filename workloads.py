"""Seeded synthetic inputs for the BASS verification step.

This module only DRAWS inputs (lengths, tensors, probability rows, uniforms) with
the shapes and value distributions of the benchmark configurations.  It holds none
of the method's arithmetic and is the one module shared by the CPU oracle's tests
and the HIP path's tests / benchmark.  numpy only.

Conventions
  * bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even of the
    fp32 draw), fp32 tensors as float32.
  * K, V are "logical" token-major caches [B, Lrows, Hkv, D]: row j of sequence b is
    token j; rows [0, ctx_len[b]+draft_len[b]) are drawn, the rest are zero.  The
    draft tokens' own K/V rows are the last draft_len[b] valid rows.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class AttnWorkload:
    name: str
    B: int
    kmax: int
    Hq: int
    Hkv: int
    D: int
    dtype: str            # "bf16" | "fp32"
    scale: float
    ctx_len: np.ndarray   # [B] int32
    draft_len: np.ndarray  # [B] int32
    Lcap: int             # cache capacity (tokens) to allocate on the device
    Q: np.ndarray = field(repr=False, default=None)   # [B,kmax,Hq,D]
    K: np.ndarray = field(repr=False, default=None)   # [B,Lrows,Hkv,D]
    V: np.ndarray = field(repr=False, default=None)

    @property
    def elt_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def kv_bytes(self) -> int:
        """Algorithmic KV bytes of one verify-attention call: every valid K and V row once."""
        tokens = int((self.ctx_len.astype(np.int64) + self.draft_len).sum())
        return tokens * 2 * self.Hkv * self.D * self.elt_bytes

    @property
    def verified_tokens(self) -> int:
        return int(self.draft_len.sum())


def _draw(rng, shape, dtype, mult=1.0):
    x = rng.standard_normal(shape, dtype=np.float32)
    if mult != 1.0:
        x *= np.float32(mult)
    return to_bf16_bits(x) if dtype == "bf16" else x


def make_attention(name, B, Hq, Hkv, D, dtype, ctx_len, draft_len, seed, kmax=None, Lcap=None,
                   q_mult=1.0, tensors=True) -> AttnWorkload:
    """Draw Q, K, V ~ N(0,1) (Q optionally scaled by q_mult) for given lengths."""
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    draft_len = np.asarray(draft_len, dtype=np.int32)
    kmax = int(kmax if kmax is not None else max(1, int(draft_len.max())))
    total = ctx_len + draft_len
    Lrows = max(1, int(total.max()))
    Lcap = int(Lcap if Lcap is not None else Lrows)
    w = AttnWorkload(name, B, kmax, Hq, Hkv, D, dtype, 1.0 / math.sqrt(D), ctx_len, draft_len, Lcap)
    if not tensors:
        return w
    rng = np.random.default_rng([seed, 0xA77E])
    w.Q = _draw(rng, (B, kmax, Hq, D), dtype, q_mult)
    zero = np.uint16 if dtype == "bf16" else np.float32
    w.K = np.zeros((B, Lrows, Hkv, D), zero)
    w.V = np.zeros((B, Lrows, Hkv, D), zero)
    for b in range(B):
        n = int(total[b])
        w.K[b, :n] = _draw(rng, (n, Hkv, D), dtype)
        w.V[b, :n] = _draw(rng, (n, Hkv, D), dtype)
    return w


def config1(seed=0, tensors=True) -> AttnWorkload:
    """Tiny ragged verify: B=2, Hq=Hkv=4, D=64, fp32; ctx_len={37,90}, draft_len={4,3}."""
    return make_attention("cfg1_tiny_fp32", 2, 4, 4, 64, "fp32", [37, 90], [4, 3], seed, tensors=tensors)


def config2(seed=0, tensors=True) -> AttnWorkload:
    """7.8B-like MHA verify: B=8, Hq=Hkv=32, D=128, bf16; ctx ~ U{512..2048}, drafts ~ U{1..6}."""
    rng = np.random.default_rng([seed, 2])
    ctx = rng.integers(512, 2049, size=8)
    nq = rng.integers(1, 7, size=8)
    return make_attention("cfg2_mha_b8", 8, 32, 32, 128, "bf16", ctx, nq, seed, kmax=6, Lcap=2048 + 8,
                          tensors=tensors)


def config3(seed=0, tensors=True) -> AttnWorkload:
    """Large-batch long-context ragged: B=32, H=32, D=128, bf16; ctx log-uniform [128,8192], drafts U{1..8}."""
    rng = np.random.default_rng([seed, 3])
    ctx = np.rint(np.exp(rng.uniform(math.log(128), math.log(8192), size=32))).astype(np.int64)
    ctx = np.clip(ctx, 128, 8192)
    nq = rng.integers(1, 9, size=32)
    return make_attention("cfg3_large_ragged", 32, 32, 32, 128, "bf16", ctx, nq, seed, kmax=8,
                          Lcap=8192 + 8, tensors=tensors)


def config4(seed=0, tensors=True) -> AttnWorkload:
    """GQA verify: B=16, Hq=64, Hkv=8, D=128, bf16; ctx ~ U{1024..4096}, drafts ~ U{2..6}; Q ~ N(0,1)/sqrt(D)."""
    rng = np.random.default_rng([seed, 4])
    ctx = rng.integers(1024, 4097, size=16)
    nq = rng.integers(2, 7, size=16)
    return make_attention("cfg4_gqa", 16, 64, 8, 128, "bf16", ctx, nq, seed, kmax=6, Lcap=4096 + 8,
                          q_mult=1.0 / math.sqrt(128), tensors=tensors)


@dataclass
class AcceptWorkload:
    name: str
    B: int
    kmax: int
    V: int
    p: np.ndarray = field(repr=False)          # [B,kmax+1,V] float32 main-model probabilities
    q: np.ndarray = field(repr=False)          # [B,kmax,V]   float32 draft-model probabilities
    draft_tok: np.ndarray = field(repr=False)  # [B,kmax] int32, x_i ~ q_i
    n_draft: np.ndarray = field(repr=False)    # [B] int32
    u: np.ndarray = field(repr=False)          # [B,kmax+1] float32 in [0,1)


def softmax_f32(x: np.ndarray) -> np.ndarray:
    """Row softmax in float32: how the synthetic probability rows are produced from logits."""
    x = x.astype(np.float32)
    e = np.exp(x - x.max(axis=-1, keepdims=True), dtype=np.float32)
    return (e / e.sum(axis=-1, keepdims=True, dtype=np.float32)).astype(np.float32)


def make_logits(B, kmax, V, seed, sigma_target, sigma_noise=None):
    """Raw logits of the acceptance recipes: main-model rows [B, kmax+1, V] ~ N(0, sigma_target^2) and
    draft-model rows [B, kmax, V], independent with the same sigma (sigma_noise None) or the main
    model's plus N(0, sigma_noise^2).  fp32.  Inputs of the logits front end (temperature, top-p)."""
    rng = np.random.default_rng([seed, 0x106175])
    lt = rng.standard_normal((B, kmax + 1, V), dtype=np.float32) * np.float32(sigma_target)
    if sigma_noise is None:
        ld = rng.standard_normal((B, kmax, V), dtype=np.float32) * np.float32(sigma_target)
    else:
        ld = lt[:, :kmax] + rng.standard_normal((B, kmax, V), dtype=np.float32) * np.float32(sigma_noise)
    return lt, ld


def make_accept(name, B, kmax, V, seed, sigma_target, sigma_noise=None, n_draft=None) -> AcceptWorkload:
    """p = softmax(target logits ~ N(0, sigma_target^2)); q = softmax of independent logits with the
    same sigma (sigma_noise None) or of target logits + N(0, sigma_noise^2); drafts x_i ~ q_i."""
    rng = np.random.default_rng([seed, 0xACC])
    lt = rng.standard_normal((B, kmax + 1, V), dtype=np.float32) * np.float32(sigma_target)
    if sigma_noise is None:
        ld = rng.standard_normal((B, kmax, V), dtype=np.float32) * np.float32(sigma_target)
    else:
        ld = lt[:, :kmax] + rng.standard_normal((B, kmax, V), dtype=np.float32) * np.float32(sigma_noise)
    p, q = softmax_f32(lt), softmax_f32(ld)
    tok = np.zeros((B, kmax), np.int32)
    for b in range(B):
        for i in range(kmax):
            q64 = q[b, i].astype(np.float64)
            tok[b, i] = int(rng.choice(V, p=q64 / q64.sum()))
    if n_draft is None:
        n_draft = np.full(B, kmax, np.int32)
    u = rng.random((B, kmax + 1), dtype=np.float32)
    return AcceptWorkload(name, B, kmax, V, p, q, tok, np.asarray(n_draft, np.int32), u)


def config1_accept(seed=0) -> AcceptWorkload:
    """Acceptance part of the tiny config: vocab 64, p and q from independent N(0, 2^2) logits."""
    return make_accept("cfg1_accept_v64", 2, 4, 64, seed, 2.0, None, n_draft=[4, 3])


def config5_accept(seed=0) -> AcceptWorkload:
    """Full-step acceptance: B=8, k=5, vocab 50k; target logits N(0,3^2), draft = target + N(0,1)."""
    return make_accept("cfg5_accept_v50k", 8, 5, 50000, seed, 3.0, 1.0)
