"""Device-side plumbing around the binding: uploads numpy inputs, owns caches and workspace.

No arithmetic of the method happens here; every step is a call into libbass.
bf16 tensors travel as uint16 bit patterns on the numpy side.
"""
from __future__ import annotations

import numpy as np
import torch

from . import (bass_kv_gather_int8, bass_warp_probs, bass_warp_accept, bass_warp_accept_workspace_bytes, AttnDesc, alloc_kv_cache, alloc_workspace, bass_append_verify_attention, bass_kv_append, bass_kv_gather,
               bass_spec_accept, bass_verify_attention, bass_verify_attention_pad, bass_verify_attention_split, make_desc)


def to_device(a: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy -> torch on the GPU; uint16 arrays are reinterpreted as bf16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DeviceAttention:
    """Caches + workspace of one attention layer for a fixed shape."""

    def __init__(self, B, kmax, Hq, Hkv, D, Lcap, dtype, scale, device="cuda", poison=False):
        self.desc: AttnDesc = make_desc(B, kmax, Hq, Hkv, D, Lcap, dtype, scale)
        self.device = device
        fill = 0xFF if poison else 0  # 0xFF.. is a NaN pattern in bf16 and fp32
        self.Kc = alloc_kv_cache(self.desc, device, fill)
        self.Vc = alloc_kv_cache(self.desc, device, fill)
        self.ws = alloc_workspace(self.desc, device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.O = torch.empty((B, kmax, Hq, D), dtype=torch.float32, device=device)
        self.lse = torch.empty((B, kmax, Hq), dtype=torch.float32, device=device)

    def append(self, K_rows, V_rows, offset, count):
        """Write rows [B, n, Hkv, D] (torch, on device) at per-sequence offsets."""
        d = self.desc.replace(kmax=int(K_rows.shape[1]))
        bass_kv_append(d, self.Kc, self.Vc, K_rows, V_rows, offset, count, self.status)

    def gather_int8(self, start, count, n):
        """INT8 caches: (K codes, V codes, K scales, V scales) of tokens start .. start + count - 1."""
        d = self.desc.replace(kmax=int(n))
        Kq = torch.zeros((d.B, n, d.Hkv, d.D), dtype=torch.int8, device=self.device)
        Vq = torch.zeros_like(Kq)
        Ks = torch.zeros((d.B, n, d.Hkv), dtype=torch.float32, device=self.device)
        Vs = torch.zeros_like(Ks)
        bass_kv_gather_int8(d, self.Kc, self.Vc, Kq, Vq, Ks, Vs, start, count, self.status)
        return Kq, Vq, Ks, Vs

    def gather(self, start, count, n):
        d = self.desc.replace(kmax=int(n))
        et = torch.bfloat16 if d.dtype == 0 else torch.float32
        K = torch.zeros((d.B, n, d.Hkv, d.D), dtype=et, device=self.device)
        V = torch.zeros_like(K)
        bass_kv_gather(d, self.Kc, self.Vc, K, V, start, count, self.status)
        return K, V

    def verify(self, Q, ctx_len, draft_len, want_lse=True, variant="ragged", padded_len=0):
        """variant: "ragged" (one launch, true lengths), "pad" (BASS-PAD), "split" (BASS-SPLIT)."""
        lse = self.lse if want_lse else None
        if variant == "pad":
            bass_verify_attention_pad(self.desc, Q, self.Kc, self.Vc, ctx_len, draft_len, padded_len, self.O, lse,
                                      self.ws, self.status)
        elif variant == "split":
            bass_verify_attention_split(self.desc, Q, self.Kc, self.Vc, ctx_len, draft_len, self.O, lse, self.ws,
                                        self.status)
        else:
            bass_verify_attention(self.desc, Q, self.Kc, self.Vc, ctx_len, draft_len, self.O, lse, self.ws,
                                  self.status)
        return self.O, self.lse

    def append_verify(self, Q, K_new, V_new, ctx_len, draft_len, want_lse=True):
        """Append this step's rows and verify in one launch."""
        bass_append_verify_attention(self.desc, Q, K_new, V_new, self.Kc, self.Vc, ctx_len, draft_len, self.O,
                                     self.lse if want_lse else None, self.ws, self.status)
        return self.O, self.lse


def i32(a, device="cuda"):
    return torch.as_tensor(np.asarray(a, dtype=np.int32), device=device)


def run_attention_workload(w, poison=True, device="cuda", fused=False):
    """Whole attention path on a synthetic workload (see workloads.AttnWorkload): fill the cache
    with the context rows, append the step's own rows, verify (two launches, or one with
    fused=True).  Returns (O, lse, status, DeviceAttention) with O, lse on the host."""
    da = DeviceAttention(w.B, w.kmax, w.Hq, w.Hkv, w.D, w.Lcap, w.dtype, w.scale, device, poison)
    K, V = to_device(w.K, device), to_device(w.V, device)
    ctx, nq = i32(w.ctx_len, device), i32(w.draft_len, device)
    zero = torch.zeros_like(ctx)
    da.append(K, V, zero, ctx)  # context (prompt + earlier accepted tokens)
    # this step's rows, gathered on the host into the [B, kmax, Hkv, D] layout of a model's K/V projection
    Kn = np.zeros((w.B, w.kmax, w.Hkv, w.D), w.K.dtype)
    Vn = np.zeros_like(Kn)
    for b in range(w.B):
        L, n = int(w.ctx_len[b]), int(w.draft_len[b])
        Kn[b, :n] = w.K[b, L:L + n]
        Vn[b, :n] = w.V[b, L:L + n]
    if fused:
        O, lse = da.append_verify(to_device(w.Q, device), to_device(Kn, device), to_device(Vn, device), ctx, nq)
    else:
        da.append(to_device(Kn, device), to_device(Vn, device), ctx, nq)
        O, lse = da.verify(to_device(w.Q, device), ctx, nq)
    torch.cuda.synchronize()
    return to_host(O), to_host(lse), int(da.status.item()), da


def run_accept_workload(a, ctx_len=None, device="cuda"):
    """bass_spec_accept on a synthetic workload (see workloads.AcceptWorkload); host results."""
    B = a.B
    n_accept = torch.full((B,), -1, dtype=torch.int32, device=device)
    next_token = torch.full((B,), -1, dtype=torch.int32, device=device)
    status = torch.zeros(1, dtype=torch.int32, device=device)
    ctx = None if ctx_len is None else i32(ctx_len, device)
    bass_spec_accept(to_device(a.p, device), to_device(a.q, device), i32(a.draft_tok, device).reshape(B, a.kmax),
                     i32(a.n_draft, device), to_device(a.u, device), n_accept, next_token, ctx, status)
    torch.cuda.synchronize()
    out = (to_host(n_accept), to_host(next_token), int(status.item()))
    return out if ctx is None else out + (to_host(ctx),)


def run_warp_accept(logits_main, logits_draft, temperature, top_p, draft_tok, n_draft, u, ctx_len=None, device="cuda",
                    two_calls=False):
    """bass_warp_accept on host logits, or (two_calls) bass_warp_probs on both tensors followed by
    bass_spec_accept; returns (n_accept, next_token, status[, ctx_len]) on the host."""
    lm = to_device(np.asarray(logits_main, np.float32), device)
    B, k1, V = lm.shape
    kmax = k1 - 1
    ld = to_device(np.asarray(logits_draft, np.float32), device) if kmax else None
    tok = i32(draft_tok, device).reshape(B, kmax) if kmax else None
    n_accept = torch.full((B,), -1, dtype=torch.int32, device=device)
    next_token = torch.full((B,), -1, dtype=torch.int32, device=device)
    status = torch.zeros(1, dtype=torch.int32, device=device)
    ctx = None if ctx_len is None else i32(ctx_len, device)
    uu, nd = to_device(np.asarray(u, np.float32), device), i32(n_draft, device)
    if two_calls:
        p = torch.full_like(lm, float("nan"))
        bass_warp_probs(lm, temperature, top_p, p, status)
        q = None
        if kmax:
            q = torch.full_like(ld, float("nan"))
            bass_warp_probs(ld, temperature, top_p, q, status)
        bass_spec_accept(p, q, tok, nd, uu, n_accept, next_token, ctx, status)
    else:
        # poisoned workspace: the call may not depend on its contents
        ws = torch.full((bass_warp_accept_workspace_bytes(B, kmax, V),), 0xA5, dtype=torch.uint8, device=device)
        bass_warp_accept(lm, ld, temperature, top_p, tok, nd, uu, n_accept, next_token, ws, ctx, status)
    torch.cuda.synchronize()
    out = (to_host(n_accept), to_host(next_token), int(status.item()))
    return out if ctx is None else out + (to_host(ctx),)


def run_warp_probs(logits: np.ndarray, temperature, top_p, device="cuda"):
    """bass_warp_probs on host logits [..., V]; returns (probs on the host, status)."""
    lg = to_device(np.asarray(logits, np.float32), device)
    probs = torch.full_like(lg, float("nan"))
    status = torch.zeros(1, dtype=torch.int32, device=device)
    bass_warp_probs(lg, temperature, top_p, probs, status)
    torch.cuda.synchronize()
    return to_host(probs), int(status.item())
