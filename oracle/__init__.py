"""CPU oracle for the BASS verification step.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's `cpu_baseline` leg may import
this package; the product path (the HIP library and its binding) never does,
and this package never imports the product.

`bass_oracle.c` holds the arithmetic (plain fp64 C loops); this file only
compiles it with gcc and marshals numpy arrays into it.  `draft_length.py`
holds the draft-length heuristic (Algorithm 1) as plain Python, `logit_warp.py`
the logits front end (temperature, nucleus top-p, softmax) in numpy, `kv_int8.py`
the INT8 KV-cache quantizer in numpy.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bass_oracle.c")
_LIB = os.path.join(_HERE, "libbass_oracle.so")

DTYPE_BF16 = 0
DTYPE_FP32 = 1

STATUS_LEN_CLAMPED = 1
STATUS_TOKEN_CLAMPED = 2
STATUS_ZERO_MASS = 4


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp, no fast-math). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_verify_attention_row.restype = ctypes.c_double
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _elt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return DTYPE_FP32
    if a.dtype == np.uint16:
        return DTYPE_BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bit patterns), got {a.dtype}")


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def verify_attention(Q, K, V, ctx_len, draft_len, scale):
    """Ragged verify attention.

    Q [B,kmax,Hq,D]; K,V [B,Lrows,Hkv,D] logical token-major caches whose rows
    [0, ctx_len[b]+draft_len[b]) are valid (draft tokens' own K/V at the end);
    float32 or uint16 (bf16 bit patterns).  Returns (O [B,kmax,Hq,D], lse [B,kmax,Hq]) fp64.
    """
    Q, K, V = (np.ascontiguousarray(x) for x in (Q, K, V))
    dt = _elt(Q)
    assert _elt(K) == dt and _elt(V) == dt
    B, kmax, Hq, D = Q.shape
    Bk, Lrows, Hkv, Dk = K.shape
    assert (Bk, Dk) == (B, D) and V.shape == K.shape and Hq % Hkv == 0
    ctx_len, draft_len = _i32(ctx_len), _i32(draft_len)
    assert ctx_len.shape == (B,) and draft_len.shape == (B,)
    assert (ctx_len >= 0).all() and (draft_len >= 0).all() and (draft_len <= kmax).all()
    assert (ctx_len + draft_len <= Lrows).all()
    O = np.empty((B, kmax, Hq, D), np.float64)
    lse = np.empty((B, kmax, Hq), np.float64)
    _load().oracle_verify_attention(
        B, kmax, Hq, Hkv, D, Lrows, dt, ctypes.c_double(scale), _ptr(Q), _ptr(K), _ptr(V),
        _ptr(ctx_len), _ptr(draft_len), _ptr(O), _ptr(lse))
    return O, lse


def verify_attention_row(Q, K, V, b, i, h, ctx_len_b, scale, want_probs=False):
    """One output row (b, i, h) of the same attention: (out[D], lse[, P row])."""
    Q, K, V = (np.ascontiguousarray(x) for x in (Q, K, V))
    dt = _elt(Q)
    B, kmax, Hq, D = Q.shape
    _, Lrows, Hkv, _ = K.shape
    assert 0 <= b < B and 0 <= i < kmax and 0 <= h < Hq and ctx_len_b + i + 1 <= Lrows
    out = np.empty(D, np.float64)
    probs = np.empty(ctx_len_b + i + 1, np.float64) if want_probs else None
    lse = _load().oracle_verify_attention_row(
        kmax, Hq, Hkv, D, Lrows, dt, ctypes.c_double(scale), _ptr(Q), _ptr(K), _ptr(V),
        int(b), int(i), int(h), int(ctx_len_b), _ptr(out), _ptr(probs))
    return (out, float(lse), probs) if want_probs else (out, float(lse))


def kv_append(cache, rows, ctx_len, n_new):
    """In-place append of this step's K (or V) rows into a logical cache [B,Lrows,Hkv,D]."""
    assert cache.flags.c_contiguous and cache.dtype == rows.dtype
    rows = np.ascontiguousarray(rows)
    B, Lrows, Hkv, D = cache.shape
    kmax = rows.shape[1]
    assert rows.shape == (B, kmax, Hkv, D)
    ctx_len, n_new = _i32(ctx_len), _i32(n_new)
    assert (n_new >= 0).all() and (n_new <= kmax).all() and (ctx_len + n_new <= Lrows).all()
    _load().oracle_kv_append(B, kmax, Hkv, D, Lrows, cache.dtype.itemsize, _ptr(cache), _ptr(rows),
                             _ptr(ctx_len), _ptr(n_new))
    return cache


def spec_accept(p, q, draft_tok, n_draft, u, ctx_len=None):
    """Speculative-sampling acceptance.

    p [B,kmax+1,V], q [B,kmax,V] float32; draft_tok [B,kmax]; n_draft [B]; u [B,kmax+1] float32.
    Returns (n_accept [B], next_token [B], status) and, when ctx_len is given, the
    advanced lengths as a fourth item.
    """
    p = np.ascontiguousarray(p, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float32)
    B, k1, V = p.shape
    kmax = k1 - 1
    assert kmax >= 0 and u.shape == (B, kmax + 1)
    assert q.shape == (B, kmax, V)
    draft_tok = _i32(draft_tok).reshape(B, kmax)
    n_draft = _i32(n_draft)
    n_accept = np.empty(B, np.int32)
    next_token = np.empty(B, np.int32)
    status = np.zeros(1, np.int32)
    ctx = None if ctx_len is None else _i32(ctx_len).copy()
    _load().oracle_spec_accept(B, kmax, V, _ptr(p), _ptr(q), _ptr(draft_tok), _ptr(n_draft), _ptr(u),
                               _ptr(n_accept), _ptr(next_token), _ptr(ctx), _ptr(status))
    if ctx is None:
        return n_accept, next_token, int(status[0])
    return n_accept, next_token, int(status[0]), ctx
