"""Python binding of libbass, the MI355X (gfx950) library for the BASS verification step.

Argument marshalling only: every function here has the name and the argument order of
the C entry point in include/bass.h and passes raw device pointers of torch tensors to it;
all arithmetic runs in the HIP kernels.  torch is used for device memory and streams.
There is no CPU fallback: without the built library (paper_2404_15778_amd/libbass.so,
see build.py) importing works but every call raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbass.so")

OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_HIP = -1, -2, -3, -4
STATUS_LEN_CLAMPED, STATUS_TOKEN_CLAMPED, STATUS_ZERO_MASS, STATUS_PLAN_MISMATCH = 1, 2, 4, 8
PLAN_APPEND = 1
DTYPE_BF16, DTYPE_FP32, DTYPE_INT8KV = 0, 1, 2

# every symbol include/bass.h declares
EXPORTS = (
    "bass_version", "bass_status_string", "bass_kv_cache_bytes", "bass_verify_attention_workspace_bytes",
    "bass_kv_append", "bass_kv_gather", "bass_kv_gather_int8", "bass_verify_attention", "bass_verify_attention_pad",
    "bass_verify_attention_split", "bass_append_verify_attention", "bass_spec_accept", "bass_warp_probs",
    "bass_warp_accept", "bass_warp_accept_workspace_bytes",
    "bass_set_attention_waves", "bass_draft_len_init", "bass_next_draft_len",
    "bass_attention_plan_bytes", "bass_attention_plan", "bass_attention_plan_host", "bass_verify_attention_planned",
    "bass_bench_stream_read", "bass_verify_attention_noalloc",
)


class AttnDesc(ctypes.Structure):
    """Mirror of `bass_attn_desc`."""
    _fields_ = [("B", ctypes.c_int32), ("kmax", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("Lcap", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float)]

    def replace(self, **kw):
        vals = {f: getattr(self, f) for f, _ in self._fields_}
        vals.update(kw)
        return AttnDesc(**vals)


class DraftLenState(ctypes.Structure):
    """Mirror of `bass_draft_len_state`."""
    _fields_ = [("l_draft", ctypes.c_int32), ("s", ctypes.c_int32)]


class BassError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what} failed: {code} ({bass_status_string(code)})")
        self.code = code


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2404_15778_amd.build` "
                               "(there is no fallback path)")
        # One HIP runtime per process: torch's wheel carries its own copy of libamdhip64, which libbass.so
        # (linked against the soname) shares only if torch has loaded it first.  Loaded the other way round
        # the process holds two runtimes, and kernels launched through one on memory of the other fail.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp = ctypes.POINTER(AttnDesc)
        L.bass_version.restype = ctypes.c_int
        L.bass_status_string.restype = ctypes.c_char_p
        L.bass_status_string.argtypes = [ctypes.c_int]
        L.bass_kv_cache_bytes.restype = sz
        L.bass_kv_cache_bytes.argtypes = [dp]
        L.bass_verify_attention_workspace_bytes.restype = sz
        L.bass_verify_attention_workspace_bytes.argtypes = [dp]
        L.bass_kv_append.restype = ctypes.c_int
        L.bass_kv_append.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bass_kv_gather.restype = ctypes.c_int
        L.bass_kv_gather.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bass_kv_gather_int8.restype = ctypes.c_int
        L.bass_kv_gather_int8.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bass_verify_attention.restype = ctypes.c_int
        L.bass_verify_attention.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
        L.bass_verify_attention_pad.restype = ctypes.c_int
        L.bass_verify_attention_pad.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp, vp]
        L.bass_verify_attention_split.restype = ctypes.c_int
        L.bass_verify_attention_split.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
        L.bass_append_verify_attention.restype = ctypes.c_int
        L.bass_append_verify_attention.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
        L.bass_spec_accept.restype = ctypes.c_int
        L.bass_spec_accept.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bass_warp_probs.restype = ctypes.c_int
        L.bass_warp_probs.argtypes = [i32, i32, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp]
        L.bass_warp_accept_workspace_bytes.restype = ctypes.c_size_t
        L.bass_warp_accept_workspace_bytes.argtypes = [i32, i32, i32]
        L.bass_warp_accept.restype = ctypes.c_int
        L.bass_warp_accept.argtypes = [i32, i32, i32, vp, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp, vp, vp, vp,
                                       ctypes.c_size_t, vp, vp]
        L.bass_draft_len_init.restype = None
        L.bass_draft_len_init.argtypes = [ctypes.POINTER(DraftLenState), i32]
        L.bass_next_draft_len.restype = i32
        L.bass_next_draft_len.argtypes = [ctypes.POINTER(DraftLenState), ctypes.POINTER(i32), i32, i32, i32, i32]
        L.bass_set_attention_waves.restype = ctypes.c_int
        L.bass_set_attention_waves.argtypes = [ctypes.c_int]
        L.bass_attention_plan_bytes.restype = sz
        L.bass_attention_plan_bytes.argtypes = [dp]
        L.bass_attention_plan.restype = ctypes.c_int
        L.bass_attention_plan.argtypes = [dp, vp, vp, i32, i32, vp, sz, vp, vp]
        L.bass_attention_plan_host.restype = ctypes.c_int
        L.bass_attention_plan_host.argtypes = [dp, vp, vp, i32, i32, vp, sz, vp]
        L.bass_verify_attention_noalloc.restype = ctypes.c_int
        L.bass_verify_attention_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.bass_bench_stream_read.restype = ctypes.c_int64
        L.bass_bench_stream_read.argtypes = [vp, vp, sz, i32, vp, vp]
        L.bass_verify_attention_planned.restype = ctypes.c_int
        L.bass_verify_attention_planned.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
        _lib = L
    return _lib


def bass_version() -> int:
    return int(lib().bass_version())


def bass_status_string(code: int) -> str:
    return lib().bass_status_string(int(code)).decode()


def bass_set_attention_waves(waves: int) -> int:
    return int(lib().bass_set_attention_waves(int(waves)))


def bass_draft_len_init(l0: int = 0) -> DraftLenState:
    st = DraftLenState()
    lib().bass_draft_len_init(ctypes.byref(st), int(l0))
    return st


def bass_next_draft_len(state: DraftLenState, n_accept, l_incre: int = 0, l_mod: int = 0, l_limit: int = 0) -> int:
    """Host-side Algorithm 1 update; n_accept is a host sequence of ints."""
    vals = [int(x) for x in n_accept]
    arr = (ctypes.c_int32 * len(vals))(*vals)
    r = int(lib().bass_next_draft_len(ctypes.byref(state), arr, len(vals), int(l_incre), int(l_mod), int(l_limit)))
    _check(r if r < 0 else OK, "bass_next_draft_len")
    return r


def make_desc(B, kmax, Hq, Hkv, D, Lcap, dtype, scale) -> AttnDesc:
    code = {"bf16": DTYPE_BF16, "fp32": DTYPE_FP32, "int8kv": DTYPE_INT8KV}.get(dtype, dtype)
    return AttnDesc(int(B), int(kmax), int(Hq), int(Hkv), int(D), int(Lcap), int(code), float(scale))


def bass_kv_cache_bytes(desc: AttnDesc) -> int:
    return int(lib().bass_kv_cache_bytes(ctypes.byref(desc)))


def bass_verify_attention_workspace_bytes(desc: AttnDesc) -> int:
    return int(lib().bass_verify_attention_workspace_bytes(ctypes.byref(desc)))


# ---- marshalling helpers -------------------------------------------------------------------

def _torch():
    import torch
    return torch


def _elt_dtype(desc):
    torch = _torch()
    return torch.float32 if desc.dtype == DTYPE_FP32 else torch.bfloat16  # INT8 caches: Q and new rows are bf16


def _dev(t, name, dtype=None, shape=None, optional=False):
    """Device pointer of a contiguous CUDA tensor after shape / dtype checks."""
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(getattr(stream, "cuda_stream", stream))


def _check(code, what):
    if code != OK:
        raise BassError(code, what)


def _cache_ptr(t, desc, name):
    if t is None or not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous GPU tensor")
    if t.numel() * t.element_size() < bass_kv_cache_bytes(desc):
        raise ValueError(f"{name} holds fewer than bass_kv_cache_bytes(desc) bytes")
    return ctypes.c_void_p(t.data_ptr())


# ---- entry points (same names and argument order as include/bass.h) --------------------------

def bass_kv_append(desc, Kcache, Vcache, K_new, V_new, ctx_len, n_new, dev_status=None, stream=None):
    torch = _torch()
    rows = (desc.B, desc.kmax, desc.Hkv, desc.D)
    et = _elt_dtype(desc)
    _check(lib().bass_kv_append(
        ctypes.byref(desc), _cache_ptr(Kcache, desc, "Kcache"), _cache_ptr(Vcache, desc, "Vcache"),
        _dev(K_new, "K_new", et, rows), _dev(V_new, "V_new", et, rows),
        _dev(ctx_len, "ctx_len", torch.int32, (desc.B,)), _dev(n_new, "n_new", torch.int32, (desc.B,)),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_kv_append")


def bass_kv_gather(desc, Kcache, Vcache, K_out, V_out, start, n, dev_status=None, stream=None):
    torch = _torch()
    rows = (desc.B, desc.kmax, desc.Hkv, desc.D)
    et = _elt_dtype(desc)
    _check(lib().bass_kv_gather(
        ctypes.byref(desc), _cache_ptr(Kcache, desc, "Kcache"), _cache_ptr(Vcache, desc, "Vcache"),
        _dev(K_out, "K_out", et, rows), _dev(V_out, "V_out", et, rows),
        _dev(start, "start", torch.int32, (desc.B,)), _dev(n, "n", torch.int32, (desc.B,)),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_kv_gather")


def bass_kv_gather_int8(desc, Kcache, Vcache, K_codes, V_codes, K_scales, V_scales, start, n, dev_status=None,
                        stream=None):
    torch = _torch()
    rows = (desc.B, desc.kmax, desc.Hkv, desc.D)
    _check(lib().bass_kv_gather_int8(
        ctypes.byref(desc), _cache_ptr(Kcache, desc, "Kcache"), _cache_ptr(Vcache, desc, "Vcache"),
        _dev(K_codes, "K_codes", torch.int8, rows), _dev(V_codes, "V_codes", torch.int8, rows),
        _dev(K_scales, "K_scales", torch.float32, rows[:3]), _dev(V_scales, "V_scales", torch.float32, rows[:3]),
        _dev(start, "start", torch.int32, (desc.B,)), _dev(n, "n", torch.int32, (desc.B,)),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_kv_gather_int8")


def bass_verify_attention(desc, Q, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace, dev_status=None,
                          stream=None):
    torch = _torch()
    qshape = (desc.B, desc.kmax, desc.Hq, desc.D)
    if workspace is None or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    _check(lib().bass_verify_attention(
        ctypes.byref(desc), _dev(Q, "Q", _elt_dtype(desc), qshape),
        _cache_ptr(Kcache, desc, "Kcache"), _cache_ptr(Vcache, desc, "Vcache"),
        _dev(ctx_len, "ctx_len", torch.int32, (desc.B,)), _dev(draft_len, "draft_len", torch.int32, (desc.B,)),
        _dev(O, "O", torch.float32, qshape), _dev(lse, "lse", torch.float32, qshape[:3], optional=True),
        ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_verify_attention")


def _verify_args(desc, Q, Kcache, Vcache, ctx_len, draft_len):
    torch = _torch()
    qshape = (desc.B, desc.kmax, desc.Hq, desc.D)
    return (ctypes.byref(desc), _dev(Q, "Q", _elt_dtype(desc), qshape),
            _cache_ptr(Kcache, desc, "Kcache"), _cache_ptr(Vcache, desc, "Vcache"),
            _dev(ctx_len, "ctx_len", torch.int32, (desc.B,)), _dev(draft_len, "draft_len", torch.int32, (desc.B,)))


def _result_args(desc, O, lse, workspace, dev_status, stream):
    torch = _torch()
    qshape = (desc.B, desc.kmax, desc.Hq, desc.D)
    if workspace is None or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    return (_dev(O, "O", torch.float32, qshape), _dev(lse, "lse", torch.float32, qshape[:3], optional=True),
            ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
            _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream))


def bass_verify_attention_pad(desc, Q, Kcache, Vcache, ctx_len, draft_len, padded_len, O, lse, workspace,
                              dev_status=None, stream=None):
    _check(lib().bass_verify_attention_pad(
        *_verify_args(desc, Q, Kcache, Vcache, ctx_len, draft_len), ctypes.c_int32(int(padded_len)),
        *_result_args(desc, O, lse, workspace, dev_status, stream)), "bass_verify_attention_pad")


def bass_verify_attention_split(desc, Q, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace, dev_status=None,
                                stream=None):
    _check(lib().bass_verify_attention_split(
        *_verify_args(desc, Q, Kcache, Vcache, ctx_len, draft_len),
        *_result_args(desc, O, lse, workspace, dev_status, stream)), "bass_verify_attention_split")


def bass_append_verify_attention(desc, Q, K_new, V_new, Kcache, Vcache, ctx_len, draft_len, O, lse, workspace,
                                 dev_status=None, stream=None):
    torch = _torch()
    qshape = (desc.B, desc.kmax, desc.Hq, desc.D)
    rows = (desc.B, desc.kmax, desc.Hkv, desc.D)
    et = _elt_dtype(desc)
    if workspace is None or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    _check(lib().bass_append_verify_attention(
        ctypes.byref(desc), _dev(Q, "Q", et, qshape), _dev(K_new, "K_new", et, rows), _dev(V_new, "V_new", et, rows),
        _cache_ptr(Kcache, desc, "Kcache"), _cache_ptr(Vcache, desc, "Vcache"),
        _dev(ctx_len, "ctx_len", torch.int32, (desc.B,)), _dev(draft_len, "draft_len", torch.int32, (desc.B,)),
        _dev(O, "O", torch.float32, qshape), _dev(lse, "lse", torch.float32, qshape[:3], optional=True),
        ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_append_verify_attention")


NOALLOC_SCRATCH_BYTES = 16 << 20  # BASS_NOALLOC_SCRATCH_BYTES of include/bass.h


def bass_verify_attention_noalloc(desc, Q, Kcache, Vcache, ctx_len, draft_len, O, lse, dev_status=None, stream=None):
    torch = _torch()
    qshape = (desc.B, desc.kmax, desc.Hq, desc.D)
    _check(lib().bass_verify_attention_noalloc(
        *_verify_args(desc, Q, Kcache, Vcache, ctx_len, draft_len),
        _dev(O, "O", torch.float32, qshape), _dev(lse, "lse", torch.float32, qshape[:3], optional=True),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_verify_attention_noalloc")


def bass_attention_plan_bytes(desc: AttnDesc) -> int:
    return int(lib().bass_attention_plan_bytes(ctypes.byref(desc)))


def bass_attention_plan(desc, ctx_len, draft_len, flags, padded_len, plan, dev_status=None, stream=None):
    torch = _torch()
    if plan is None or not plan.is_cuda or not plan.is_contiguous():
        raise ValueError("plan must be a contiguous GPU tensor")
    _check(lib().bass_attention_plan(
        ctypes.byref(desc), _dev(ctx_len, "ctx_len", torch.int32, (desc.B,)),
        _dev(draft_len, "draft_len", torch.int32, (desc.B,)), ctypes.c_int32(int(flags)), ctypes.c_int32(int(padded_len)),
        ctypes.c_void_p(plan.data_ptr()), ctypes.c_size_t(plan.numel() * plan.element_size()),
        _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)), "bass_attention_plan")


def bass_attention_plan_host(desc, ctx_len, draft_len, flags=0, padded_len=0):
    """Host planner: ctx_len / draft_len are host sequences of ints; returns (plan bytes as a numpy uint8 array,
    host status word).  Needs no GPU."""
    import numpy as np
    cl = np.ascontiguousarray(np.asarray(ctx_len, dtype=np.int32))
    dl = np.ascontiguousarray(np.asarray(draft_len, dtype=np.int32))
    if cl.shape != (desc.B,) or dl.shape != (desc.B,):
        raise ValueError("ctx_len and draft_len must have B entries")
    nbytes = bass_attention_plan_bytes(desc)
    buf = np.zeros(nbytes + 16, dtype=np.uint8)
    off = (-buf.ctypes.data) % 16  # the entry point wants 16-byte alignment
    plan = buf[off:off + nbytes]
    status = ctypes.c_int32(0)
    _check(lib().bass_attention_plan_host(
        ctypes.byref(desc), ctypes.c_void_p(cl.ctypes.data), ctypes.c_void_p(dl.ctypes.data), ctypes.c_int32(int(flags)),
        ctypes.c_int32(int(padded_len)), ctypes.c_void_p(plan.ctypes.data), ctypes.c_size_t(nbytes),
        ctypes.cast(ctypes.byref(status), ctypes.c_void_p)), "bass_attention_plan_host")
    return plan, int(status.value)


def bass_verify_attention_planned(desc, Q, K_new, V_new, Kcache, Vcache, plan, O, lse, workspace, dev_status=None,
                                  stream=None):
    torch = _torch()
    qshape = (desc.B, desc.kmax, desc.Hq, desc.D)
    rows = (desc.B, desc.kmax, desc.Hkv, desc.D)
    et = _elt_dtype(desc)
    if plan is None or not plan.is_cuda or not plan.is_contiguous():
        raise ValueError("plan must be a contiguous GPU tensor")
    if plan.numel() * plan.element_size() < bass_attention_plan_bytes(desc):
        raise ValueError("plan holds fewer than bass_attention_plan_bytes(desc) bytes")
    _check(lib().bass_verify_attention_planned(
        ctypes.byref(desc), _dev(Q, "Q", et, qshape), _dev(K_new, "K_new", et, rows, optional=True),
        _dev(V_new, "V_new", et, rows, optional=True), _cache_ptr(Kcache, desc, "Kcache"),
        _cache_ptr(Vcache, desc, "Vcache"), ctypes.c_void_p(plan.data_ptr()),
        *_result_args(desc, O, lse, workspace, dev_status, stream)), "bass_verify_attention_planned")


def bass_bench_stream_read(K, V, bytes_each, waves, sink=None, stream=None) -> int:
    """Plain streaming read of the first bytes_each bytes of the byte tensors K and V; returns the bytes read."""
    for t, name in ((K, "K"), (V, "V")):
        if t is None or not t.is_cuda or not t.is_contiguous() or t.numel() * t.element_size() < bytes_each:
            raise ValueError(f"{name} must be a contiguous GPU tensor of at least bytes_each bytes")
    r = int(lib().bass_bench_stream_read(ctypes.c_void_p(K.data_ptr()), ctypes.c_void_p(V.data_ptr()),
                                         ctypes.c_size_t(int(bytes_each)), ctypes.c_int32(int(waves)),
                                         _dev(sink, "sink", _torch().int32, optional=True), _stream(stream)))
    _check(r if r < 0 else OK, "bass_bench_stream_read")
    return r


def alloc_plan(desc, device="cuda"):
    """A plan buffer (bass_attention_plan fills it; it needs no clearing)."""
    torch = _torch()
    return torch.empty(bass_attention_plan_bytes(desc), dtype=torch.uint8, device=device)


def bass_spec_accept(p, q, draft_tok, n_draft, u, n_accept, next_token, ctx_len=None, dev_status=None, stream=None):
    torch = _torch()
    if p is None or p.dim() != 3:
        raise ValueError("p must be [B, kmax+1, V]")
    B, k1, V = p.shape
    kmax = k1 - 1
    f32, i32 = torch.float32, torch.int32
    _check(lib().bass_spec_accept(
        B, kmax, V, _dev(p, "p", f32), _dev(q, "q", f32, (B, kmax, V), optional=(kmax == 0)),
        _dev(draft_tok, "draft_tok", i32, (B, kmax), optional=(kmax == 0)), _dev(n_draft, "n_draft", i32, (B,)),
        _dev(u, "u", f32, (B, kmax + 1)), _dev(n_accept, "n_accept", i32, (B,)),
        _dev(next_token, "next_token", i32, (B,)), _dev(ctx_len, "ctx_len", i32, (B,), optional=True),
        _dev(dev_status, "dev_status", i32, optional=True), _stream(stream)), "bass_spec_accept")


def bass_warp_probs(logits, temperature, top_p, probs, dev_status=None, stream=None):
    """logits [..., V] fp32 -> probs of the same shape (temperature, nucleus top-p, softmax)."""
    torch = _torch()
    if logits is None or logits.dim() < 1:
        raise ValueError("logits must be [..., V]")
    V = int(logits.shape[-1])
    R = int(logits.numel() // max(V, 1))
    shape = tuple(logits.shape)
    lp, pp = _dev(logits, "logits", torch.float32, shape), _dev(probs, "probs", torch.float32, shape)
    if lp.value == pp.value:
        raise ValueError("probs may not alias logits")
    _check(lib().bass_warp_probs(R, V, lp, ctypes.c_float(float(temperature)), ctypes.c_float(float(top_p)), pp,
                                 _dev(dev_status, "dev_status", torch.int32, optional=True), _stream(stream)),
           "bass_warp_probs")


def bass_warp_accept_workspace_bytes(B, kmax, V):
    return int(lib().bass_warp_accept_workspace_bytes(int(B), int(kmax), int(V)))


def bass_warp_accept(logits_main, logits_draft, temperature, top_p, draft_tok, n_draft, u, n_accept, next_token,
                     workspace, ctx_len=None, dev_status=None, stream=None):
    """logits_main [B, kmax+1, V], logits_draft [B, kmax, V] fp32 -> n_accept, next_token (ctx_len advanced):
    bass_warp_probs on both tensors followed by bass_spec_accept, without the probability rows."""
    torch = _torch()
    if logits_main is None or logits_main.dim() != 3:
        raise ValueError("logits_main must be [B, kmax+1, V]")
    B, k1, V = logits_main.shape
    kmax = k1 - 1
    f32, i32 = torch.float32, torch.int32
    wsp = _dev(workspace, "workspace", torch.uint8)
    _check(lib().bass_warp_accept(
        B, kmax, V, _dev(logits_main, "logits_main", f32),
        _dev(logits_draft, "logits_draft", f32, (B, kmax, V), optional=(kmax == 0)),
        ctypes.c_float(float(temperature)), ctypes.c_float(float(top_p)),
        _dev(draft_tok, "draft_tok", i32, (B, kmax), optional=(kmax == 0)), _dev(n_draft, "n_draft", i32, (B,)),
        _dev(u, "u", f32, (B, kmax + 1)), _dev(n_accept, "n_accept", i32, (B,)),
        _dev(next_token, "next_token", i32, (B,)), _dev(ctx_len, "ctx_len", i32, (B,), optional=True),
        wsp, ctypes.c_size_t(workspace.numel()), _dev(dev_status, "dev_status", i32, optional=True), _stream(stream)),
        "bass_warp_accept")


# ---- allocation helpers (plumbing; no arithmetic) ----------------------------------------------

def alloc_kv_cache(desc, device="cuda", fill_byte=None):
    """One cache (K or V) as an opaque byte tensor; optionally filled with a byte pattern."""
    torch = _torch()
    t = torch.empty(bass_kv_cache_bytes(desc), dtype=torch.uint8, device=device)
    if fill_byte is not None:
        t.fill_(fill_byte)
    return t


def alloc_workspace(desc, device="cuda"):
    """Attention workspace, zeroed once as the header requires (calls leave its counters zero)."""
    torch = _torch()
    return torch.zeros(bass_verify_attention_workspace_bytes(desc), dtype=torch.uint8, device=device)
