"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
sizes caches / workspaces on the host, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2404_15778_amd as bass

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if not os.path.exists(bass.LIB_PATH):
        from paper_2404_15778_amd import build
        build.build()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bass.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bass_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree_on_the_export_list():
    assert declared_functions() == sorted(bass.EXPORTS)


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(bass.LIB_PATH)
    for name in declared_functions():
        assert hasattr(L, name), name


def test_version_and_status_strings():
    assert bass.bass_version() >= 100
    assert bass.bass_status_string(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert bass.bass_status_string(code) not in ("ok", "unknown status")


def test_cache_and_workspace_sizes():
    d = bass.make_desc(8, 6, 32, 32, 128, 2056, "bf16", 0.1)
    # bf16 caches are stored in whole 32-token blocks
    assert bass.bass_kv_cache_bytes(d) == 8 * 32 * 65 * 32 * 128 * 2
    assert bass.bass_verify_attention_workspace_bytes(d) > 0
    f = bass.make_desc(2, 4, 4, 4, 64, 100, "fp32", 0.125)
    assert bass.bass_kv_cache_bytes(f) == 2 * 4 * 100 * 64 * 4


@pytest.mark.parametrize("kw", [dict(B=0), dict(kmax=0), dict(Hkv=3), dict(Lcap=0), dict(D=0)])
def test_invalid_shapes_are_rejected_on_the_host(kw):
    d = bass.make_desc(2, 4, 4, 2, 64, 100, "bf16", 0.125).replace(**kw)
    assert bass.bass_kv_cache_bytes(d) == 0
    assert bass.bass_verify_attention_workspace_bytes(d) == 0
    rc = bass.lib().bass_verify_attention(ctypes.byref(d), None, None, None, None, None, None, None, None, 0, None, None)
    assert rc == bass.ERR_INVALID_ARG


def test_unsupported_shapes():
    d = bass.make_desc(2, 4, 4, 2, 96, 100, "bf16", 0.125)       # bf16 head size must be 64 or 128
    assert bass.lib().bass_kv_append(ctypes.byref(d), None, None, None, None, None, None, None, None) == bass.ERR_UNSUPPORTED
    d = bass.make_desc(2, 4, 4, 2, 64, 100, 7, 0.125)             # unknown dtype
    assert bass.bass_kv_cache_bytes(d) == 0
    one = ctypes.c_void_p(16)  # never dereferenced: the checks below fail before any launch
    d = bass.make_desc(2, 9, 64, 8, 128, 100, "bf16", 0.125)      # 72 query rows per kv head > 64
    assert bass.lib().bass_verify_attention(ctypes.byref(d), one, one, one, one, one, one, None, one, 1 << 40, None, None) == bass.ERR_UNSUPPORTED
    assert bass.lib().bass_spec_accept(1, 1, (1 << 19) + 1, one, one, one, one, one, one, one, None, None, None) == bass.ERR_UNSUPPORTED


def test_null_pointers_and_small_workspace():
    d = bass.make_desc(2, 4, 4, 2, 64, 100, "bf16", 0.125)
    one = ctypes.c_void_p(16)
    L = bass.lib()
    assert L.bass_verify_attention(ctypes.byref(d), one, one, None, one, one, one, None, one, 1 << 40, None, None) == bass.ERR_INVALID_ARG
    assert L.bass_verify_attention(ctypes.byref(d), one, one, one, one, one, one, None, one, 8, None, None) == bass.ERR_WORKSPACE_TOO_SMALL
    assert L.bass_verify_attention(ctypes.byref(d), one, one, one, one, one, one, None, ctypes.c_void_p(8), 1 << 40, None, None) == bass.ERR_INVALID_ARG
    assert L.bass_kv_append(ctypes.byref(d), one, one, one, None, one, one, None, None) == bass.ERR_INVALID_ARG
    assert L.bass_spec_accept(0, 1, 8, one, one, one, one, one, one, one, None, None, None) == bass.ERR_INVALID_ARG
    assert L.bass_spec_accept(1, 1, 8, one, None, one, one, one, one, one, None, None, None) == bass.ERR_INVALID_ARG


def test_attention_waves_knob_is_clamped():
    assert bass.bass_set_attention_waves(1) == 64
    assert bass.bass_set_attention_waves(10**6) == 8192
    assert bass.bass_set_attention_waves(1022) == 1020
    assert bass.bass_set_attention_waves(0) == 768


def test_kernel_times_summarize_reads_a_kernel_trace(tmp_path, capsys):
    """Host logic of the timing utility: groups a rocprofv3 kernel trace by kernel, grid and registers."""
    import argparse
    from paper_2404_15778_amd import kernel_times
    trace = tmp_path / "t_kernel_trace.csv"
    trace.write_text(
        "Kernel_Name,Grid_Size_X,VGPR_Count,Start_Timestamp,End_Timestamp\n"
        '"void bass::verify_attn_bf16<128, 1, false>(bass::AttnParams)",49152,256,1000,33000\n'
        '"void bass::verify_attn_bf16<128, 1, false>(bass::AttnParams)",49152,256,40000,70000\n'
        '"void at::native::fill(int)",64,8,0,5\n')
    kernel_times.summarize(argparse.Namespace(trace=str(trace)))
    out = capsys.readouterr().out.strip().splitlines()
    assert len(out) == 1 and "verify_attn_bf16<128, 1, false>" in out[0]
    assert "n=2" in out[0] and "avg 31.00 us" in out[0] and "min 30.00 us" in out[0]


def test_recorded_hbm_traffic_belongs_to_this_library_version():
    """bench.py reports roofline.traffic only from a counter summary made with the library it times: the
    summary under profiles/ must carry the current version, and its figure must be a plausible multiple of
    the algorithmic bytes of the benchmark launch (cfg2, seed 0)."""
    import importlib.util
    import workloads as wl
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    traffic = bench.measured_traffic(bass.bass_version())
    assert traffic is not None, "profiles/verify_attn_bf16_cfg2_hbm_traffic.txt was made with another library version"
    w = wl.config2(0, tensors=False)
    algorithmic = int((w.ctx_len + w.draft_len).sum()) * 2 * w.Hkv * w.D * 2
    assert algorithmic == 158515200
    assert 1.0 <= traffic / algorithmic <= 1.15
    assert bench.measured_traffic(bass.bass_version() + 1) is None


def test_one_hip_runtime_whatever_is_imported_first():
    """torch's wheel ships its own HIP runtime; the process must end up with that one alone, also when the
    binding is used before torch was imported (two runtimes: launches through one on memory of the other fail)."""
    import subprocess
    import sys
    code = (
        "import os, sys\n"
        f"sys.path.insert(0, {ROOT!r})\n"
        "import paper_2404_15778_amd as bass\n"
        "assert bass.bass_version() >= 100\n"
        "import torch\n"
        "paths = {l.split()[-1] for l in open(f'/proc/{os.getpid()}/maps') if 'libamdhip64' in l}\n"
        "print(len(paths), sorted(paths))\n"
    )
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.split()[0] == "1", out.stdout


def test_inline_assembly_is_limited_to_wait_counts():
    """The compiler inserts the wait states some instruction pairs need (a vector-memory instruction behind a
    vector instruction that wrote its scalar address, ...) only for instructions it emits itself, not for
    opaque assembly text.  The kernels therefore contain no instruction written as inline assembly except
    `s_waitcnt vmcnt(0)`, which has no operands; empty assembly strings (optimisation barriers) are fine."""
    import glob
    found = []
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2404_15778_amd", "csrc", "*"))):
        text = open(path).read()
        for m in re.finditer(r'\basm\s+volatile\s*\(\s*"((?:[^"\\]|\\.)*)"', text):
            found.append((os.path.basename(path), m.group(1)))
        # every asm statement is of the form matched above
        assert len(re.findall(r'\basm\b', re.sub(r'//[^\n]*', '', text))) == len(
            re.findall(r'\basm\s+volatile\s*\(\s*"', re.sub(r'//[^\n]*', '', text))), path
    assert found, "the sources are expected to hold the explicit acknowledgement waits"
    for name, body in found:
        assert body in ("", "s_waitcnt vmcnt(0)"), (name, body)


def test_benchmark_refuses_more_than_one_gpu():
    """The build runs on one GPU; asking the benchmark for more ends with a message, before any GPU is touched."""
    import subprocess
    import sys
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert out.returncode == 2
    assert "ONE GPU" in out.stderr and out.stdout.strip() == ""
