"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2601_18401_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)       # non-null, 16-byte aligned, never dereferenced on these paths
FAKE_WS = ctypes.c_void_p(0x10000)


def good(**kw):
    p = B.SlParams()
    p.L, p.Lq, p.q_pos0 = 4096, 4096, 0
    p.Hq, p.Hkv, p.D, p.S, p.topk, p.dtype = 8, 2, 128, 64, 4, B.SL_BF16
    p.scale = 0.0
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_library_exports_every_declared_symbol():
    lib = B.load()
    header = open(os.path.join(ROOT, "include", "sl.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sl_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.sl_version() >= 100
    assert B.status_string(0) == "SL_OK"
    for s in range(1, 5):
        assert B.status_string(s).startswith("SL_ERR_")


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 and as C++ on its own."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "sl.h")
    if shutil.which("gcc"):
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                       check=True)
    if shutil.which("g++"):
        subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr], check=True)


def test_library_is_callable_from_plain_c(tmp_path):
    """A C99 program includes sl.h, loads libsl.so and calls the host-only entry points."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    B.load()   # raises if the library has not been built
    exe = str(tmp_path / "call_from_c")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "cabi", "call_from_c.c"), "-o", exe, "-ldl"], check=True)
    out = subprocess.run([exe, B.LIB_PATH], check=True, capture_output=True, text=True).stdout
    assert "ok=SL_OK" in out and "bad=SL_ERR_INVALID_ARG" in out, out


def test_validation_layer_under_address_and_undefined_sanitizers(tmp_path):
    """The host side of the library (validation, size arithmetic) built with ASan + UBSan, driven by
    a C program built the same way through every rejection path; nothing is launched."""
    import glob
    import shutil
    import subprocess
    from paper_2601_18401_amd import build as _build
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not os.path.exists(clang) or not shutil.which("hipcc"):
        pytest.skip("no ROCm clang")
    lib = _build.build(sanitize=True)
    exe = str(tmp_path / "validate_from_c")
    subprocess.run([clang, "-std=c99", "-Wall", "-Wextra", "-Werror", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", "-shared-libsan", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "cabi", "validate_from_c.c"), "-o", exe, "-ldl"], check=True)
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux")[0]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               LD_LIBRARY_PATH=rt + ":" + os.environ.get("LD_LIBRARY_PATH", ""))
    run = subprocess.run([exe, lib], capture_output=True, text=True, env=env)
    assert run.returncode == 0 and "failures=0" in run.stdout, (run.stdout, run.stderr[-3000:])
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-3000:]


def test_struct_layouts_match_the_header():
    # sl_anchor_geometry: int64 + 4 x int32; sl_decode_seq: 9 pointers + int64
    assert ctypes.sizeof(B.SlAnchorGeometry) == 24
    assert ctypes.sizeof(B.SlDecodeSeq) == 80
    assert B.SlDecodeSeq.L.offset == 72 and B.SlDecodeSeq.idx.offset == 40


def test_params_struct_matches_header_size():
    # 3 x int64, 6 x int32, float, int32, 4 x int64
    assert ctypes.sizeof(B.SlParams) == 24 + 24 + 8 + 32


BAD = [
    (dict(L=0), 1), (dict(Lq=0), 1), (dict(q_pos0=-1), 1), (dict(q_pos0=1), 1),
    (dict(Hq=0), 1), (dict(Hkv=3), 1), (dict(S=0), 1), (dict(topk=-1), 1), (dict(dtype=7), 1),
    (dict(scale=-1.0), 1), (dict(scale=float("inf")), 1), (dict(scale=float("nan")), 1),
    (dict(D=96), 2), (dict(topk=B.SL_MAX_TOPK + 1), 2), (dict(Hq=130, Hkv=2), 2),
    (dict(q_stride_t=64), 1), (dict(kv_stride_t=129), 1), (dict(q_stride_h=4), 1),
    (dict(span_stride=-1), 1), (dict(span_stride=65), 1),      # anchor spacing must be within [0, S]
]


@pytest.mark.parametrize("kw,status", BAD)
def test_invalid_params_rejected_before_launch(kw, status):
    lib = B.load()
    p = good(**kw)
    for fn in (lib.sl_span_search_prefill, ):
        assert fn(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, None, FAKE_WS, 1 << 40, None) == status
    assert lib.sl_span_attention_prefill(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                         FAKE_WS, 1 << 40, None) == status
    assert lib.sl_workspace_bytes(ctypes.byref(p), B.OP_ATTENTION_DECODE) == B.WORKSPACE_INVALID


def test_null_and_misaligned_pointers():
    lib = B.load()
    p = good()
    odd = ctypes.c_void_p(0x1004)
    assert lib.sl_span_search_prefill(None, FAKE, FAKE, FAKE, FAKE, None, FAKE_WS, 1 << 40, None) == 1
    assert lib.sl_span_search_prefill(ctypes.byref(p), None, FAKE, FAKE, FAKE, None, FAKE_WS, 1 << 40, None) == 1
    assert lib.sl_span_search_prefill(ctypes.byref(p), FAKE, None, None, FAKE, None, FAKE_WS, 1 << 40, None) == 1
    assert lib.sl_span_search_prefill(ctypes.byref(p), FAKE, FAKE, FAKE, None, None, FAKE_WS, 1 << 40, None) == 1
    assert lib.sl_span_search_prefill(ctypes.byref(p), odd, FAKE, FAKE, FAKE, None, FAKE_WS, 1 << 40, None) == 1
    for pos in range(6):
        args = [FAKE] * 6
        args[pos] = None
        assert lib.sl_span_attention_prefill(ctypes.byref(p), *args, FAKE_WS, 1 << 40, None) == 1
        args[pos] = odd
        assert lib.sl_span_attention_prefill(ctypes.byref(p), *args, FAKE_WS, 1 << 40, None) == 1
    assert lib.sl_span_keys(None, FAKE, FAKE, None) == 1
    assert lib.sl_span_keys(ctypes.byref(p), None, FAKE, None) == 1


def test_decode_requires_single_query_row_and_search_needs_topk():
    lib = B.load()
    p = good()
    assert lib.sl_span_search_decode(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, None, FAKE_WS, 1 << 40, None) == 1
    assert lib.sl_span_attention_decode(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE_WS, 1 << 40, None) == 1
    p = good(topk=0)
    assert lib.sl_span_search_prefill(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, None, FAKE_WS, 1 << 40, None) == 1


def test_workspace_checks():
    lib = B.load()
    p = good(Lq=1, q_pos0=4095)
    need = lib.sl_workspace_bytes(ctypes.byref(p), B.OP_ATTENTION_DECODE)
    assert need > 0
    args = [FAKE] * 6
    assert lib.sl_span_attention_decode(ctypes.byref(p), *args, None, 0, None) == 3
    assert lib.sl_span_attention_decode(ctypes.byref(p), *args, FAKE_WS, need - 1, None) == 3
    assert lib.sl_span_attention_decode(ctypes.byref(p), *args, ctypes.c_void_p(0x10010), need, None) == 3
    # decode search: one fp32 score row per head, whole 256-byte lines
    assert lib.sl_workspace_bytes(ctypes.byref(p), B.OP_SEARCH_DECODE) == p.Hq * 64 * ((-(-p.L // p.S) + 63) // 64) * 4


def test_batched_decode_argument_checks():
    lib = B.load()
    assert ctypes.sizeof(B.SlDecodeSeq) == 80          # 9 pointers + int64
    p = good(Lq=1, q_pos0=4095)
    need = lib.sl_decode_batched_workspace_bytes(ctypes.byref(p), 3)
    assert need > 0 and need % 3 == 0
    assert lib.sl_decode_batched_workspace_bytes(ctypes.byref(p), 0) == B.WORKSPACE_INVALID
    assert lib.sl_decode_batched_workspace_bytes(ctypes.byref(good()), 3) == B.WORKSPACE_INVALID     # Lq != 1
    assert lib.sl_span_search_decode_batched(ctypes.byref(p), None, 3, None) == 1
    assert lib.sl_span_search_decode_batched(ctypes.byref(p), FAKE, 0, None) == 1
    assert lib.sl_span_search_decode_batched(ctypes.byref(p), ctypes.c_void_p(0x1004), 3, None) == 1
    assert lib.sl_span_search_decode_batched(ctypes.byref(good()), FAKE, 3, None) == 1
    big = good(L=64 * 13000, Lq=1, q_pos0=64 * 13000 - 1)                            # > 12288 spans
    assert lib.sl_span_search_decode_batched(ctypes.byref(big), FAKE, 3, None) == 2
    assert lib.sl_span_attention_decode_batched(ctypes.byref(p), FAKE, 3, None, 0, None) == 3
    assert lib.sl_span_attention_decode_batched(ctypes.byref(p), FAKE, 3, FAKE_WS, need - 1, None) == 3
    assert lib.sl_span_attention_decode_batched(ctypes.byref(p), FAKE, 0, FAKE_WS, need, None) == 1


def test_batched_combination_and_anchor_argument_checks():
    lib = B.load()
    p = good(Lq=1, q_pos0=4095)
    g = B.SlAnchorGeometry(1088, 4, 2, 2, 0)
    bad_g = B.SlAnchorGeometry(1088, 4, 2, 5, 0)          # exponent 1/5 is not offered
    need = lib.sl_anchor_batched_workspace_bytes(ctypes.byref(p), ctypes.byref(g), 2)
    assert need > 0
    assert lib.sl_anchor_batched_workspace_bytes(ctypes.byref(p), ctypes.byref(bad_g), 2) == B.WORKSPACE_INVALID
    assert lib.sl_anchor_batched_workspace_bytes(ctypes.byref(p), ctypes.byref(g), 0) == B.WORKSPACE_INVALID
    assert lib.sl_anchor_search_decode_batched(ctypes.byref(p), ctypes.byref(g), None, 2, None) == 1
    assert lib.sl_anchor_search_decode_batched(ctypes.byref(p), ctypes.byref(bad_g), FAKE, 2, None) == 1
    assert lib.sl_anchor_search_decode_batched(ctypes.byref(good()), ctypes.byref(g), FAKE, 2, None) == 1
    assert lib.sl_anchor_attention_decode_batched(ctypes.byref(p), ctypes.byref(g), FAKE, 2, FAKE_WS, need - 1, None) == 3
    assert lib.sl_anchor_attention_decode_batched(ctypes.byref(p), ctypes.byref(g), FAKE, 0, FAKE_WS, need, None) == 1
    need_c = lib.sl_decode_batched_workspace_bytes(ctypes.byref(p), 2)
    assert lib.sl_span_attention_combined_decode_batched(ctypes.byref(p), FAKE, 2, None, 0, None) == 3
    assert lib.sl_span_attention_combined_decode_batched(ctypes.byref(p), None, 2, FAKE_WS, need_c, None) == 1


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.load()


def test_workloads_are_seeded_and_shaped():
    import torch
    from paper_2601_18401_amd import workloads as W
    cfg = W.CONFIGS["C4"].scaled(L=4096, S=64)
    a = W.generate(cfg)
    b = W.generate(cfg)
    assert torch.equal(a["K"], b["K"]) and torch.equal(a["Q"], b["Q"])
    assert a["Q"].shape == (32, 4096, 128) and a["K"].shape == (4, 4096, 128)
    assert a["K"].dtype == torch.bfloat16
    assert len(set(a["needle_spans"].tolist())) == 16
    d = W.generate(W.CONFIGS["C3"].scaled(L=8192, S=128), n_queries=3)
    assert d["Q"].shape == (3, 32, 1, 128)
    assert [W.CONFIGS[c].n_spans for c in ("C1", "C2", "C3", "C4", "C5")] == [64, 256, 1024, 512, 2560]
