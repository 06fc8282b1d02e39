"""CPU-side checks of the boundary: the shared library loads and exports every symbol the header
declares; the Python parameter block mirrors the C struct; no compute is called here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ttt_attn.h")


@pytest.fixture(scope="module")
def lib_path():
    from paper_2603_18567_amd.build import LIB_PATH, build_library
    if not os.path.exists(LIB_PATH):
        build_library()
    return LIB_PATH


def declared_functions():
    """Every function that any header under include/ declares."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, fn)).read(), flags=re.S)
            names |= set(re.findall(r"\b(ttt_(?:attn|loss|qkv|o)_\w+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_entry_points():
    names = declared_functions()
    for need in ("ttt_attn_fwd", "ttt_attn_bwd", "ttt_attn_workspace_bytes", "ttt_attn_last_error"):
        assert need in names


def test_library_exports_every_declared_symbol(lib_path):
    lib = ctypes.CDLL(lib_path)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared under include/ but not exported"
    from paper_2603_18567_amd.binding import EXPORTS
    assert sorted(EXPORTS) == declared_functions()


def test_param_struct_mirrors_the_header():
    from paper_2603_18567_amd.binding import TttAttnParams
    text = open(HEADER).read()
    body = re.search(r"typedef struct ttt_attn_params \{(.*?)\} ttt_attn_params;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|int64_t|float)\s+(\w+)\s*;", body)
    ctype = {"int32_t": ctypes.c_int32, "int64_t": ctypes.c_int64, "float": ctypes.c_float}
    assert [(n, ctype[t]) for t, n in fields] == list(TttAttnParams._fields_)
    assert ctypes.sizeof(TttAttnParams) == 72


def test_constants_match_the_header():
    from paper_2603_18567_amd import binding as B
    text = open(HEADER).read()
    for name in ("TTT_OK", "TTT_ERR_INVALID_ARG", "TTT_ERR_UNSUPPORTED", "TTT_ERR_WORKSPACE", "TTT_ERR_HIP",
                 "TTT_F32", "TTT_BF16", "TTT_PASS_FWD", "TTT_PASS_BWD", "TTT_PASS_BWD_ACCUM"):
        m = re.search(rf"\b{name}\s*=\s*(-?\d+)", text)
        assert m and int(m.group(1)) == getattr(B, name), name
    assert int(re.search(r"#define TTT_MAX_STEPS (\d+)", text).group(1)) == B.TTT_MAX_STEPS


def test_workspace_query_and_argument_errors_need_no_gpu(lib_path):
    """Validation happens on the host before any HIP call: exercise it without a device."""
    from paper_2603_18567_amd import binding as B
    lib = B.load_library()
    p = B.TttAttnParams(B.TTT_BF16, 7, 0, 7, 4096, 1, 32, 8, 128, 0.0883883, 4096, 128, 1024, 128)
    n = lib.ttt_attn_workspace_bytes(ctypes.byref(p), B.TTT_PASS_FWD)
    assert n >= 2 * 4096 * 4
    nb = lib.ttt_attn_workspace_bytes(ctypes.byref(p), B.TTT_PASS_BWD)
    na = lib.ttt_attn_workspace_bytes(ctypes.byref(p), B.TTT_PASS_BWD_ACCUM)
    assert n < nb < na
    assert na - nb >= 2 * 6 * 4096 * 8 * 128 * 4
    bad = B.TttAttnParams(B.TTT_BF16, 7, 0, 7, 4096, 1, 32, 5, 128, 0.0883883, 4096, 128, 1024, 128)
    assert lib.ttt_attn_workspace_bytes(ctypes.byref(bad), B.TTT_PASS_FWD) == 0
    assert "hkv" in B.ttt_attn_last_error()
    for field, val, code in (("k", 0, B.TTT_ERR_INVALID_ARG), ("k", 33, B.TTT_ERR_INVALID_ARG),
                             ("head_dim", 96, B.TTT_ERR_UNSUPPORTED), ("dtype", 5, B.TTT_ERR_UNSUPPORTED),
                             ("step_end", 9, B.TTT_ERR_INVALID_ARG), ("q_stride_head", 100, B.TTT_ERR_INVALID_ARG),
                             ("softmax_scale", 0.0, B.TTT_ERR_INVALID_ARG)):
        q = B.TttAttnParams.from_buffer_copy(p)
        setattr(q, field, val)
        null = ctypes.POINTER(ctypes.c_void_p)()
        rc = lib.ttt_attn_fwd(ctypes.byref(q), null, null, null, None, None, null, null, None, 0, None)
        assert rc == code, (field, rc, B.ttt_attn_last_error())
    # valid params, NULL arrays / bad cu_seqlens / missing workspace are still host-side errors
    null = ctypes.POINTER(ctypes.c_void_p)()
    assert lib.ttt_attn_fwd(ctypes.byref(p), null, null, null, None, None, null, null, None, 0, None) == B.TTT_ERR_INVALID_ARG
    arr = (ctypes.c_void_p * 7)()
    cu_bad = (ctypes.c_int32 * 2)(0, 4000)
    rc = lib.ttt_attn_fwd(ctypes.byref(p), arr, arr, arr, ctypes.c_void_p(256), cu_bad, arr, arr, None, 0, None)
    assert rc == B.TTT_ERR_INVALID_ARG and "total_tokens" in B.ttt_attn_last_error()
    cu = (ctypes.c_int32 * 2)(0, 4096)
    rc = lib.ttt_attn_fwd(ctypes.byref(p), arr, arr, arr, ctypes.c_void_p(256), cu, arr, arr, None, 0, None)
    assert rc == B.TTT_ERR_INVALID_ARG and "NULL" in B.ttt_attn_last_error()
    for i in range(7):
        arr[i] = 4096 * (i + 1)
    rc = lib.ttt_attn_fwd(ctypes.byref(p), arr, arr, arr, ctypes.c_void_p(256), cu, arr, arr, None, 0, None)
    assert rc == B.TTT_ERR_WORKSPACE
    arr[3] = 4096 * 4 + 8
    rc = lib.ttt_attn_fwd(ctypes.byref(p), arr, arr, arr, ctypes.c_void_p(256), cu, arr, arr, ctypes.c_void_p(512), 1 << 30, None)
    assert rc == B.TTT_ERR_INVALID_ARG and "aligned" in B.ttt_attn_last_error()
    # empty problems are successful no-ops
    empty = B.TttAttnParams(B.TTT_BF16, 7, 0, 7, 0, 0, 32, 8, 128, 0.0883883, 4096, 128, 1024, 128)
    cu0 = (ctypes.c_int32 * 1)(0)
    assert lib.ttt_attn_fwd(ctypes.byref(empty), arr, arr, arr, ctypes.c_void_p(256), cu0, arr, arr, None, 0, None) == B.TTT_OK
    assert lib.ttt_attn_bwd(ctypes.byref(empty), arr, arr, arr, arr, arr, arr, ctypes.c_void_p(256), cu0, arr, arr, arr, 0, None, 0, None) == B.TTT_OK


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2603_18567_amd import binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        B.load_library()


def test_workload_table_matches_the_stated_configs():
    from paper_2603_18567_amd.workloads import WORKLOADS
    w = WORKLOADS
    assert (w["tiny_f32"].T, w["tiny_f32"].hq, w["tiny_f32"].hkv, w["tiny_f32"].d, w["tiny_f32"].k) == (128, 4, 4, 64, 3)
    assert (w["llama8b_2k"].T, w["llama8b_2k"].hq, w["llama8b_2k"].hkv, w["llama8b_2k"].d, w["llama8b_2k"].k) == (2048, 32, 8, 128, 7)
    v = w["varlen_16k"]
    assert v.T == 16384 and all(256 <= L <= 4096 for L in v.doc_lens)
    assert w["qwen235b_8k"].doc_lens == (8192, 8192) and w["qwen235b_8k"].hq == 64 and w["qwen235b_8k"].hkv == 4
    assert w["long_32k"].T == 32768 and w["long_32k"].qk_mult == 2.0
    h = w["headline_4k"]
    assert (h.T, h.hq, h.hkv, h.d, h.k) == (4096, 32, 8, 128, 7)
    # useful work of the headline shape: 14*d*pairs = 3.373 TFLOP
    assert abs(h.useful_flops()["fwd_bwd"] / 1e12 - 3.373) < 1e-3
