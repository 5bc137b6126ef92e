"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2502_00340_amd import binding as Bn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = C.c_void_p(0x10000)      # never dereferenced: all calls below fail validation first


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(Bn.LIB_PATH):
        from paper_2502_00340_amd import build
        build.build_library(verbose=False)
    return Bn.lib()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "centrifuge.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cf_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = _declared_symbols()
    assert set(names) == set(Bn.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None, n


def test_status_strings(L):
    assert L.cf_status_str(0) == b"ok"
    for code in range(1, 7):
        assert len(L.cf_status_str(code)) > 0
    assert b"gfx950" in L.cf_version()


def _desc(**kw):
    base = dict(B=2, S=128, H=256, Hq=4, Hkv=4, d=64, F=688, dtype="f32")
    base.update(kw)
    return Bn.make_desc(**base)


def test_workspace_sizes(L):
    d = _desc()
    full = L.cf_layer_workspace_bytes(C.byref(d), 256)
    half = L.cf_layer_workspace_bytes(C.byref(d), 128)
    assert full > half > 0 and full % 256 == 0
    assert L.cf_layer_workspace_bytes(C.byref(_desc(Hq=3)), 256) == 0     # Hq % Hkv != 0
    assert L.cf_layer_workspace_bytes(C.byref(_desc(dtype="bf16", F=687)), 256) == 0
    assert L.cf_index_workspace_bytes(1 << 24) >= 4 * (1 << 24) // 8192      # one count per span of 8192 tokens
    assert L.cf_attn_workspace_bytes(C.byref(d), 100) >= 100 * 4 * 4


def test_keep_index_argument_errors(L):
    n = C.c_int32(0)
    f = L.cf_build_keep_index
    assert f(None, 2, 8, FAKE, FAKE, None, C.byref(n), FAKE, 256, None) == 1
    assert f(FAKE, 0, 8, FAKE, FAKE, None, C.byref(n), FAKE, 256, None) == 2
    assert f(FAKE, 2, 8, FAKE, FAKE, None, C.byref(n), None, 0, None) == 4
    assert f(FAKE, 2, 8, FAKE, FAKE, None, C.byref(n), C.c_void_p(0x10010), 256, None) == 4   # misaligned ws
    assert f(FAKE, 1 << 20, 1 << 20, FAKE, FAKE, None, C.byref(n), FAKE, 1 << 30, None) == 2


def test_static_keep_index_argument_errors(L):
    f = L.cf_build_keep_index_static
    assert f(None, 2, 8, FAKE, FAKE, None, None) == 1
    assert f(FAKE, 2, 8, None, FAKE, None, None) == 1
    assert f(FAKE, 0, 8, FAKE, FAKE, None, None) == 2
    assert f(FAKE, 2, 8, C.c_void_p(0x10002), FAKE, None, None) == 2
    assert f(FAKE, 1, (1 << 24) + 1, FAKE, FAKE, None, None) == 5      # beyond the built-in scratch
    assert f(FAKE, 4097, 4096, FAKE, FAKE, None, None) == 5


def test_gather_argument_errors(L):
    f = L.cf_gather_rows
    assert f(None, 4, 8, 1, FAKE, None, 2, FAKE, None) == 1
    assert f(FAKE, 4, 8, 7, FAKE, None, 2, FAKE, None) == 3
    assert f(FAKE, 4, 0, 1, FAKE, None, 2, FAKE, None) == 2
    assert f(FAKE, 4, 3, 0, FAKE, None, 2, FAKE, None) == 2        # 3 bf16 = 6 bytes per row
    assert f(FAKE, 4, 8, 1, FAKE, None, -1, FAKE, None) == 2
    assert f(FAKE, 4, 8, 1, FAKE, C.c_void_p(0x10002), 2, FAKE, None) == 2   # misaligned device count


def test_linear_argument_errors(L):
    f = L.cf_linear_bwd_reduced
    assert f(FAKE, None, FAKE, 4, 8, 8, 1, FAKE, FAKE, 0.0, None) == 1
    assert f(FAKE, FAKE, None, 4, 8, 8, 1, FAKE, None, 0.0, None) == 1   # dx wanted, no W
    assert f(None, FAKE, FAKE, 4, 8, 8, 1, None, FAKE, 0.0, None) == 1   # dw wanted, no X
    assert f(FAKE, FAKE, FAKE, 4, 8, 8, 9, FAKE, FAKE, 0.0, None) == 3
    assert f(FAKE, FAKE, FAKE, 4, 6, 8, 1, FAKE, FAKE, 0.0, None) == 2   # in % 4
    assert f(FAKE, FAKE, FAKE, 4, 12, 8, 0, FAKE, FAKE, 0.0, None) == 2  # bf16 needs % 8
    assert f(FAKE, FAKE, FAKE, 4, 8, 8, 1, FAKE, FAKE, 0.5, None) == 2   # beta must be 0 or 1
    assert f(FAKE, FAKE, FAKE, -1, 8, 8, 1, FAKE, FAKE, 0.0, None) == 2
    assert f(C.c_void_p(0x10004), FAKE, FAKE, 4, 8, 8, 1, FAKE, FAKE, 0.0, None) == 2  # misaligned
    assert f(FAKE, FAKE, FAKE, 1 << 20, 14336, 4096, 0, FAKE, FAKE, 0.0, None) == 5    # bf16 matrix of 2 GiB or more


def test_attention_argument_errors(L):
    f = L.cf_attn_bwd_filtered
    d = _desc()
    args = [FAKE] * 8
    assert f(None, *args, 4, FAKE, FAKE, FAKE, FAKE, 4096, None) == 1
    assert f(C.byref(d), None, *args[1:], 4, FAKE, FAKE, FAKE, FAKE, 4096, None) == 1
    assert f(C.byref(_desc(Hq=6, Hkv=4)), *args, 4, FAKE, FAKE, FAKE, FAKE, 4096, None) == 2
    assert f(C.byref(_desc(dtype="bf16", d=96)), *args, 4, FAKE, FAKE, FAKE, FAKE, 4096, None) == 5   # no kernel for this head size
    assert f(C.byref(_desc(dtype="bf16", d=100)), *args, 4, FAKE, FAKE, FAKE, FAKE, 4096, None) == 2
    # 32-bit byte offsets inside one sequence's q rows: refused, not wrapped
    assert f(C.byref(_desc(dtype="bf16", B=1, S=1 << 20, Hq=32, Hkv=8, d=128)), *args, 4, FAKE, FAKE, FAKE, FAKE,
             4096, None) == 5
    assert f(C.byref(_desc(d=48)), *args, 4, FAKE, FAKE, FAKE, FAKE, 4096, None) == 2
    assert f(C.byref(d), *args, 257, FAKE, FAKE, FAKE, FAKE, 1 << 20, None) == 2   # n_kept > T
    assert f(C.byref(d), *args, 4, FAKE, FAKE, FAKE, None, 0, None) == 4
    assert f(C.byref(d), *args, 200, FAKE, FAKE, FAKE, FAKE, 256, None) == 4       # ws too small


def test_layer_argument_errors(L):
    d = _desc()
    sv = Bn.Saved(*([0x10000] * 9 + [None, None]))
    w = Bn.Weights(*([0x10000] * 9))
    g = Bn.Grads(*([0x10000] * 10))
    n = C.c_int32(0)
    f = L.cf_layer_bwd_filtered
    ok_ws = L.cf_layer_workspace_bytes(C.byref(d), 256)
    tail = (None, None, None, C.byref(n), FAKE, ok_ws, None)     # idx_out, cu_out, n_dev_out, n_host, ws, bytes, stream
    assert f(None, C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g), *tail) == 1
    assert f(C.byref(d), C.byref(sv), C.byref(w), FAKE, None, 0, C.byref(g), *tail) == 1                # no mask
    assert f(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, -1, C.byref(g), *tail) == 2               # max_kept < 0
    sv_bad = Bn.Saved(*([0x10000] * 8 + [0, None, None]))
    assert f(C.byref(d), C.byref(sv_bad), C.byref(w), FAKE, FAKE, 0, C.byref(g), *tail) == 1
    assert f(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g), None, None, None, C.byref(n), FAKE, 16, None) == 4
    # a workspace sized for 128 kept tokens does not do for max_kept = T, but does for max_kept = 128
    half_ws = L.cf_layer_workspace_bytes(C.byref(d), 128)
    assert f(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g), None, None, None, C.byref(n), FAKE, half_ws, None) == 4
    assert f(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g), C.c_void_p(0x10002), None, None, C.byref(n),
             FAKE, ok_ws, None) == 2                                                                    # misaligned idx_out
    assert f(C.byref(_desc(H=250)), C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g), *tail) == 2
    sv_rope = Bn.Saved(*([0x10000] * 9 + [0x10000, None]))      # one rotary table without the other
    assert f(C.byref(d), C.byref(sv_rope), C.byref(w), FAKE, FAKE, 0, C.byref(g), *tail) == 1
    # a [T,F] matrix of 2 GiB or more is beyond the bf16 GEMM's 32-bit offsets: refused up front
    big = _desc(dtype="bf16", B=64, S=8192, H=4096, Hq=32, Hkv=8, d=128, F=14336)
    assert f(C.byref(big), C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g), *tail) == 5
    assert L.cf_layer_workspace_bytes(C.byref(big), 1024) == 0
    g_bad = Bn.Grads(*([0x10000] * 10 + [2]))                   # main_grad is 0 or 1
    assert f(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, 0, C.byref(g_bad), *tail) == 2
    fc = L.cf_layer_bwd_compact
    assert fc(C.byref(d), C.byref(sv), C.byref(w), FAKE, None, FAKE, 4, C.byref(g), FAKE, ok_ws, None) == 1
    assert fc(C.byref(d), C.byref(sv), C.byref(w), None, FAKE, FAKE, 4, C.byref(g), FAKE, ok_ws, None) == 1
    assert fc(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, FAKE, 257, C.byref(g), FAKE, ok_ws, None) == 2   # n_kept > T
    assert fc(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, FAKE, -1, C.byref(g), FAKE, ok_ws, None) == 2
    assert fc(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, FAKE, 200, C.byref(g), FAKE, 4096, None) == 4
    fv = L.cf_layer_bwd_compact_dev
    assert fv(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, FAKE, None, 0, C.byref(g), FAKE, ok_ws, None) == 1   # no device count
    assert fv(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, FAKE, FAKE, -3, C.byref(g), FAKE, ok_ws, None) == 2
    assert fv(C.byref(d), C.byref(sv), C.byref(w), FAKE, FAKE, FAKE, FAKE, 0, C.byref(g), FAKE, half_ws, None) == 4
    fd = L.cf_layer_bwd_dense
    assert fd(C.byref(d), C.byref(sv), C.byref(w), None, C.byref(g), FAKE, ok_ws, None) == 1
    assert fd(C.byref(d), C.byref(sv), C.byref(w), FAKE, C.byref(g), FAKE, ok_ws - 256, None) == 4
    assert fd(C.byref(_desc(dtype="bf16", d=32)), C.byref(sv), C.byref(w), FAKE, C.byref(g), FAKE, ok_ws, None) == 5


def test_lora_argument_errors(L):
    d = _desc()
    sv = Bn.Saved(*([0x10000] * 9 + [None, None]))
    w = Bn.Weights(*([0x10000] * 9))
    g = Bn.LoraGrads(*([0x10000] * 9))
    n = C.c_int32(0)
    f = L.cf_layer_bwd_lora
    ok_ws = L.cf_lora_workspace_bytes(C.byref(d), 8, 256)
    assert ok_ws > L.cf_layer_workspace_bytes(C.byref(d), 256)
    assert L.cf_lora_workspace_bytes(C.byref(d), 0, 256) == 0
    lo = Bn.Lora(*([0x10000] * 8 + [8, 2.0]))
    assert f(C.byref(d), C.byref(sv), C.byref(w), None, FAKE, FAKE, 0, C.byref(g), None, None, None, C.byref(n), FAKE, ok_ws, None) == 1
    lo_bad = Bn.Lora(*([0x10000] * 7 + [0, 8, 2.0]))
    assert f(C.byref(d), C.byref(sv), C.byref(w), C.byref(lo_bad), FAKE, FAKE, 0, C.byref(g), None, None, None, C.byref(n), FAKE, ok_ws, None) == 1
    lo_rank = Bn.Lora(*([0x10000] * 8 + [6, 2.0]))
    assert f(C.byref(d), C.byref(sv), C.byref(w), C.byref(lo_rank), FAKE, FAKE, 0, C.byref(g), None, None, None, C.byref(n), FAKE, ok_ws, None) == 2
    # a negative bound, a misaligned device count pointer, a workspace that is too small (sized for T when max_kept is 0)
    assert f(C.byref(d), C.byref(sv), C.byref(w), C.byref(lo), FAKE, FAKE, -1, C.byref(g), None, None, None, C.byref(n), FAKE, ok_ws, None) == 2
    assert f(C.byref(d), C.byref(sv), C.byref(w), C.byref(lo), FAKE, FAKE, 0, C.byref(g), None, None, C.c_void_p(0x10002), C.byref(n), FAKE, ok_ws, None) == 2
    assert f(C.byref(d), C.byref(sv), C.byref(w), C.byref(lo), FAKE, FAKE, 256, C.byref(g), None, None, None, C.byref(n), FAKE, 256, None) == 4
    assert f(C.byref(d), C.byref(sv), C.byref(w), C.byref(lo), FAKE, None, 0, C.byref(g), None, None, None, None, FAKE, 256, None) == 4


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_00340_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.replace("the CPU oracle's tests", ""), fn
