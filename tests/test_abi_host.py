"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, and rejects bad arguments before touching the GPU runtime."""
import ctypes
import os
import re

import pytest

from paper_2505_22179_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "w4a16.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:w4a16|tree|rms|rope|lm_head)_\w+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = B.load()
    names = _declared()
    assert "w4a16_gemm" in names and "tree_verify_attn" in names and "w4a16_pack" in names and "tree_accept" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_version_and_strerror():
    assert B.w4a16_version() >= 100
    assert B.strerror(0) == "ok"
    for code in range(-6, 0):
        assert B.strerror(code) not in ("ok", "unknown error code")
    assert B.strerror(-99) == "unknown error code"


def test_sizes():
    rec = 8192 + 256 + 64
    assert B.w4a16_packed_bytes(4096, 4096) == 32 * 32 * rec
    assert B.w4a16_packed_bytes(8, 128) == rec                 # padded to one 128-column block
    assert B.w4a16_packed_bytes(136, 256) == 2 * 2 * rec
    assert B.w4a16_packed_bytes(4096, 4096, 64) == 0            # group size other than 128
    assert B.w4a16_packed_bytes(4096, 4100) == 0
    assert B.w4a16_packed_bytes(4100, 4096) == 0
    # minimal bytes per weight: 0.5 code + 2/128 scale + 0.5/128 zero
    assert B.w4a16_packed_bytes(8192, 8192) / (8192 * 8192) == pytest.approx(0.51953125)
    for shape in ((4096, 4096), (57344, 8192), (8192, 28672)):
        assert B.w4a16_workspace_bytes(64, *shape) >= 16384
    assert B.w4a16_workspace_bytes(65, 4096, 4096) == 0
    assert B.tree_verify_attn_workspace_bytes(60, 2048, 64, 8, 128) > 16384
    assert B.tree_verify_attn_workspace_bytes(60, 2048, 64, 8, 64) == 0


def test_params():
    B.w4a16_set_param("split_k", 3)
    assert B.w4a16_get_param("split_k") == 3
    B.w4a16_set_param("split_k", 0)
    with pytest.raises(B.W4A16Error):
        B.w4a16_set_param("no_such_knob", 1)
    with pytest.raises(B.W4A16Error):
        B.w4a16_set_param("split_k", -1)


def test_argument_validation_happens_before_any_gpu_call():
    lib = B.load()
    a = 0x1000  # fake, aligned, never dereferenced: every call below must fail validation first
    EINVAL, ENULL, EALIGN, EUNSUP, EWS = -1, -2, -3, -4, -5
    g = lib.w4a16_gemm
    assert g(a, a, a, 0, 4096, 4096, 128, a, 1 << 30, None) == EINVAL      # M = 0
    assert g(a, a, a, 65, 4096, 4096, 128, a, 1 << 30, None) == EUNSUP     # M > 64
    assert g(a, a, a, 1, 4096, 4000, 128, a, 1 << 30, None) == EINVAL      # K % G
    assert g(a, a, a, 1, 4100, 4096, 128, a, 1 << 30, None) == EINVAL      # N % 8
    assert g(a, a, a, 1, 4096, 4096, 64, a, 1 << 30, None) == EUNSUP       # G != 128
    assert g(None, a, a, 1, 4096, 4096, 128, a, 1 << 30, None) == ENULL
    assert g(a, None, a, 1, 4096, 4096, 128, a, 1 << 30, None) == ENULL
    assert g(a, a, None, 1, 4096, 4096, 128, a, 1 << 30, None) == ENULL
    assert g(a + 2, a, a, 1, 4096, 4096, 128, a, 1 << 30, None) == EALIGN
    assert g(a, a, a, 1, 8192, 28672, 128, None, 0, None) == EWS           # a shape that splits K, no workspace
    assert g(a, a, a, 1, 8192, 28672, 128, a, 100, None) == EWS
    p = lib.w4a16_pack
    assert p(None, a, a, a, 4096, 4096, 128, None) == ENULL
    assert p(a, a, a, a + 4, 4096, 4096, 128, None) == EALIGN
    assert p(a, a, a, a, 4096, 4096, 32, None) == EUNSUP
    assert lib.w4a16_unpack(a, a, a, None, 4096, 4096, 128, None) == ENULL
    assert lib.w4a16_dequant(a, None, 4096, 4096, 128, None) == ENULL
    assert lib.w4a16_dequant(a, a, -1, 4096, 128, None) == EINVAL
    assert lib.w4a16_workspace_init(None, 1 << 20, None) == ENULL
    assert lib.w4a16_workspace_init(a, 16, None) == EWS
    t = lib.tree_verify_attn
    f = ctypes.c_float(0.1)
    assert t(a, a, a, a, a, 60, 2048, 64, 8, 64, f, a, 1 << 30, None) == EUNSUP    # D != 128
    assert t(a, a, a, a, a, 65, 2048, 64, 8, 128, f, a, 1 << 30, None) == EUNSUP   # M > 64
    assert t(a, a, a, a, a, 60, 2048, 64, 7, 128, f, a, 1 << 30, None) == EINVAL   # Hq % Hkv
    assert t(a, a, a, a, a, 0, 2048, 64, 8, 128, f, a, 1 << 30, None) == EINVAL
    assert t(a, a, a, a, a, 1, 2048, 64, 4, 128, f, a, 1 << 30, None) == EUNSUP    # more than 8 query heads per KV head
    assert t(a, a, a, None, a, 60, 2048, 64, 8, 128, f, a, 1 << 30, None) == ENULL
    for bad_scale in (0.0, -0.1, float("nan"), float("inf")):   # row maxima are taken before scaling: the scale is positive
        assert t(a, a, a, a, a, 60, 2048, 64, 8, 128, ctypes.c_float(bad_scale), a, 1 << 30, None) == EINVAL
    assert t(a, a, a, a, a, 60, 2048, 64, 8, 128, f, None, 0, None) == EWS


def test_plan_describe():
    out = (ctypes.c_int * 8)()
    lib = B.load()
    assert lib.w4a16_plan_describe(1, 4096, 4096, 128, None) == -2
    assert lib.w4a16_plan_describe(0, 4096, 4096, 128, out) == -1
    assert lib.w4a16_plan_describe(65, 4096, 4096, 128, out) == -4
    assert lib.w4a16_plan_describe(1, 4096, 4096, 64, out) == -4
    for M in (1, 8, 16, 17, 64):
        for N, K in ((4096, 4096), (57344, 8192), (8192, 28672), (1000, 1536)):
            plan = B.w4a16_plan_describe(M, N, K)
            assert plan[0] in (0, 1, 2, 3) and plan[1] == (M + 15) // 16 and plan[2] in (2, 4, 8), plan
    B.w4a16_set_param("tiles_per_wave", 8)
    B.w4a16_set_param("waves_per_wg", 16)
    try:
        assert lib.w4a16_plan_describe(40, 128, 256, 128, out) == -4   # a variant that is not compiled
    finally:
        B.w4a16_set_param("tiles_per_wave", 0)
        B.w4a16_set_param("waves_per_wg", 0)


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_22179_amd")
    bad = re.compile(r"^\s*(from|import)\s+oracle\b|liboracle|w4a16_oracle|#include\s+\"[^\"]*oracle", re.M)
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                assert not bad.search(open(os.path.join(dirpath, fn)).read()), (dirpath, fn)


def test_tree_accept_rejects_bad_arguments_before_the_gpu():
    L = B.load()
    fake, fake2 = 0x1000, 0x2000
    args = lambda **kw: [kw.get("parent", fake), fake, fake, kw.get("M", 60), fake, kw.get("result", fake),
                         kw.get("k", fake2), kw.get("v", fake2), kw.get("P", 2048), kw.get("Hkv", 8), kw.get("D", 128), None]
    assert L.tree_accept(*args(M=0)) == -1
    assert L.tree_accept(*args(M=65)) == -4
    assert L.tree_accept(*args(P=-1)) == -1
    assert L.tree_accept(*args(parent=None)) == -2
    assert L.tree_accept(*args(v=None)) == -2          # k without v
    assert L.tree_accept(*args(result=0x1002)) == -3   # 4-byte alignment of the integer buffers
    assert L.tree_accept(*args(k=0x2008)) == -3        # 16-byte alignment of the cache
    assert L.tree_accept(*args(Hkv=1, D=4)) == -4      # rows that are not a multiple of 16 bytes


def test_layer_glue_validation_happens_before_any_gpu_call():
    lib = B.load()
    a = 0x1000
    EINVAL, ENULL, EALIGN, EUNSUP = -1, -2, -3, -4
    f = lib.w4a16_gemm_fused
    assert f(a, a, a, 1, 4096, 4096, 128, 3, None, a, 1 << 30, None) == EINVAL       # unknown epilogue
    assert f(a, a, a, 1, 4096, 4096, 128, 1, None, a, 1 << 30, None) == ENULL        # residual missing
    assert f(a, a, a, 1, 4096, 4096, 128, 1, a + 8, a, 1 << 30, None) == EALIGN
    assert f(a, a, a, 1, 4096, 4096, 128, 0, a, a, 1 << 30, None) == EINVAL          # residual without the epilogue
    assert f(a, a, a, 1, 4112, 4096, 128, 2, None, a, 1 << 30, None) == EINVAL       # gate/up halves need N % 32 == 0
    assert f(a, a, a, 65, 4096, 4096, 128, 2, None, a, 1 << 30, None) == EUNSUP
    assert lib.w4a16_pack_gate_up(a, a, a, a, 4112, 4096, 128, None) == EINVAL
    assert lib.w4a16_pack_gate_up(a, a, None, a, 4096, 4096, 128, None) == ENULL
    n = lib.rms_norm
    assert n(a, a, a, 0, 4096, 1e-5, None) == EINVAL
    assert n(a, a, a, 1, 4100, 1e-5, None) == EINVAL
    assert n(a, a, a, 1, 4096, -1.0, None) == EINVAL
    assert n(a, a, a, 1, 32768, 1e-5, None) == EUNSUP
    assert n(a, None, a, 1, 4096, 1e-5, None) == ENULL
    assert n(a, a, a + 4, 1, 4096, 1e-5, None) == EALIGN
    r = lib.rope_append
    assert r(a, a, a, a, 64, a, a, a, 0, 10, 8, 2, 128, None) == EINVAL              # M = 0
    assert r(a, a, a, a, 64, a, a, a, 4, -1, 8, 2, 128, None) == EINVAL              # P < 0
    assert r(a, a, a, a, 64, a, a, a, 4, 10, 8, 2, 127, None) == EINVAL              # odd head size
    assert r(a, a, a, a, 0, a, a, a, 4, 10, 8, 2, 128, None) == EINVAL               # empty tables
    assert r(a, None, a, a, 64, a, a, a, 4, 10, 8, 2, 128, None) == ENULL
    assert r(a, a + 2, a, a, 64, a, a, a, 4, 10, 8, 2, 128, None) == EALIGN
    assert r(a, a, a, a, 64, a + 8, a, a, 4, 10, 8, 2, 128, None) == EALIGN


def test_workspaces_must_be_256_byte_aligned():
    lib = B.load()
    a = 0x1000
    assert lib.w4a16_workspace_init(a + 128, 1 << 20, None) == -3
    assert lib.w4a16_gemm(a, a, a, 1, 4096, 4096, 128, a + 16, 1 << 30, None) == -3
    assert lib.tree_verify_attn(a, a, a, a, a, 4, 100, 8, 2, 128, 0.1, a + 64, 1 << 30, None) == -3


def test_gemm_rope_validation_happens_before_any_gpu_call():
    lib = B.load()
    a = 0x1000
    EINVAL, ENULL, EALIGN, EUNSUP = -1, -2, -3, -4
    ph = lib.w4a16_pack_heads
    assert ph(a, a, a, a, 10240, 8192, 128, 16, None) == EINVAL      # heads of fewer than 32 columns
    assert ph(a, a, a, a, 10240, 8192, 128, 48, None) == EINVAL      # not a multiple of 32
    assert ph(a, a, a, a, 10240, 8192, 128, 96, None) == EINVAL      # N is not a whole number of heads
    assert ph(a, a, None, a, 10240, 8192, 128, 128, None) == ENULL
    assert ph(a, a, a, a + 8, 10240, 8192, 128, 128, None) == EALIGN
    g = lib.w4a16_gemm_rope
    ok = dict(x=a, packed=a, M=4, K=8192, G=128, pos=a, cos=a, sin=a, n_pos=64, q=a, k=a, v=a, P=10, Hq=64, Hkv=8, D=128)

    def call(**kw):
        v = {**ok, **kw}
        return g(v["x"], v["packed"], v["M"], v["K"], v["G"], v["pos"], v["cos"], v["sin"], v["n_pos"], v["q"], v["k"], v["v"],
                 v["P"], v["Hq"], v["Hkv"], v["D"], a, 1 << 30, None)

    assert call(P=-1) == EINVAL and call(Hkv=0) == EINVAL and call(n_pos=0) == EINVAL
    assert call(D=16) == EINVAL and call(D=80) == EINVAL           # head size: a multiple of 32
    assert call(pos=None) == ENULL and call(q=None) == ENULL and call(v=None) == ENULL
    assert call(cos=a + 4) == EALIGN and call(k=a + 8) == EALIGN and call(pos=a + 2) == EALIGN
    assert call(M=0) == EINVAL and call(M=65) == EUNSUP and call(x=None) == ENULL   # the linear's own checks
    assert call(K=8200) == EINVAL


def test_lm_head_validation_happens_before_any_gpu_call():
    lib = B.load()
    a = 0x1000
    EINVAL, ENULL, EALIGN, EUNSUP, EWS = -1, -2, -3, -4, -5
    f = lib.lm_head_topk
    assert f(a, a, 0, 1000, 4096, 10, a, a, a, a, 1 << 30, None) == EINVAL        # M = 0
    assert f(a, a, 65, 1000, 4096, 10, a, a, a, a, 1 << 30, None) == EUNSUP       # more than four row tiles
    assert f(a, a, 4, 1000, 4000, 10, a, a, a, a, 1 << 30, None) == EINVAL        # K % 128
    assert f(a, a, 4, 8, 4096, 10, a, a, a, a, 1 << 30, None) == EINVAL           # top_k > V
    assert f(a, a, 4, 1000, 4096, 65, a, a, a, a, 1 << 30, None) == EUNSUP
    assert f(a, a, 4, 128256, 4096, 64, a, a, a, a, 1 << 30, None) == EUNSUP      # too many candidates to merge
    assert f(a, a, 4, 300000, 4096, 4, a, a, a, a, 1 << 30, None) == EUNSUP        # too many chunks
    assert f(a, None, 4, 1000, 4096, 10, a, a, a, a, 1 << 30, None) == ENULL
    assert f(a, a, 4, 1000, 4096, 10, a, a + 2, a, a, 1 << 30, None) == EALIGN
    assert f(a, a, 4, 1000, 4096, 10, a, a, a, None, 0, None) == EWS
    assert f(a, a, 4, 1000, 4096, 10, a, a, a, a, 16, None) == EWS
    assert B.lm_head_packed_bytes(128256, 4096) == 128256 * 4096 * 2
    assert B.lm_head_packed_bytes(1001, 128) == 1008 * 128 * 2           # padded to whole 16-token tiles
    assert B.lm_head_packed_bytes(1000, 100) == 0
    assert lib.lm_head_pack(a, a, 1000, 100, None) == EINVAL
    assert lib.lm_head_pack(None, a, 1000, 128, None) == ENULL
    assert lib.lm_head_pack(a, a + 4, 1000, 128, None) == EALIGN
    assert B.lm_head_workspace_bytes(10, 128256, 4096, 10) > 0
    assert B.lm_head_workspace_bytes(65, 128256, 4096, 10) == 0


def test_decoder_layer_validation_happens_before_any_gpu_call():
    import ctypes
    lib = B.load()
    a = 0x1000
    EINVAL, ENULL = -1, -2
    w = B.LayerWeights(a, a, a, a, a, a, 1024, 8, 2, 128, 2816, 1e-5)
    s = B.LayerScratch(a, a, a, a, a, a, 1 << 20, a, 1 << 20)
    f = lib.w4a16_decoder_layer
    args = lambda ww, ss, h=a, M=4, P=10: (ww, h, M, P, a, a, a, 64, a, a, a, ss, None)
    assert f(*args(None, ctypes.byref(s))) == ENULL
    assert f(*args(ctypes.byref(w), None)) == ENULL
    assert f(*args(ctypes.byref(w), ctypes.byref(s), h=None)) == ENULL
    assert f(*args(ctypes.byref(w), ctypes.byref(s), M=0)) == EINVAL
    assert f(*args(ctypes.byref(w), ctypes.byref(s), P=-1)) == EINVAL
    bad = B.LayerWeights(a, a, None, a, a, a, 1024, 8, 2, 128, 2816, 1e-5)
    assert f(*args(ctypes.byref(bad), ctypes.byref(s))) == ENULL
    bad = B.LayerWeights(a, a, a, a, a, a, 1024, 0, 2, 128, 2816, 1e-5)
    assert f(*args(ctypes.byref(bad), ctypes.byref(s))) == EINVAL
    nos = B.LayerScratch(a, None, a, a, a, a, 1 << 20, a, 1 << 20)
    assert f(*args(ctypes.byref(w), ctypes.byref(nos))) == ENULL
    # the first step's own validation: hidden size the norm cannot take, before anything is enqueued
    bad = B.LayerWeights(a, a, a, a, a, a, 1000 * 1024, 8, 2, 128, 2816, 1e-5)
    assert f(*args(ctypes.byref(bad), ctypes.byref(s))) == -4
