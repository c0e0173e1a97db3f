"""ctypes binding of libw4a16.so: argument marshalling only.  Every function has the name of
the C entry point it forwards to (include/w4a16.h); tensors are torch CUDA tensors used purely
as device buffers, and the work is enqueued on torch's current stream.  There is no fallback: if
the library has not been built, loading raises."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("W4A16_LIB") or os.path.join(_HERE, "lib", "libw4a16.so")   # W4A16_LIB: load another build of the same ABI

EXPORTS = (
    "w4a16_version", "w4a16_strerror", "w4a16_set_param", "w4a16_get_param", "w4a16_packed_bytes",
    "w4a16_workspace_bytes", "w4a16_workspace_init", "w4a16_pack", "w4a16_unpack", "w4a16_dequant",
    "w4a16_gemm", "w4a16_gemm_fused", "w4a16_gemm_rope", "w4a16_pack_heads", "w4a16_pack_gate_up", "w4a16_read_probe", "tree_verify_attn_workspace_bytes",
    "tree_verify_attn", "tree_accept", "rms_norm", "rope_append", "lm_head_workspace_bytes", "lm_head_topk",
    "lm_head_packed_bytes", "lm_head_pack", "w4a16_decoder_layer", "w4a16_plan_describe", "w4a16_gemm_static", "w4a16_weight_is_symmetric",
)

EPI_NONE, EPI_RESIDUAL, EPI_SILU_MUL = 0, 1, 2
SYMMETRIC = 0x100   # OR-ed into an epilogue code: every zero-point of the weight is 8

_lib = None


class LayerWeights(ctypes.Structure):
    """w4a16_layer_weights of include/w4a16.h"""
    _fields_ = [("qkv_packed", ctypes.c_void_p), ("o_packed", ctypes.c_void_p), ("gate_up_packed", ctypes.c_void_p),
                ("down_packed", ctypes.c_void_p), ("norm1_gamma", ctypes.c_void_p), ("norm2_gamma", ctypes.c_void_p),
                ("hidden", ctypes.c_int), ("n_q_heads", ctypes.c_int), ("n_kv_heads", ctypes.c_int),
                ("head_dim", ctypes.c_int), ("ffn", ctypes.c_int), ("eps", ctypes.c_float),
                ("qkv_heads_packed", ctypes.c_int), ("symmetric", ctypes.c_int)]


class LayerScratch(ctypes.Structure):
    """w4a16_layer_scratch of include/w4a16.h"""
    _fields_ = [("norm", ctypes.c_void_p), ("qkv", ctypes.c_void_p), ("q", ctypes.c_void_p), ("attn", ctypes.c_void_p),
                ("act", ctypes.c_void_p), ("gemm_workspace", ctypes.c_void_p), ("gemm_workspace_bytes", ctypes.c_size_t),
                ("attn_workspace", ctypes.c_void_p), ("attn_workspace_bytes", ctypes.c_size_t)]


class W4A16Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def load() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_22179_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.w4a16_version.restype = i
    L.w4a16_strerror.restype = ctypes.c_char_p
    L.w4a16_strerror.argtypes = [i]
    L.w4a16_set_param.argtypes = [ctypes.c_char_p, i]
    L.w4a16_get_param.argtypes = [ctypes.c_char_p]
    L.w4a16_packed_bytes.restype = sz
    L.w4a16_packed_bytes.argtypes = [i, i, i]
    L.w4a16_workspace_bytes.restype = sz
    L.w4a16_workspace_bytes.argtypes = [i, i, i, i]
    L.w4a16_workspace_init.argtypes = [vp, sz, vp]
    L.w4a16_pack.argtypes = [vp, vp, vp, vp, i, i, i, vp]
    L.w4a16_unpack.argtypes = [vp, vp, vp, vp, i, i, i, vp]
    L.w4a16_dequant.argtypes = [vp, vp, i, i, i, vp]
    L.w4a16_gemm.argtypes = [vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.w4a16_read_probe.argtypes = [vp, sz, vp, vp]
    L.w4a16_gemm_static.argtypes = [vp, vp, vp, i, i, i, i, vp]
    L.w4a16_weight_is_symmetric.argtypes = [vp, i, i, i, vp, vp]
    L.w4a16_plan_describe.argtypes = [i, i, i, i, ctypes.POINTER(ctypes.c_int)]
    L.tree_verify_attn_workspace_bytes.restype = sz
    L.tree_verify_attn_workspace_bytes.argtypes = [i, i, i, i, i]
    L.tree_verify_attn.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, ctypes.c_float, vp, sz, vp]
    L.tree_accept.argtypes = [vp, vp, vp, i, vp, vp, vp, vp, i, i, i, vp]
    L.w4a16_gemm_fused.argtypes = [vp, vp, vp, i, i, i, i, i, vp, vp, sz, vp]
    L.w4a16_pack_gate_up.argtypes = [vp, vp, vp, vp, i, i, i, vp]
    L.w4a16_pack_heads.argtypes = [vp, vp, vp, vp, i, i, i, i, vp]
    L.w4a16_gemm_rope.argtypes = [vp, vp, i, i, i, vp, vp, vp, i, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.rms_norm.argtypes = [vp, vp, vp, i, i, ctypes.c_float, vp]
    L.rope_append.argtypes = [vp, vp, vp, vp, i, vp, vp, vp, i, i, i, i, i, vp]
    L.w4a16_decoder_layer.argtypes = [ctypes.POINTER(LayerWeights), vp, i, i, vp, vp, vp, i, vp, vp, vp,
                                      ctypes.POINTER(LayerScratch), vp]
    L.lm_head_packed_bytes.restype = sz
    L.lm_head_packed_bytes.argtypes = [i, i]
    L.lm_head_pack.argtypes = [vp, vp, i, i, vp]
    L.lm_head_workspace_bytes.restype = sz
    L.lm_head_workspace_bytes.argtypes = [i, i, i, i]
    L.lm_head_topk.argtypes = [vp, vp, i, i, i, i, vp, vp, vp, vp, sz, vp]
    _lib = L
    return L


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(code: int, where: str) -> None:
    if code != 0:
        raise W4A16Error(code, where)


def w4a16_version() -> int:
    return load().w4a16_version()


def strerror(code: int) -> str:
    return load().w4a16_strerror(code).decode()


def w4a16_set_param(name: str, value: int) -> None:
    _check(load().w4a16_set_param(name.encode(), int(value)), "w4a16_set_param")


def w4a16_get_param(name: str) -> int:
    return load().w4a16_get_param(name.encode())


def w4a16_packed_bytes(N: int, K: int, G: int = 128) -> int:
    return load().w4a16_packed_bytes(N, K, G)


def w4a16_workspace_bytes(M_max: int, N: int, K: int, G: int = 128) -> int:
    return load().w4a16_workspace_bytes(M_max, N, K, G)


def tree_verify_attn_workspace_bytes(M: int, P: int, Hq: int, Hkv: int, D: int) -> int:
    return load().tree_verify_attn_workspace_bytes(M, P, Hq, Hkv, D)


def w4a16_workspace_init(workspace) -> None:
    _check(load().w4a16_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "w4a16_workspace_init")


def new_workspace(nbytes: int, device="cuda"):
    """Allocate and initialise a workspace of at least nbytes."""
    ws = torch.empty(max(int(nbytes), 16384), dtype=torch.uint8, device=device)
    w4a16_workspace_init(ws)
    return ws


def w4a16_pack(qweight, scales, qzeros, packed, N: int, K: int, G: int = 128) -> None:
    _check(load().w4a16_pack(_ptr(qweight), _ptr(scales), _ptr(qzeros), _ptr(packed), N, K, G, _stream()), "w4a16_pack")


def w4a16_unpack(packed, qweight, scales, qzeros, N: int, K: int, G: int = 128) -> None:
    _check(load().w4a16_unpack(_ptr(packed), _ptr(qweight), _ptr(scales), _ptr(qzeros), N, K, G, _stream()), "w4a16_unpack")


def w4a16_dequant(packed, W, N: int, K: int, G: int = 128) -> None:
    _check(load().w4a16_dequant(_ptr(packed), _ptr(W), N, K, G, _stream()), "w4a16_dequant")


def w4a16_gemm(x, packed, y, M: int, N: int, K: int, G: int, workspace) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().w4a16_gemm(_ptr(x), _ptr(packed), _ptr(y), M, N, K, G, _ptr(workspace), nbytes, _stream()), "w4a16_gemm")


def w4a16_gemm_static(x, packed, y, M: int, N: int, K: int, G: int = 128) -> None:
    _check(load().w4a16_gemm_static(_ptr(x), _ptr(packed), _ptr(y), M, N, K, G, _stream()), "w4a16_gemm_static")


def w4a16_gemm_fused(x, packed, y, M: int, N: int, K: int, G: int, epilogue: int, residual, workspace) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().w4a16_gemm_fused(_ptr(x), _ptr(packed), _ptr(y), M, N, K, G, int(epilogue), _ptr(residual),
                                   _ptr(workspace), nbytes, _stream()), "w4a16_gemm_fused")


def w4a16_weight_is_symmetric(packed, N: int, K: int, flag, G: int = 128) -> None:
    _check(load().w4a16_weight_is_symmetric(_ptr(packed), N, K, G, _ptr(flag), _stream()), "w4a16_weight_is_symmetric")


def w4a16_pack_gate_up(qweight, scales, qzeros, packed, N: int, K: int, G: int = 128) -> None:
    _check(load().w4a16_pack_gate_up(_ptr(qweight), _ptr(scales), _ptr(qzeros), _ptr(packed), N, K, G, _stream()),
           "w4a16_pack_gate_up")


def w4a16_pack_heads(qweight, scales, qzeros, packed, N: int, K: int, head_dim: int, G: int = 128) -> None:
    _check(load().w4a16_pack_heads(_ptr(qweight), _ptr(scales), _ptr(qzeros), _ptr(packed), N, K, G, head_dim, _stream()),
           "w4a16_pack_heads")


def w4a16_gemm_rope(x, packed, M: int, K: int, G: int, pos, cos_table, sin_table, n_pos: int, q, k_cache, v_cache,
                    P: int, Hq: int, Hkv: int, D: int, workspace) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().w4a16_gemm_rope(_ptr(x), _ptr(packed), M, K, G, _ptr(pos), _ptr(cos_table), _ptr(sin_table), n_pos,
                                  _ptr(q), _ptr(k_cache), _ptr(v_cache), P, Hq, Hkv, D, _ptr(workspace), nbytes, _stream()),
           "w4a16_gemm_rope")


def rms_norm(x, gamma, y, M: int, K: int, eps: float) -> None:
    _check(load().rms_norm(_ptr(x), _ptr(gamma), _ptr(y), M, K, float(eps), _stream()), "rms_norm")


def rope_append(qkv, pos, cos_table, sin_table, n_pos: int, q, k_cache, v_cache, M: int, P: int, Hq: int, Hkv: int,
                D: int) -> None:
    _check(load().rope_append(_ptr(qkv), _ptr(pos), _ptr(cos_table), _ptr(sin_table), n_pos, _ptr(q), _ptr(k_cache),
                              _ptr(v_cache), M, P, Hq, Hkv, D, _stream()), "rope_append")


def layer_weights(qkv_packed, o_packed, gate_up_packed, down_packed, norm1_gamma, norm2_gamma, hidden: int,
                  n_q_heads: int, n_kv_heads: int, head_dim: int, ffn: int, eps: float,
                  qkv_heads_packed: bool = False, symmetric: bool = False) -> LayerWeights:
    return LayerWeights(_ptr(qkv_packed), _ptr(o_packed), _ptr(gate_up_packed), _ptr(down_packed), _ptr(norm1_gamma),
                        _ptr(norm2_gamma), hidden, n_q_heads, n_kv_heads, head_dim, ffn, float(eps), int(qkv_heads_packed),
                        int(symmetric))


def layer_scratch(norm, qkv, q, attn, act, gemm_workspace, attn_workspace) -> LayerScratch:
    nb = lambda t: 0 if t is None else t.numel() * t.element_size()
    return LayerScratch(_ptr(norm), _ptr(qkv), _ptr(q), _ptr(attn), _ptr(act), _ptr(gemm_workspace), nb(gemm_workspace),
                        _ptr(attn_workspace), nb(attn_workspace))


def w4a16_decoder_layer(weights: LayerWeights, h, M: int, P: int, pos, cos_table, sin_table, n_pos: int, mask, k_cache,
                        v_cache, scratch: LayerScratch) -> None:
    _check(load().w4a16_decoder_layer(ctypes.byref(weights), _ptr(h), M, P, _ptr(pos), _ptr(cos_table), _ptr(sin_table),
                                      n_pos, _ptr(mask), _ptr(k_cache), _ptr(v_cache), ctypes.byref(scratch), _stream()),
           "w4a16_decoder_layer")


def lm_head_workspace_bytes(M: int, V: int, K: int, top_k: int) -> int:
    return int(load().lm_head_workspace_bytes(M, V, K, top_k))


def lm_head_packed_bytes(V: int, K: int) -> int:
    return int(load().lm_head_packed_bytes(V, K))


def lm_head_pack(W, packed, V: int, K: int) -> None:
    _check(load().lm_head_pack(_ptr(W), _ptr(packed), V, K, _stream()), "lm_head_pack")


def lm_head_topk(x, packed, M: int, V: int, K: int, top_k: int, logits, top_idx, top_logprob, workspace) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().lm_head_topk(_ptr(x), _ptr(packed), M, V, K, top_k, _ptr(logits), _ptr(top_idx), _ptr(top_logprob),
                               _ptr(workspace), nbytes, _stream()), "lm_head_topk")


def w4a16_read_probe(buf, nbytes: int, sink) -> None:
    _check(load().w4a16_read_probe(_ptr(buf), int(nbytes), _ptr(sink), _stream()), "w4a16_read_probe")


PLAN_FIELDS = ("family", "row_tiles", "tiles_per_wave", "waves_or_k_sets", "depth_or_groups", "split_k", "fused_reduce",
               "has_symmetric_variant")


def w4a16_plan_describe(M: int, N: int, K: int, G: int = 128) -> tuple:
    """the eight plan fields of include/w4a16.h (see PLAN_FIELDS); host only"""
    out = (ctypes.c_int * 8)()
    _check(load().w4a16_plan_describe(M, N, K, G, out), "w4a16_plan_describe")
    return tuple(out)


def tree_verify_attn(q, k, v, mask, out, M: int, P: int, Hq: int, Hkv: int, D: int, scale: float, workspace) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().tree_verify_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(mask), _ptr(out), M, P, Hq, Hkv, D,
                                   float(scale), _ptr(workspace), nbytes, _stream()), "tree_verify_attn")


def tree_accept(parent, token, target, M: int, path, result, k=None, v=None, P: int = 0, Hkv: int = 0, D: int = 0) -> None:
    _check(load().tree_accept(_ptr(parent), _ptr(token), _ptr(target), M, _ptr(path), _ptr(result), _ptr(k), _ptr(v),
                              P, Hkv, D, _stream()), "tree_accept")


# ---- conveniences for tests and the benchmark (still marshalling only) ----

def pack_from_numpy(inp, device="cuda", gate_up: bool = False, head_dim: int = 0):
    """Upload a LinearInputs' canonical tensors and return the packed device buffer (plain, gate/up paired,
    or -- head_dim > 0 -- with the halves of every head paired)."""
    qw = torch.from_numpy(inp.qweight).to(device)
    sc = torch.from_numpy(inp.scales).to(device)
    qz = torch.from_numpy(inp.qzeros).to(device)
    packed = torch.empty(w4a16_packed_bytes(inp.N, inp.K, inp.G), dtype=torch.uint8, device=device)
    if head_dim:
        w4a16_pack_heads(qw, sc, qz, packed, inp.N, inp.K, head_dim, inp.G)
    else:
        (w4a16_pack_gate_up if gate_up else w4a16_pack)(qw, sc, qz, packed, inp.N, inp.K, inp.G)
    return packed
