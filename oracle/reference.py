"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke
check and by the benchmark's cpu_baseline leg, never by the product package.

Linear layer (paper section 2.2, W4A16 with group size 128): thin ctypes wrappers around the C
file next to this one, which carries the definition (unpack, exact fp32 dequantisation, fp32
k-ascending sum with an fp64 shadow, round-to-nearest-even fp16).

Tree-verify attention (paper section 2.1: the target model scores all n draft-tree tokens in one
forward pass; a draft token may attend to the committed prefix, to itself and to its ancestors in
the tree): plain numpy in fp64, written below.

Greedy tree acceptance and K/V compaction (the integer step right after verification): plain
Python below; pinned in tests/test_oracle_accept.py by brute force over all root paths, chain
closed forms, planted paths and library gathers.

Layer glue (RMS norm, residual and SiLU-gate epilogues of the linears, rotary embedding with K/V
append): plain numpy in fp64 at the end of this file; pinned in tests/test_oracle_layer.py by
closed forms, one-hot inputs that reduce the linear to a table lookup, rotation invariants and the
torch library routines.

Draft-side LM head with log-softmax and top-k: numpy fp64 at the end of this file; pinned in
tests/test_oracle_lm_head.py (one-hot rows, planted winners, probabilities that sum to one, ties,
torch's log_softmax / topk).

Pin status.  The paper prints no worked numerical example for any of these operations, so beyond the
pins in tests/test_oracle_*.py (nibble-order fixtures, round trips, closed forms, exact rational
brute force, numpy/torch library cross-checks, structural invariants) the numerics are unpinned
by the paper and this oracle is the definition.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        path = _build.build()
        L = ctypes.CDLL(path)
        vp, i = ctypes.c_void_p, ctypes.c_int
        L.orc_f16_to_f32.restype = ctypes.c_float
        L.orc_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.orc_f32_to_f16.restype = ctypes.c_uint16
        L.orc_f32_to_f16.argtypes = [ctypes.c_float]
        L.orc_f16_to_f32_array.argtypes = [vp, vp, ctypes.c_size_t]
        L.orc_f32_to_f16_array.argtypes = [vp, vp, ctypes.c_size_t]
        L.orc_unpack_codes.argtypes = [vp, vp, i, i]
        L.orc_unpack_zeros.argtypes = [vp, vp, i, i]
        L.orc_dequant.argtypes = [vp, vp, vp, vp, i, i, i]
        L.orc_matmul.argtypes = [vp, vp, vp, vp, vp, i, i, i]
        L.orc_gemm.argtypes = [vp] * 8 + [i] * 4
        L.orc_set_threads.restype = i
        L.orc_set_threads.argtypes = [i]
        for name in ("orc_f16_to_f32_array", "orc_f32_to_f16_array", "orc_unpack_codes",
                     "orc_unpack_zeros", "orc_dequant", "orc_matmul", "orc_gemm"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _p(a: np.ndarray) -> ctypes.c_void_p:
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def set_threads(n: int) -> int:
    """n > 0 sets the OpenMP thread count; returns the count in effect."""
    return int(lib().orc_set_threads(int(n)))


def f16_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h).view(np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().orc_f16_to_f32_array(_p(h), _p(out), h.size)
    return out


def f32_to_f16(f: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(f, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.uint16)
    lib().orc_f32_to_f16_array(_p(f), _p(out), f.size)
    return out.view(np.float16)


def unpack_codes(qweight: np.ndarray) -> np.ndarray:
    """int32 [K/8, N] -> uint8 [K, N]"""
    qweight = np.ascontiguousarray(qweight, dtype=np.int32)
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    q = np.empty((K, N), dtype=np.uint8)
    lib().orc_unpack_codes(_p(qweight), _p(q), K, N)
    return q


def unpack_zeros(qzeros: np.ndarray) -> np.ndarray:
    """int32 [K/G, N/8] -> uint8 [K/G, N]"""
    qzeros = np.ascontiguousarray(qzeros, dtype=np.int32)
    R, N = qzeros.shape[0], qzeros.shape[1] * 8
    z = np.empty((R, N), dtype=np.uint8)
    lib().orc_unpack_zeros(_p(qzeros), _p(z), R, N)
    return z


def dequant(qweight: np.ndarray, scales: np.ndarray, qzeros: np.ndarray, G: int = 128) -> np.ndarray:
    """-> fp32 [K, N], w = (q - z) * s, exact"""
    qweight = np.ascontiguousarray(qweight, dtype=np.int32)
    qzeros = np.ascontiguousarray(qzeros, dtype=np.int32)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    assert scales.shape == (K // G, N) and qzeros.shape == (K // G, N // 8)
    W = np.empty((K, N), dtype=np.float32)
    lib().orc_dequant(_p(qweight), _p(scales.view(np.uint16)), _p(qzeros), _p(W), N, K, G)
    return W


def matmul(x: np.ndarray, W: np.ndarray, want64: bool = True):
    """x fp16 [M, K], W fp32 [K, N] -> (y32, y64 or None, y16)"""
    x = np.ascontiguousarray(x, dtype=np.float16)
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = x.shape
    N = W.shape[1]
    assert W.shape[0] == K
    y32 = np.empty((M, N), dtype=np.float32)
    y64 = np.empty((M, N), dtype=np.float64) if want64 else None
    y16 = np.empty((M, N), dtype=np.uint16)
    lib().orc_matmul(_p(x.view(np.uint16)), _p(W), _p(y32), _p(y64) if want64 else None, _p(y16), M, N, K)
    return y32, y64, y16.view(np.float16)


def w4a16_gemm(x, qweight, scales, qzeros, G: int = 128, want64: bool = True):
    """The whole layer: returns (y32, y64 or None, y16)."""
    W = dequant(qweight, scales, qzeros, G)
    return matmul(x, W, want64)


# ---------------------------------------------------------------------------------------------
# tree-verify attention, fp64


def tree_verify_attn(q, k, v, mask, scale: float | None = None):
    """q fp16 [M, Hq, D]; k, v fp16 [P+M, Hkv, D]; mask [M, M] (non-zero = visible).
    Query row i of head h attends, through KV head h // (Hq/Hkv), to all P prefix keys and to the
    draft keys j with mask[i, j] != 0.  Returns (out64 [M, Hq, D] fp64, out16 fp16)."""
    q = np.asarray(q)
    k = np.asarray(k)
    v = np.asarray(v)
    mask = np.asarray(mask)
    M, Hq, D = q.shape
    T, Hkv, _ = k.shape
    P = T - M
    assert P >= 0 and mask.shape == (M, M) and Hq % Hkv == 0
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    rep = Hq // Hkv
    q64, k64, v64 = q.astype(np.float64), k.astype(np.float64), v.astype(np.float64)
    out = np.zeros((M, Hq, D), dtype=np.float64)
    for i in range(M):
        visible = np.concatenate([np.ones(P, dtype=bool), mask[i] != 0])
        for h in range(Hq):
            kh = h // rep
            logits = scale * (k64[visible, kh, :] @ q64[i, h, :])
            logits -= logits.max()
            p = np.exp(logits)
            p /= p.sum()
            out[i, h, :] = p @ v64[visible, kh, :]
    return out, out.astype(np.float16)


# ---------------------------------------------------------------------------------------------
# greedy acceptance of a verified draft tree and compaction of the accepted K/V rows


def tree_accept(parent, token, target):
    """Greedy draft-then-verify acceptance on a tree draft (paper section 2.1: the target model
    verifies the n draft-tree tokens in one pass and accepts some of them; section 4: verifying a
    tree turns it into a sequence).  Node 0 is the root, i.e. the last committed token; parent[i] < i.
    token[i] is the draft token at node i, target[i] the target model's greedy next token after
    the sequence ending in node i.  The walk starts at the root; at node cur, a child is accepted
    iff its draft token equals target[cur]; among several such children the lowest index is taken;
    the walk stops at the first node without an accepted child.
    Returns (path, next_token): the accepted node indices, root first, and target[path[-1]], the
    token the target model itself contributes after the last accepted node.  Pure integer work."""
    parent = [int(p) for p in parent]
    token = [int(t) for t in token]
    target = [int(t) for t in target]
    n = len(parent)
    assert n >= 1 and parent[0] < 0 and all(0 <= parent[i] < i for i in range(1, n))
    path = [0]
    cur = 0
    while True:
        nxt = -1
        for i in range(cur + 1, n):
            if parent[i] == cur and token[i] == target[cur]:
                nxt = i
                break
        if nxt < 0:
            break
        path.append(nxt)
        cur = nxt
    return path, target[cur]


def kv_compact(k, v, path, P: int):
    """After acceptance the cache keeps the accepted nodes only, in order: cache row P + j receives
    the K and V rows of node path[j] (stored at row P + path[j]) for every j < len(path).  Rows
    below P and rows from P + len(path) on are left as they are.  Returns new arrays."""
    k2, v2 = np.array(k, copy=True), np.array(v, copy=True)
    for j, node in enumerate(path):
        k2[P + j] = k[P + node]
        v2[P + j] = v[P + node]
    return k2, v2


# ---------------------------------------------------------------------------------------------
# the other steps of a decoder layer around the four linears (paper section 2.1: one target-model
# forward pass over the draft tokens is the unit of cost T_v(n); the target is a Llama-3 model, whose
# layer is  h += Wo.attn(rope(Wqkv.norm(h)));  h += Wdown.(silu(Wgate.norm(h)) * Wup.norm(h)) ).
# All in fp64 from the fp16 inputs, one rounding to fp16 at the end of each function.


def silu(v):
    """v * sigmoid(v) = v / (1 + exp(-v)), fp64"""
    v = np.asarray(v, dtype=np.float64)
    return v / (1.0 + np.exp(-v))


def rms_norm(x, gamma, eps: float):
    """x fp16 [M, K], gamma fp16 [K] -> (y64, y16):  y[m,k] = x[m,k] * gamma[k] / sqrt(mean_k x[m,:]^2 + eps)"""
    x64 = np.asarray(x).astype(np.float64)
    g64 = np.asarray(gamma).astype(np.float64)
    ms = (x64 * x64).sum(axis=1, keepdims=True) / x64.shape[1]
    y = x64 * g64[None, :] / np.sqrt(ms + float(eps))
    return y, y.astype(np.float16)


def w4a16_gemm_residual(x, qweight, scales, qzeros, residual, G: int = 128):
    """(y64, y16):  y = residual + x . W   (the o_proj and down projections add into the hidden state)"""
    _, y64, _ = w4a16_gemm(x, qweight, scales, qzeros, G, want64=True)
    y = y64 + np.asarray(residual).astype(np.float64)
    return y, y.astype(np.float16)


def w4a16_gemm_silu_mul(x, qweight, scales, qzeros, G: int = 128):
    """(y64, y16) of shape [M, N/2]: columns 0..N/2-1 of the weight are the gate projection, columns
    N/2..N-1 the up projection;  y[m,n] = silu(x.W[:, n]) * (x.W[:, N/2 + n])"""
    _, y64, _ = w4a16_gemm(x, qweight, scales, qzeros, G, want64=True)
    half = y64.shape[1] // 2
    assert 2 * half == y64.shape[1]
    y = silu(y64[:, :half]) * y64[:, half:]
    return y, y.astype(np.float16)


def rope_append(qkv, pos, cos, sin, k_cache, v_cache, P: int, Hq: int, Hkv: int, D: int):
    """Rotary position embedding of the q and k parts of a fused projection output and the append of
    the new keys and values to the cache.
    qkv fp16 [M, (Hq + 2 Hkv) D]: per row Hq query heads, then Hkv key heads, then Hkv value heads;
    pos int [M]: position of each row (for a draft tree: prefix length + depth of the node);
    cos, sin fp32 [n_pos, D/2]: caller's tables, entry [p, i] belongs to position p and the pair of
    head elements (i, i + D/2):  out[i] = a[i] cos - a[i + D/2] sin,  out[i + D/2] = a[i + D/2] cos + a[i] sin.
    Returns (q64 [M, Hq, D], q16, k_cache', v_cache') where rows P..P+M-1 of the fp16 caches
    [>= P+M, Hkv, D] hold the rotated keys and the unchanged values; other rows are untouched."""
    qkv = np.asarray(qkv)
    M = qkv.shape[0]
    assert qkv.shape[1] == (Hq + 2 * Hkv) * D and D % 2 == 0
    a = qkv.astype(np.float64).reshape(M, Hq + 2 * Hkv, D)
    c = np.asarray(cos).astype(np.float64)[np.asarray(pos)][:, None, :]   # [M, 1, D/2]
    s = np.asarray(sin).astype(np.float64)[np.asarray(pos)][:, None, :]
    h = D // 2

    def rot(t):
        lo, hi = t[..., :h], t[..., h:]
        return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)

    q = rot(a[:, :Hq])
    k = rot(a[:, Hq:Hq + Hkv])
    k2, v2 = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    k2[P:P + M] = k.astype(np.float16)
    v2[P:P + M] = qkv.reshape(M, Hq + 2 * Hkv, D)[:, Hq + Hkv:]
    return q, q.astype(np.float16), k2, v2


# ---------------------------------------------------------------------------------------------
# draft side: fp16 language-model head, log-softmax and top-k (paper section 2.1: the draft model
# uses the target's LM head and expands its beam search by the softmax output; section 3.1: the
# draft stays in fp16 because LM head and softmax are its bottleneck and are not quantisable)


def lm_head_topk(x, W, top_k: int):
    """x fp16 [M, K] (draft hidden states), W fp16 [V, K] (LM-head weight, one row per token).
    logits[m, v] = sum_k x[m, k] W[v, k];  logprob = logits - log(sum_v exp(logits)), per row.
    Returns (logits64 [M, V], idx int64 [M, top_k], logprob64 [M, top_k]): per row the top_k tokens by
    logit, largest first, equal logits in ascending token order, with their log-probabilities."""
    x64 = np.asarray(x).astype(np.float64)
    W64 = np.asarray(W).astype(np.float64)
    logits = x64 @ W64.T
    mx = logits.max(axis=1, keepdims=True)
    lse = mx[:, 0] + np.log(np.exp(logits - mx).sum(axis=1))
    M, V = logits.shape
    idx = np.empty((M, top_k), dtype=np.int64)
    for m in range(M):
        order = sorted(range(V), key=lambda v: (-logits[m, v], v))   # plain definition of the order
        idx[m] = order[:top_k]
    lp = np.take_along_axis(logits, idx, axis=1) - lse[:, None]
    return logits, idx, lp
