"""Seeded synthetic inputs for the W4A16 linear layer and the tree-verify attention step.

This module only draws random numbers and arranges them in the canonical interchange format
(int32 words holding eight 4-bit fields).  It contains none of the method's arithmetic: no
dequantisation, no contraction, no softmax.  Both the CPU oracle's tests and the GPU tests
take their inputs from here, so that the two sides see identical bits.

Canonical format (group-wise 4-bit weights with fp16 activations, paper section 2.2; the
paper does not print a storage layout, so the widespread one is used):
  qweight int32 [K/8, N]   code of row k in bits 4*(k%8) .. 4*(k%8)+3 of word [k//8, n]
  scales  fp16  [K/G, N]
  qzeros  int32 [K/G, N/8] zero-point of column n in bits 4*(n%8) .. +3 of word [g, n//8]

The real workloads (GPTQ-quantised Llama-3 weights, MT-Bench / SpecBench activations) are not
available offline; these generators stand in for them with the same shapes, dtypes and value
ranges.
"""
from __future__ import annotations

import dataclasses

import numpy as np

SEED_BASE = 20250522 * 1000

#: (name, K, N) of the four linears of one decoder layer
LLAMA3_8B = (("qkv", 4096, 6144), ("o_proj", 4096, 4096), ("gate_up", 4096, 28672), ("down", 14336, 4096))
LLAMA3_70B = (("qkv", 8192, 10240), ("o_proj", 8192, 8192), ("gate_up", 8192, 57344), ("down", 28672, 8192))
M_SWEEP_8B = (1, 4, 8, 16, 32, 48, 64)
M_SWEEP_70B = (1, 4, 8, 16, 32, 64)


def seed_for(config_index: int, gemm_index: int) -> int:
    return SEED_BASE + 100 * config_index + gemm_index


def pack_rows(codes: np.ndarray) -> np.ndarray:
    """uint8 [K, N] with values 0..15 -> int32 [K/8, N]; eight consecutive rows share a word."""
    K, N = codes.shape
    assert K % 8 == 0
    c = codes.astype(np.uint32).reshape(K // 8, 8, N)
    word = np.zeros((K // 8, N), dtype=np.uint32)
    for i in range(8):
        word |= c[:, i, :] << np.uint32(4 * i)
    return word.view(np.int32)


def pack_cols(zeros: np.ndarray) -> np.ndarray:
    """uint8 [R, N] with values 0..15 -> int32 [R, N/8]; eight consecutive columns share a word."""
    R, N = zeros.shape
    assert N % 8 == 0
    z = zeros.astype(np.uint32).reshape(R, N // 8, 8)
    word = np.zeros((R, N // 8), dtype=np.uint32)
    for i in range(8):
        word |= z[:, :, i] << np.uint32(4 * i)
    return word.view(np.int32)


@dataclasses.dataclass
class LinearInputs:
    M: int
    K: int
    N: int
    G: int
    x: np.ndarray        # fp16 [M, K]
    codes: np.ndarray    # uint8 [K, N]   (what qweight encodes; kept for tests)
    zeros: np.ndarray    # uint8 [K/G, N] (what qzeros encodes)
    qweight: np.ndarray  # int32 [K/8, N]
    scales: np.ndarray   # fp16 [K/G, N]
    qzeros: np.ndarray   # int32 [K/G, N/8]


def make_linear(seed: int, M: int, K: int, N: int, G: int = 128, *, x_kind: str = "normal",
                scale_kind: str = "uniform", m_max: int | None = None, zero_kind: str = "uniform") -> LinearInputs:
    """Draw order: x [m_max, K], codes [K, N], scales [K/G, N], zeros [K/G, N].

    x_kind:     "normal"  fp16(N(0,1))            | "small_int" uniform in {-2,-1,0,1,2}
    scale_kind: "uniform" fp16(U[1e-3, 1e-2])     | "pow2" the constant 2**-7
    zero_kind:  "uniform" integers in 0..15       | "eight" the constant 8 (a symmetrically quantised weight,
                the scheme of paper section 2.2)
    Rows 0..M-1 of the x draw are returned, so a smaller M sees a prefix of the same matrix.
    """
    assert K % G == 0 and K % 8 == 0 and N % 8 == 0
    rng = np.random.default_rng(seed)
    m_draw = max(M, m_max or M)
    if x_kind == "normal":
        x = rng.standard_normal((m_draw, K), dtype=np.float32).astype(np.float16)
    elif x_kind == "small_int":
        x = rng.integers(-2, 3, size=(m_draw, K)).astype(np.float16)
    else:
        raise ValueError(x_kind)
    codes = rng.integers(0, 16, size=(K, N), dtype=np.uint8)
    if scale_kind == "uniform":
        scales = rng.uniform(1e-3, 1e-2, size=(K // G, N)).astype(np.float16)
    elif scale_kind == "pow2":
        rng.uniform(1e-3, 1e-2, size=(K // G, N))  # keep the stream position identical
        scales = np.full((K // G, N), 2.0 ** -7, dtype=np.float16)
    else:
        raise ValueError(scale_kind)
    zeros = rng.integers(0, 16, size=(K // G, N), dtype=np.uint8)
    if zero_kind == "eight":
        zeros = np.full((K // G, N), 8, dtype=np.uint8)   # drawn all the same: the stream position stays identical
    elif zero_kind != "uniform":
        raise ValueError(zero_kind)
    return LinearInputs(M, K, N, G, np.ascontiguousarray(x[:M]), codes, zeros,
                        pack_rows(codes), scales, pack_cols(zeros))


# ----------------------------------------------------------------------------------------------
# draft tree for the verify step (paper section 2.1: a tree of n draft tokens found by a depth-d
# beam search; the target model scores all n in one pass under an ancestor mask)


def make_tree(seed: int, n_nodes: int = 60, depth: int = 6, max_children: int = 4):
    """Random draft tree.  Node 0 is the root (depth 0); parent[i] < i; every node has at most
    `max_children` children; the deepest node sits at exactly `depth`.  Returns (parent, depth_of,
    mask) with mask uint8 [n, n], mask[i, j] = 1 iff j == i or j is an ancestor of i."""
    attempt = 0
    while True:
        rng = np.random.default_rng([seed, attempt])
        parent = np.full(n_nodes, -1, dtype=np.int64)
        dep = np.zeros(n_nodes, dtype=np.int64)
        nchild = np.zeros(n_nodes, dtype=np.int64)
        for i in range(1, n_nodes):
            cand = [j for j in range(i) if dep[j] < depth and nchild[j] < max_children]
            p = cand[int(rng.integers(0, len(cand)))]
            parent[i] = p
            dep[i] = dep[p] + 1
            nchild[p] += 1
        if dep.max() == depth or n_nodes <= depth:
            break
        attempt += 1
    return parent, dep, ancestor_mask(parent)


def chain_tree(n_nodes: int):
    parent = np.arange(-1, n_nodes - 1, dtype=np.int64)
    return parent, np.arange(n_nodes, dtype=np.int64), ancestor_mask(parent)


def ancestor_mask(parent: np.ndarray) -> np.ndarray:
    n = len(parent)
    mask = np.zeros((n, n), dtype=np.uint8)
    for i in range(n):
        j = i
        while j >= 0:
            mask[i, j] = 1
            j = int(parent[j])
    return mask


@dataclasses.dataclass
class AttnInputs:
    M: int
    P: int
    Hq: int
    Hkv: int
    D: int
    q: np.ndarray     # fp16 [M, Hq, D]
    k: np.ndarray     # fp16 [P+M, Hkv, D]
    v: np.ndarray     # fp16 [P+M, Hkv, D]
    mask: np.ndarray  # uint8 [M, M]
    parent: np.ndarray
    scale: float


def make_attn(seed: int, M: int = 60, P: int = 2048, Hq: int = 64, Hkv: int = 8, D: int = 128,
              *, tree: str = "random", depth: int = 6, max_children: int = 4) -> AttnInputs:
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((M, Hq, D), dtype=np.float32).astype(np.float16)
    k = rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16)
    v = rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16)
    if tree == "random":
        parent, _, mask = make_tree(seed + 7, M, depth, max_children)
    elif tree == "chain":
        parent, _, mask = chain_tree(M)
    elif tree == "identity":
        parent = np.full(M, -1, dtype=np.int64)
        mask = np.eye(M, dtype=np.uint8)
    else:
        raise ValueError(tree)
    return AttnInputs(M, P, Hq, Hkv, D, q, k, v, mask, parent, 1.0 / float(np.sqrt(D)))


def make_verify(seed: int, parent: np.ndarray, vocab: int = 128256, p_accept: float = 0.7):
    """Draft tokens and target-model greedy tokens for a draft tree (stand-ins for a draft model's
    beam-search tokens and the target model's argmax, which need trained weights).  Siblings carry
    distinct tokens, as the children of a beam-search node do.  For every node the target token
    equals the token of one of its children (picked uniformly) with probability p_accept, and is
    otherwise a token none of its children carries.  Returns (token int32 [n], target int32 [n])."""
    rng = np.random.default_rng(seed)
    n = len(parent)
    children = [[] for _ in range(n)]
    for i in range(1, n):
        children[int(parent[i])].append(i)
    token = np.zeros(n, dtype=np.int32)
    token[0] = int(rng.integers(0, vocab))
    for p in range(n):
        if children[p]:
            draws = rng.choice(vocab, size=len(children[p]), replace=False)
            for ch, t in zip(children[p], draws):
                token[ch] = int(t)
    target = np.zeros(n, dtype=np.int32)
    for p in range(n):
        kids = children[p]
        if kids and rng.random() < p_accept:
            target[p] = token[kids[int(rng.integers(0, len(kids)))]]
        else:
            taken = {int(token[ch]) for ch in kids}
            t = int(rng.integers(0, vocab))
            while t in taken:
                t = int(rng.integers(0, vocab))
            target[p] = t
    return token, target


def make_hidden(seed: int, M: int, K: int, n_outlier_channels: int = 8) -> np.ndarray:
    """fp16 [M, K] stand-in for a decoder layer's hidden state: unit normal with a few channels of
    eight times the spread (transformer residual streams carry such outlier channels)."""
    rng = np.random.default_rng(seed)
    h = rng.standard_normal((M, K), dtype=np.float32)
    if n_outlier_channels:
        cols = rng.choice(K, size=min(n_outlier_channels, K), replace=False)
        h[:, cols] *= 8.0
    return h.astype(np.float16)


def make_gamma(seed: int, K: int) -> np.ndarray:
    """fp16 [K] norm weights around one"""
    rng = np.random.default_rng(seed)
    return (1.0 + 0.1 * rng.standard_normal(K, dtype=np.float32)).astype(np.float16)


def make_rope_tables(n_pos: int, D: int = 128, base: float = 500000.0):
    """The caller-supplied rotary tables of the boundary: cos, sin fp32 [n_pos, D/2] of the angle
    p * base^(-2i/D) for position p and element pair i (base of the Llama-3 models)."""
    i = np.arange(D // 2, dtype=np.float64)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * base ** (-2.0 * i / D)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def tree_positions(parent: np.ndarray, P: int) -> np.ndarray:
    """int32 [n]: position of each draft-tree node = P + its depth (root at depth 0)"""
    n = len(parent)
    depth = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        depth[i] = depth[int(parent[i])] + 1
    return (P + depth).astype(np.int32)


def make_lm_head(seed: int, M: int, K: int, V: int, w_std: float = 0.02):
    """Draft hidden states x fp16 [M, K] ~ N(0, 1) and an LM-head weight W fp16 [V, K] ~ N(0, w_std^2)
    (stand-ins for an EAGLE-2 draft layer's output and Llama-3's output embedding): logits of spread
    sqrt(K) * w_std."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K), dtype=np.float32).astype(np.float16)
    W = (rng.standard_normal((V, K), dtype=np.float32) * np.float32(w_std)).astype(np.float16)
    return x, W
