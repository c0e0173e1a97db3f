#!/usr/bin/env python3
"""Benchmark of the W4A16 small-M linear layer on one MI355X.

A "step" is one pass over the four W4A16 linears of one Llama-3-70B decoder layer (qkv, o_proj,
gate_up, down; group size 128) at M token rows, with all operands already resident in HBM.  The
headline value is the weight-HBM rate at M = 1 (bytes of codes + scales + zero-points streamed per
second); the same loop is repeated for the other M of the sweep, for the Llama-3-8B layer, and for
the tree-verify step (attention + the four linears at M = 60).  Consecutive steps use different
copies of the layer's weights so that no byte is served by the 256 MB last-level cache.

Prints ONE JSON line (see the keys below) and nothing else on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2505_22179_amd import binding as B  # noqa: E402
from paper_2505_22179_amd import inputs as I  # noqa: E402

MFMA_F16_PEAK_FLOPS = 2.5e15   # dense fp16 matrix peak of MI355X
HBM_PEAK_GBPS = 8000.0
G = 128


def weight_bytes(K: int, N: int) -> int:
    """algorithmic bytes of one GEMM's weight: 4-bit codes + fp16 scales + 4-bit zero-points"""
    return K * N // 2 + (K // G) * N * 2 + (K // G) * N // 2


HEAD_DIM = 128   # of both Llama-3 models


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """Packed weights of one decoder layer's four linears, `copies` times, built on the device
    from seeded uniform codes / zero-points and U[1e-3, 1e-2] fp16 scales."""

    def __init__(self, shapes, copies: int, seed: int, symmetric: bool = False):
        """symmetric: every zero-point is 8 (the paper's GPTQ scheme is symmetric) and the linears are called with
        W4A16_SYMMETRIC; otherwise zero-points are uniform in 0..15 as the benchmark configurations state"""
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        self.shapes = shapes
        self.copies = copies
        self.symmetric = symmetric
        self.packed = []   # [copy][gemm]
        first = []
        for (name, K, N) in shapes:
            qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (K // 8, N), dtype=torch.int32, device="cuda", generator=gen)
            sc = (torch.rand((K // G, N), device="cuda", generator=gen) * 9e-3 + 1e-3).to(torch.float16)
            qz = torch.randint(-2 ** 31, 2 ** 31 - 1, (K // G, N // 8), dtype=torch.int32, device="cuda", generator=gen)
            if symmetric:
                qz.fill_(-0x77777778)   # 0x88888888: eight zero-points of 8 per word
            p = torch.empty(B.w4a16_packed_bytes(N, K, G), dtype=torch.uint8, device="cuda")
            # gate_up in the paired tile order the fused SiLU-gate epilogue reads, qkv with the halves of every head
            # paired for the rotary epilogue (same bytes, same cost for the plain GEMM)
            if name == "gate_up":
                B.w4a16_pack_gate_up(qw, sc, qz, p, N, K, G)
            elif name == "qkv":
                B.w4a16_pack_heads(qw, sc, qz, p, N, K, HEAD_DIM, G)
            else:
                B.w4a16_pack(qw, sc, qz, p, N, K, G)
            first.append(p)
            del qw, sc, qz
        self.packed.append(first)
        for _ in range(copies - 1):
            self.packed.append([p.clone() for p in first])
        torch.cuda.synchronize()
        self.x = {}
        self.y = {}
        self.bytes = sum(weight_bytes(K, N) for (_, K, N) in shapes)
        ws_bytes = max(B.w4a16_workspace_bytes(64, N, K, G) for (_, K, N) in shapes)
        self.ws = B.new_workspace(ws_bytes)

    def buffers(self, M: int):
        if M not in self.x:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(1000 + M)
            self.x[M] = [torch.randn((M, K), device="cuda", generator=gen).to(torch.float16) for (_, K, N) in self.shapes]
            self.y[M] = [torch.empty((M, N), dtype=torch.float16, device="cuda") for (_, K, N) in self.shapes]
        return self.x[M], self.y[M]

    def step(self, M: int, copy: int, only: int | None = None):
        xs, ys = self.buffers(M)
        for gi, (_, K, N) in enumerate(self.shapes):
            if only is not None and gi != only:
                continue
            if self.symmetric:
                B.w4a16_gemm_fused(xs[gi], self.packed[copy][gi], ys[gi], M, N, K, G, B.EPI_NONE | B.SYMMETRIC, None, self.ws)
            else:
                B.w4a16_gemm(xs[gi], self.packed[copy][gi], ys[gi], M, N, K, G, self.ws)

    def solo_copies(self, gi: int, min_bytes: int = 700_000_000):
        """Enough distinct copies of one GEMM's weights that a loop over it alone never re-reads
        bytes the 256 MB last-level cache could still hold."""
        _, K, N = self.shapes[gi]
        need = max(3, min_bytes // weight_bytes(K, N) + 1)
        while len(self.packed) < need:
            self.packed.append([None] * len(self.shapes))
        for c in range(need):
            if self.packed[c][gi] is None:
                self.packed[c][gi] = self.packed[0][gi].clone()
        return need


class DecoderLayer:
    """One whole decoder layer of the target model on M draft-tree tokens over a P-token prefix, chained
    through w4a16_decoder_layer: norm, qkv with the rotary embedding and the K/V append in its store, tree
    attention, o_proj + residual, norm, gate/up with the SiLU gate, down + residual (7 kernel launches plus the
    split-K / merge passes).  The
    hidden state of a step is one of several kept per object and is updated in place."""

    def __init__(self, layer: "Layer", M: int, P: int, kv_copies: int, Hq: int = 64, Hkv: int = 8, D: int = 128):
        self.L, self.M, self.P, self.Hq, self.Hkv, self.D = layer, M, P, Hq, Hkv, D
        (_, H, Nqkv), _, (_, _, Ngu), _ = layer.shapes
        assert Nqkv == (Hq + 2 * Hkv) * D and H == Hq * D
        self.H, self.Nqkv, self.Ngu = H, Nqkv, Ngu
        f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device="cuda")
        self.h = torch.from_numpy(I.make_hidden(4242 + M, M, H)).cuda()
        self.g1 = torch.from_numpy(I.make_gamma(4243, H)).cuda()
        self.g2 = torch.from_numpy(I.make_gamma(4244, H)).cuda()
        self.n1, self.qkv, self.q, self.att = f16(M, H), f16(M, Nqkv), f16(M, Hq, D), f16(M, Hq, D)
        self.act = f16(M, Ngu // 2)
        # one hidden state per step of a replayed graph.  The layer updates it in place; both branches start
        # with a norm, so every application adds a bounded update and the values stay far inside the fp16
        # range over the few hundred applications of a benchmark run (no copy has to be timed)
        self.h_work = [self.h.clone() for _ in range(kv_copies)]
        if M > 1:
            parent, _, mask = I.make_tree(I.seed_for(5, 0) + 7, M, 6, 4)
        else:
            parent, mask = np.array([-1]), np.ones((1, 1), dtype=np.uint8)
        self.mask = torch.from_numpy(mask).cuda()
        self.pos = torch.from_numpy(I.tree_positions(parent, P)).cuda()
        cos, sin = I.make_rope_tables(P + 64, D)
        self.cos, self.sin, self.n_pos = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda(), P + 64
        gen = torch.Generator(device="cuda")
        gen.manual_seed(77)
        k0 = torch.randn((P + M, Hkv, D), device="cuda", generator=gen).to(torch.float16)
        v0 = torch.randn((P + M, Hkv, D), device="cuda", generator=gen).to(torch.float16)
        self.k = [k0] + [k0.clone() for _ in range(kv_copies - 1)]
        self.v = [v0] + [v0.clone() for _ in range(kv_copies - 1)]
        self.aws = B.new_workspace(B.tree_verify_attn_workspace_bytes(M, P, Hq, Hkv, D))
        self.scale = 1.0 / float(np.sqrt(D))

    def step(self, c: int):
        L, M, P, Hq, Hkv, D, H = self.L, self.M, self.P, self.Hq, self.Hkv, self.D, self.H
        w = L.packed[c % L.copies]
        k, v = self.k[c % len(self.k)], self.v[c % len(self.v)]
        weights = B.layer_weights(w[0], w[1], w[2], w[3], self.g1, self.g2, H, Hq, Hkv, D, self.Ngu // 2, 1e-5,
                                  qkv_heads_packed=True)
        scratch = B.layer_scratch(self.n1, self.qkv, self.q, self.att, self.act, L.ws, self.aws)
        hs = self.h_work[c % len(self.h_work)]   # updated in place
        B.w4a16_decoder_layer(weights, hs, M, P, self.pos, self.cos, self.sin, self.n_pos, self.mask, k, v, scratch)


class Model:
    """A whole target model on the device: n_layers decoder layers with their own packed weights (copies of
    one synthetic layer: the addresses differ, which is all that matters to the memory system) and their
    own K/V caches, a final norm and the fp16 LM head.  forward(M) enqueues one pass over M token rows:
    plain decoding for M = 1, verification of an M-token draft tree otherwise."""

    def __init__(self, shapes, n_layers: int, Hq: int, Hkv: int, D: int, P: int, seed: int, V: int = 128256, M_max: int = 64):
        self.layers = Layer(shapes, n_layers, seed)
        self.n_layers, self.Hq, self.Hkv, self.D, self.P, self.V = n_layers, Hq, Hkv, D, P, V
        (_, H, Nqkv), _, (_, _, Ngu), _ = shapes
        self.H, self.Nqkv, self.F = H, Nqkv, Ngu // 2
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed + 1)
        f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device="cuda")
        self.g = [torch.from_numpy(I.make_gamma(seed + 2 + i, H)).cuda() for i in range(3)]   # norm 1, norm 2, final
        self.k = [torch.randn((P + M_max, Hkv, D), device="cuda", generator=gen).to(torch.float16) for _ in range(n_layers)]
        self.v = [torch.randn((P + M_max, Hkv, D), device="cuda", generator=gen).to(torch.float16) for _ in range(n_layers)]
        raw = (torch.randn((V, H), device="cuda", generator=gen) * 0.02).to(torch.float16)
        self.head = torch.empty(B.lm_head_packed_bytes(V, H), dtype=torch.uint8, device="cuda")
        B.lm_head_pack(raw, self.head, V, H)
        del raw
        cos, sin = I.make_rope_tables(P + 64, D)
        self.cos, self.sin, self.n_pos = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda(), P + 64
        self.bufs = {}
        self.f16 = f16
        self.bytes = self.layers.bytes * n_layers + V * H * 2

    def buffers(self, M: int):
        if M not in self.bufs:
            f16, H = self.f16, self.H
            if M > 1:
                parent, _, mask = I.make_tree(I.seed_for(5, 0) + 7, M, 6, 4)
            else:
                parent, mask = np.array([-1]), np.ones((1, 1), dtype=np.uint8)
            b = {"h0": torch.from_numpy(I.make_hidden(777 + M, M, H)).cuda(), "h": f16(M, H), "hn": f16(M, H),
                 "mask": torch.from_numpy(mask).cuda(), "pos": torch.from_numpy(I.tree_positions(parent, self.P)).cuda(),
                 "logits": torch.empty((M, self.V), dtype=torch.float32, device="cuda"),
                 "top_idx": torch.empty((M, 1), dtype=torch.int32, device="cuda"),
                 "top_lp": torch.empty((M, 1), dtype=torch.float32, device="cuda"),
                 "aws": B.new_workspace(B.tree_verify_attn_workspace_bytes(M, self.P, self.Hq, self.Hkv, self.D)),
                 "lws": torch.empty(B.lm_head_workspace_bytes(M, self.V, H, 1), dtype=torch.uint8, device="cuda")}
            b["scratch"] = B.layer_scratch(f16(M, H), f16(M, self.Nqkv), f16(M, self.Hq, self.D), f16(M, self.Hq, self.D),
                                           f16(M, self.F), self.layers.ws, b["aws"])
            b["keep"] = []   # the scratch struct holds raw pointers: keep the tensors alive
            self.bufs[M] = b
        return self.bufs[M]

    def forward(self, M: int):
        b, L = self.buffers(M), self.layers
        b["h"].copy_(b["h0"])   # the embedding lookup's stand-in: a fresh hidden state per pass
        for l in range(self.n_layers):
            w = L.packed[l]
            weights = B.layer_weights(w[0], w[1], w[2], w[3], self.g[0], self.g[1], self.H, self.Hq, self.Hkv, self.D,
                                      self.F, 1e-5, qkv_heads_packed=True)
            B.w4a16_decoder_layer(weights, b["h"], M, self.P, b["pos"], self.cos, self.sin, self.n_pos, b["mask"],
                                  self.k[l], self.v[l], b["scratch"])
        B.rms_norm(b["h"], self.g[2], b["hn"], M, self.H, 1e-5)
        # greedy target tokens of all M rows
        B.lm_head_topk(b["hn"], self.head, M, self.V, self.H, 1, b["logits"], b["top_idx"], b["top_lp"], b["lws"])


def model_leg(name: str, shapes, n_layers: int, Hq: int, Hkv: int, Ms, args, use_graph: bool) -> dict:
    """One whole forward pass of the target per step (all layers with their own weights and caches, final
    norm, LM head with greedy tokens): T_t at M = 1 and T_v(M) measured, not extrapolated from one layer."""
    model = Model(shapes, n_layers, Hq, Hkv, 128, 2048, seed=1000 + n_layers)
    out = {}
    for M in Ms:
        steps, warm = max(5, min(args.steps, 20)), 3
        ms = time_steps(lambda c, M=M: model.forward(M), steps, warm, use_graph, 1, repeats=5)
        out[str(M)] = {"ms_per_forward": ms}
        log(f"{name} whole model M={M}: {ms:.3f} ms per forward pass")
    t_t = out["1"]["ms_per_forward"]
    for M in Ms:
        out[str(M)]["ratio_vs_M1"] = out[str(M)]["ms_per_forward"] / t_t
    out["plain_decoding_tokens_per_s"] = 1e3 / t_t
    out["weight_GBps_at_M1"] = model.bytes / t_t / 1e6
    out["note"] = (f"{n_layers} decoder layers + final norm + fp16 LM head (greedy tokens for all rows), prefix 2048, "
                   "one HIP graph per pass")
    del model
    torch.cuda.empty_cache()
    return out


# Expected accepted length tau(n, d) of EAGLE-2 on the W4A16 targets, read off the paper's figures
# "Accepted Length (70B, A100)" and "Accepted Length (8B, A100)" (W4A16 series; tree size n: (d draft
# passes, tau)), and the same figure groups' verification-to-decoding time ratios on an A100.
PAPER_TAU_70B_W4A16 = {24: (3, 3.283), 32: (4, 3.630), 40: (5, 3.819), 48: (6, 3.926)}
PAPER_RATIO_70B_W4A16_A100 = {24: 1.262, 32: 1.287, 40: 1.555, 48: 1.580}
PAPER_TAU_8B_W4A16 = {30: (3, 3.300), 40: (4, 3.669), 50: (5, 3.902), 60: (6, 4.046)}
PAPER_RATIO_8B_W4A16_A100 = {30: 1.317, 40: 1.548, 50: 1.790, 60: 1.803}


def eq1_projection(layer_ms: dict, read_GBps: float, *, shapes=None, n_layers: int = 80, tau=None, paper_ratio=None,
                   lm_head_ms: float | None = None, draft_lm_head_ms: float | None = None, model_ms: dict | None = None) -> dict:
    """The paper's speedup model (Eq. 1), T_sd/T_t = (d T_d/T_t + T_v(n)/T_t) / tau(n, d), fed with
    this GPU's measured decoder-layer times for T_v(n)/T_t and the paper's tau.  The draft model is
    not built here: its time is ESTIMATED as the bytes one pass of an EAGLE-2 draft has to stream (one
    fp16 decoder layer of the target's shape and the 2H->H fusion layer) at the plain-read rate
    measured above, plus the fp16 LM head -- measured with lm_head_topk when given (draft_lm_head_ms
    for the draft's beam, lm_head_ms for the target's own head, added to both T_t and T_v), else
    estimated from its bytes too.  With model_ms (ms per whole forward pass by M, as measured by model_leg)
    T_t and T_v(n) are those measured passes instead of n_layers x one layer + head.  A projection for
    context, not a measurement of speculative decoding."""
    shapes = I.LLAMA3_70B if shapes is None else shapes
    tau = PAPER_TAU_70B_W4A16 if tau is None else tau
    paper_ratio = PAPER_RATIO_70B_W4A16_A100 if paper_ratio is None else paper_ratio
    H, V = shapes[0][1], 128256
    layer_params = sum(K * N for (_, K, N) in shapes)
    head_by_bytes = V * H * 2 / (read_GBps * 1e6)
    lm_t = head_by_bytes if lm_head_ms is None else lm_head_ms
    lm_d = head_by_bytes if draft_lm_head_ms is None else draft_lm_head_ms
    draft_ms = (layer_params * 2 + 2 * H * H * 2) / (read_GBps * 1e6) + lm_d
    t_t = model_ms[1] if model_ms else layer_ms[1] * n_layers + lm_t
    out = {"inputs": {"tau": "paper, figures 'Accepted Length (70B / 8B, A100)', W4A16 series",
                      "T_v_over_T_t": ("measured here: whole forward passes (all layers, final norm, LM head with greedy tokens)"
                                       if model_ms else f"measured here: {n_layers} x decoder layer (prefix 2048) + fp16 LM head"),
                      "T_d": "fp16 draft layer estimated from bytes at the measured plain-read rate, not measured",
                      "lm_head": "measured (lm_head_topk)" if lm_head_ms is not None else "estimated from bytes",
                      "T_t_ms": t_t, "T_d_ms_estimated": draft_ms, "lm_head_ms": lm_t}}
    for n, (d, ta) in tau.items():
        t_v = model_ms[n] if model_ms else layer_ms[n] * n_layers + lm_t
        out[str(n)] = {"d": d, "tau_paper": ta, "T_v_over_T_t": t_v / t_t,
                       "T_v_over_T_t_paper_A100": paper_ratio[n],
                       "speedup_over_own_autoregressive_no_draft_cost": ta / (t_v / t_t),
                       "speedup_over_own_autoregressive_estimated_draft": ta / (d * draft_ms / t_t + t_v / t_t)}
    return out


def lm_head_leg(args, use_graph: bool) -> dict:
    """Draft side: fp16 LM head of the Llama-3 vocabulary + log-softmax + top-10, for the draft models of
    the 8B (K = 4096) and 70B (K = 8192) targets; each weight (1.05 / 2.1 GB) exceeds the last-level cache."""
    lm = {}
    V, top_k = 128256, 10
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    for K in (4096, 8192):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(4096 + K)
        Ws = []
        for _ in range(2):
            raw = (torch.randn((V, K), device="cuda", generator=gen) * 0.02).to(torch.float16)
            pk = torch.empty(B.lm_head_packed_bytes(V, K), dtype=torch.uint8, device="cuda")
            B.lm_head_pack(raw, pk, V, K)
            Ws.append(pk)
            del raw
        nbytes = V * K * 2
        steps, warm = min(args.steps, 60), min(args.warmup, 6)
        ms_read = time_steps(lambda c: B.w4a16_read_probe(Ws[c], nbytes, sink), steps, warm, use_graph, 2)
        lm[str(K)] = {"weight_bytes": nbytes, "plain_read_us": ms_read * 1e3, "plain_read_GBps": nbytes / ms_read / 1e6}
        for M in (1, 10, 60):
            x = torch.randn((M, K), device="cuda", generator=gen).to(torch.float16)
            logits = torch.empty((M, V), dtype=torch.float32, device="cuda")
            ti = torch.empty((M, top_k), dtype=torch.int32, device="cuda")
            tp = torch.empty((M, top_k), dtype=torch.float32, device="cuda")
            lws = torch.empty(B.lm_head_workspace_bytes(M, V, K, top_k), dtype=torch.uint8, device="cuda")
            ms = time_steps(lambda c: B.lm_head_topk(x, Ws[c], M, V, K, top_k, logits, ti, tp, lws), steps, warm, use_graph, 2)
            lm[str(K)][f"M{M}"] = {"us": ms * 1e3, "weight_GBps": nbytes / ms / 1e6,
                                   "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBPS}
            log(f"LM head K={K} M={M}: {ms * 1e3:.1f} us  {nbytes / ms / 1e6:.0f} GB/s (plain read {ms_read * 1e3:.1f} us)")
        del Ws
        torch.cuda.empty_cache()
    return lm


REPEATS = 9   # timed regions per figure; the median is reported
SETTLE_S = 0.06   # least duration of the untimed warm-up of a figure, whatever --warmup says
MAX_GRAPH_STEPS = 512   # a timed region of up to this many steps is one HIP graph


def percentile(sorted_vals, q: float) -> float:
    if len(sorted_vals) == 1:
        return sorted_vals[0]
    pos = q * (len(sorted_vals) - 1)
    lo = int(pos)
    hi = min(lo + 1, len(sorted_vals) - 1)
    return sorted_vals[lo] + (sorted_vals[hi] - sorted_vals[lo]) * (pos - lo)


def time_steps(fn, steps: int, warmup: int, use_graph: bool, copies: int, stats: dict | None = None, repeats: int = REPEATS):
    """fn(copy_index) enqueues one step.  Warm up, then time exactly `steps` steps between two events on the
    launch stream, `repeats` times over, and return the median in ms per step (p10 / p90 / min go to `stats`).
    With graphs, a region of up to MAX_GRAPH_STEPS steps is ONE HIP graph (step i uses copy i % copies), so
    the host never gates the GPU inside a region whatever `steps` is; longer regions replay a graph of
    `copies` steps and finish with single-step graphs to make the count exact."""
    stream = torch.cuda.current_stream()
    if use_graph:
        for c in range(copies):   # one-time kernel attributes are set outside capture
            fn(c)
        torch.cuda.synchronize()
        if steps <= MAX_GRAPH_STEPS:
            region = torch.cuda.CUDAGraph()
            with torch.cuda.graph(region):
                for i in range(steps):
                    fn(i % copies)

            def run_region():
                region.replay()
        else:
            full = torch.cuda.CUDAGraph()
            with torch.cuda.graph(full):
                for c in range(copies):
                    fn(c)
            singles = []
            for c in range(steps % copies):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    fn(c)
                singles.append(g)

            def run_region():
                for _ in range(steps // copies):
                    full.replay()
                for g in singles:
                    g.replay()
        stream = torch.cuda.current_stream()
    else:
        def run_region():
            for i in range(steps):
                fn(i % copies)

    def run_warm():   # warm-up: at least `warmup` steps, in whole regions, so that clocks are up
        for _ in range(max(1, -(-warmup // steps))):
            run_region()

    run_warm()
    torch.cuda.synchronize()
    # settle: for some 40 ms after set-up work (building weights, freeing and allocating buffers) and 15 ms after
    # an idle gap the same graph runs up to 5 % slower; the untimed warm-up therefore lasts at least SETTLE_S
    settle_until = time.perf_counter() + SETTLE_S
    while time.perf_counter() < settle_until:
        run_region()
        torch.cuda.synchronize()
    times = []
    for _ in range(repeats):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        run_warm()          # keeps clocks up right before the timed region
        start.record(stream)
        run_region()
        stop.record(stream)
        torch.cuda.synchronize()
        times.append(start.elapsed_time(stop) / steps)
    times.sort()
    if stats is not None:
        stats.update({"median_ms": percentile(times, 0.5), "p10_ms": percentile(times, 0.1), "p90_ms": percentile(times, 0.9),
                      "min_ms": times[0], "repeats": repeats, "steps_per_region": steps})
    return percentile(times, 0.5)


def gpu_clocks():
    """Current clock levels of GPU 0 as the amdgpu driver reports them in sysfs (the starred line of pp_dpm_sclk /
    pp_dpm_mclk).  Clocks cannot be fixed from user space: recorded, not set.  Plain file reads, no child process
    (this runs after the GPU has been initialised); None where the files are not there."""
    import glob
    import re
    clocks = {}
    for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        for key, name in (("sclk_mhz", "pp_dpm_sclk"), ("mclk_mhz", "pp_dpm_mclk")):
            try:
                lines = open(os.path.join(card, name)).read().splitlines()
            except OSError:
                continue
            for line in lines:
                m = re.match(r"\s*\d+:\s*(\d+)\s*mhz\s*\*", line, flags=re.I)
                if m:
                    clocks[key] = int(m.group(1))
        if clocks:
            break
    return clocks or None


TRAFFIC_PROFILE = os.path.join("profiles", "w4a16_gemm_llama70b_hbm_traffic_m1_m8_m64.txt")
GEMM_SOURCES = ("gemm.hip", "tuned_plans.inc", "tuned_flat.inc", "layout.h")


def measured_traffic():
    """HBM bytes per gate_up launch (fetched + written) at M = 1, 8 and 64 from the committed rocprofv3 PMC summary
    (FETCH_SIZE and WRITE_SIZE runs, calibrated against the runtime's copy kernel on buffers of known size) --
    but only while that summary describes the kernels that run: it records a hash of the GEMM sources, and when
    they have changed since (or the file is not there) there is no measured figure and None is returned."""
    import hashlib
    try:
        vals = dict(ln.strip().split("=", 1) for ln in open(os.path.join(ROOT, TRAFFIC_PROFILE)) if "=" in ln and ln[0].isupper())
        h = hashlib.sha256()
        for name in GEMM_SOURCES:
            h.update(open(os.path.join(ROOT, "paper_2505_22179_amd", "csrc", name), "rb").read())
        if vals["GEMM_SOURCES_SHA256_16"] != h.hexdigest()[:16]:
            return None
        out = {f"M{M}": int(vals[f"FETCH_BYTES_PER_LAUNCH_GATE_UP_M{M}"]) + int(vals[f"WRITE_BYTES_PER_LAUNCH_GATE_UP_M{M}"])
               for M in (1, 8, 64)}
        out["source"] = {"profile": TRAFFIC_PROFILE, "commit": vals.get("SOURCE_COMMIT")}
        return out
    except (OSError, KeyError, ValueError):
        return None


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline():
    """The CPU oracle, as it stands, timed on this machine's host cores on a bounded sample of the benchmark's
    workload: the Llama-3-70B layer's four GEMMs at M = 1 (all threads: the headline figure; one thread:
    each GEMM once), and at M = 64 the Llama-3-8B layer and the 70B o_proj (all threads).  One pass each."""
    from oracle import reference as R
    threads = R.set_threads(0)

    def timed(inp, M, nthreads):
        R.set_threads(nthreads)
        t0 = time.perf_counter()
        R.w4a16_gemm(inp.x[:M], inp.qweight, inp.scales, inp.qzeros, G, want64=False)
        return time.perf_counter() - t0

    per = {"llama3_70b_M1": {}, "llama3_70b_M1_one_thread": {}, "llama3_8b_M64": {}, "llama3_70b_M64": {}}
    total_b, t_all = 0, 0.0
    for gi, (name, K, N) in enumerate(I.LLAMA3_70B):
        inp = I.make_linear(I.seed_for(4, gi), 64 if name == "o_proj" else 1, K, N)
        t = timed(inp, 1, threads)
        t_all += t
        total_b += weight_bytes(K, N)
        per["llama3_70b_M1"][name] = t * 1e6
        per["llama3_70b_M1_one_thread"][name] = timed(inp, 1, 1) * 1e6
        if name == "o_proj":
            per["llama3_70b_M64"][name] = timed(inp, 64, threads) * 1e6
        del inp
    for gi, (name, K, N) in enumerate(I.LLAMA3_8B):
        inp = I.make_linear(I.seed_for(3, gi), 64, K, N)
        per["llama3_8b_M64"][name] = timed(inp, 64, threads) * 1e6
        del inp
    R.set_threads(threads)
    one = sum(per["llama3_70b_M1_one_thread"].values())
    return {
        "value": total_b / t_all / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": f"Llama-3-70B layer: all four GEMMs at M=1, one pass each, {threads} OpenMP threads "
                  f"({t_all * 1e6:.0f} us per layer); one thread: {one:.0f} us per layer ({total_b / one / 1e3:.3f} GB/s); "
                  f"M=64, {threads} threads: 8B layer {sum(per['llama3_8b_M64'].values()):.0f} us, 70B o_proj "
                  f"{per['llama3_70b_M64']['o_proj']:.0f} us",
        "us_per_layer": t_all * 1e6, "us_per_gemm": per, "nproc": os.cpu_count(), "cpu_model": cpu_model(),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--copies", type=int, default=3, help="weight copies rotated through to defeat the last-level cache")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--quick", action="store_true", help="headline only (used under the profiler)")
    ap.add_argument("--quick-m", type=int, default=1,
                    help="with --quick: run at this M instead of 1 (profiler runs at other token counts; not the headline)")
    ap.add_argument("--lm-head-only", action="store_true", help="time only the draft-side LM head (profiler runs)")
    ap.add_argument("--attn-only", type=int, default=0, metavar="M",
                    help="time only tree_verify_attn at this M (64/8 heads, prefix 2048; profiler runs)")
    ap.add_argument("--decoder-layer-only", type=int, default=0, metavar="M",
                    help="time only the whole decoder layer at this M (profiler runs; prints that one figure)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.load()
    use_graph = not args.no_graph
    dev = torch.cuda.get_device_name(0)
    log(f"device: {dev}")

    if args.lm_head_only:
        print(json.dumps({"metric": "draft-side fp16 LM head + top-10, V = 128256", "lm_head_topk_V128256": lm_head_leg(args, use_graph)}))
        return
    if args.attn_only:
        a = I.make_attn(I.seed_for(5, 0), M=args.attn_only, tree="random" if args.attn_only > 6 else "chain")
        q, mask = torch.from_numpy(a.q).cuda(), torch.from_numpy(a.mask).cuda()
        out = torch.empty_like(q)
        k0, v0 = torch.from_numpy(a.k).cuda(), torch.from_numpy(a.v).cuda()
        ks, vs = [k0.clone() for _ in range(64)], [v0.clone() for _ in range(64)]   # 552 MB: never cache-served
        aws = B.new_workspace(B.tree_verify_attn_workspace_bytes(a.M, a.P, a.Hq, a.Hkv, a.D))
        ms = time_steps(lambda c: B.tree_verify_attn(q, ks[c % 64], vs[c % 64], mask, out, a.M, a.P, a.Hq, a.Hkv, a.D, a.scale, aws),
                        args.steps, args.warmup, use_graph, 64)
        print(json.dumps({"metric": "us per tree_verify_attn call (64/8 heads, head dim 128, prefix 2048)", "M": a.M, "value": ms * 1e3, "unit": "us"}))
        return
    big = Layer(I.LLAMA3_70B, args.copies, seed=70)
    log("70B layer packed")
    if args.decoder_layer_only:
        M = args.decoder_layer_only
        layer = DecoderLayer(big, M, 2048, kv_copies=12)
        ms = time_steps(layer.step, args.steps, args.warmup, use_graph, 12)
        print(json.dumps({"metric": "us per Llama-3-70B decoder layer (prefix 2048)", "M": M, "value": ms * 1e3, "unit": "us"}))
        return
    clocks_before = gpu_clocks()
    sweep, sweep_stats = {}, {}
    quick_ms = (args.quick_m,)
    for M in (quick_ms if args.quick else I.M_SWEEP_70B):
        sweep_stats[M] = {}
        ms = time_steps(lambda c, M=M: big.step(M, c), args.steps, args.warmup, use_graph, args.copies, sweep_stats[M])
        sweep[M] = ms
        st = sweep_stats[M]
        log(f"70B M={M}: {ms * 1e3:.1f} us/layer (p10 {st['p10_ms'] * 1e3:.1f}, p90 {st['p90_ms'] * 1e3:.1f})  {big.bytes / ms / 1e6:.0f} GB/s")
    hm = args.quick_m if args.quick else 1   # M of the headline (1 except under --quick --quick-m)
    ms1 = sweep[hm]
    value = big.bytes / ms1 / 1e6   # GB/s

    # dominant kernel: the gate_up GEMM (55 % of the layer's bytes), timed alone, back to back
    per_gemm = {}
    for M in (quick_ms if args.quick else (1, 64)):
        per_gemm[M] = {}
        for gi, (name, K, N) in enumerate(I.LLAMA3_70B):
            if args.quick and gi != 2:
                continue
            nc = big.solo_copies(gi)
            st = {}
            ms = time_steps(lambda c, M=M, gi=gi: big.step(M, c, only=gi), args.steps, args.warmup, use_graph, nc, st)
            per_gemm[M][name] = {"us": ms * 1e3, "GBps": weight_bytes(K, N) / ms / 1e6, "p10_us": st["p10_ms"] * 1e3,
                                 "p90_us": st["p90_ms"] * 1e3, "plan": dict(zip(B.PLAN_FIELDS, B.w4a16_plan_describe(M, N, K)))}
            log(f"70B {name} M={M}: {ms * 1e3:.2f} us  {weight_bytes(K, N) / ms / 1e6:.0f} GB/s")
    gu = per_gemm[hm]["gate_up"]
    # the same buffers through the plain streaming-read probe: the bandwidth this GPU reaches at each size
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    plain = {}
    for gi, (name, K, N) in enumerate(I.LLAMA3_70B):
        if args.quick and gi != 2:
            continue
        nc = big.solo_copies(gi)
        nbytes = big.packed[0][gi].numel()
        ms = time_steps(lambda c, gi=gi, nbytes=nbytes: B.w4a16_read_probe(big.packed[c][gi], nbytes, sink),
                        args.steps, args.warmup, use_graph, nc)
        plain[name] = {"us": ms * 1e3, "GBps": nbytes / ms / 1e6}
        log(f"70B {name} plain read of the packed buffer: {ms * 1e3:.2f} us  {nbytes / ms / 1e6:.0f} GB/s")
    traffic = measured_traffic()
    roofline = {"bound": "hbm", "achieved": gu["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": gu["GBps"] / HBM_PEAK_GBPS, "traffic": traffic and traffic.get(f"M{hm}"),
                "traffic_M64": traffic and traffic["M64"], "traffic_source": traffic and traffic["source"],
                "plain_read_GBps": plain["gate_up"]["GBps"], "frac_of_plain_read": gu["GBps"] / plain["gate_up"]["GBps"],
                "kernel": f"the GEMM kernel of 70B gate_up (K=8192, N=57344, M={hm})",
                "algorithmic_bytes_per_launch": weight_bytes(8192, 57344), "us_per_launch": gu["us"]}

    extra = {}
    if not args.quick:
        # cache-hot, labelled and never the headline: the same weight buffers every step.  One GEMM alone re-reads a
        # buffer that fits the 256 MB last-level cache (all but gate_up: 244 MB); the layer's 445 MB do not fit
        hot = {"note": "cache-hot: every step reads the SAME weight copy (the headline rotates copies); M = 1"}
        for gi, (name, K, N) in enumerate(I.LLAMA3_70B):
            ms = time_steps(lambda c, gi=gi: big.step(1, 0, only=gi), args.steps, args.warmup, use_graph, 1)
            hot[name] = {"us": ms * 1e3, "GBps": weight_bytes(K, N) / ms / 1e6}
        ms = time_steps(lambda c: big.step(1, 0), args.steps, args.warmup, use_graph, 1)
        hot["layer"] = {"us": ms * 1e3, "GBps": big.bytes / ms / 1e6}
        extra["llama3_70b_cache_hot_M1"] = hot
        log("70B cache-hot M=1: " + ", ".join(f"{k} {v['us']:.1f} us" for k, v in hot.items() if k != "note"))
        # tree-verify step: attention at M = 60 over a 2048-token prefix, then the four linears at M = 60
        a = I.make_attn(I.seed_for(5, 0))
        q = torch.from_numpy(a.q).cuda()
        mask = torch.from_numpy(a.mask).cuda()
        out = torch.empty_like(q)
        # K/V of consecutive calls come from 64 rotating copies (552 MB): in the model every layer has its
        # own cache, so a layer's K/V rows are never still in the 256 MB last-level cache when it runs again
        kv_copies = 64
        k0, v0 = torch.from_numpy(a.k).cuda(), torch.from_numpy(a.v).cuda()
        ks = [k0] + [k0.clone() for _ in range(kv_copies - 1)]
        vs = [v0] + [v0.clone() for _ in range(kv_copies - 1)]
        aws = B.new_workspace(B.tree_verify_attn_workspace_bytes(a.M, a.P, a.Hq, a.Hkv, a.D))

        def attn(c):
            B.tree_verify_attn(q, ks[c % kv_copies], vs[c % kv_copies], mask, out, a.M, a.P, a.Hq, a.Hkv, a.D, a.scale, aws)

        def tree_step(c):
            attn(c)
            big.step(60, c)

        ms_attn = time_steps(attn, args.steps, args.warmup, use_graph, kv_copies)
        ms_tree = time_steps(tree_step, args.steps, args.warmup, use_graph, args.copies)
        # greedy acceptance of the verified tree + compaction of the accepted K/V rows (integer step after verify)
        tok, tgt = I.make_verify(I.seed_for(5, 1), a.parent, p_accept=0.8)
        d_parent = torch.from_numpy(a.parent.astype("int32")).cuda()
        d_tok, d_tgt = torch.from_numpy(tok).cuda(), torch.from_numpy(tgt).cuda()
        d_path = torch.empty(a.M, dtype=torch.int32, device="cuda")
        d_res = torch.empty(2, dtype=torch.int32, device="cuda")
        ms_acc = time_steps(lambda c: B.tree_accept(d_parent, d_tok, d_tgt, a.M, d_path, d_res, ks[c % kv_copies],
                                                    vs[c % kv_copies], a.P, a.Hkv, a.D),
                            args.steps, args.warmup, use_graph, kv_copies)
        extra["tree_verify_step_M60"] = {"attn_us": ms_attn * 1e3, "step_us": ms_tree * 1e3,
                                         "accept_and_compact_us": ms_acc * 1e3, "accepted_nodes": int(d_res[0].item())}
        log(f"tree-verify: attn {ms_attn * 1e3:.1f} us, step {ms_tree * 1e3:.1f} us")
        del ks, vs
        # whole decoder layer (norms, rotary + append, attention, fused epilogues) as one graph per step:
        # T_t = the layer at M = 1, T_v(n) = the layer on an n-token draft tree, prefix 2048
        dl = {}
        for M in (1, 7, 8, 24, 32, 40, 48, 60, 64):
            layer = DecoderLayer(big, M, 2048, kv_copies=48)
            ms = time_steps(layer.step, args.steps, args.warmup, use_graph, 48)   # 48 = lcm-friendly with the 3 weight copies
            dl[M] = ms
            log(f"70B decoder layer M={M}: {ms * 1e3:.1f} us")
            del layer
        extra["llama3_70b_decoder_layer_P2048"] = {
            str(M): {"us_per_layer": ms * 1e3, "ratio_vs_M1": ms / dl[1], "ms_per_80_layers": ms * 80} for M, ms in dl.items()}
        del big
        torch.cuda.empty_cache()
        # the paper's own weight format: symmetric quantisation, every zero-point 8.  Same layer, zero-points 8, every
        # linear called with W4A16_SYMMETRIC (the kernels then never read them), beside the general-format figures
        # above; M = 1 plain decoding, 7 and 8 the sequence drafts of length 6 and 7, 64 a full tree
        symw = Layer(I.LLAMA3_70B, args.copies, seed=71, symmetric=True)
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.w4a16_weight_is_symmetric(symw.packed[0][2], I.LLAMA3_70B[2][2], I.LLAMA3_70B[2][1], flag)
        torch.cuda.synchronize()
        assert int(flag[0]) == 1
        sym = {}
        for M in (1, 7, 8, 64):
            st = {}
            ms = time_steps(lambda c, M=M: symw.step(M, c), args.steps, args.warmup, use_graph, args.copies, st)
            sym[str(M)] = {"us_per_layer_symmetric": ms * 1e3, "p10_us": st["p10_ms"] * 1e3, "p90_us": st["p90_ms"] * 1e3}
            if M in sweep:
                sym[str(M)]["us_per_layer_general_format"] = sweep[M] * 1e3
            log(f"70B symmetric weights M={M}: {ms * 1e3:.1f} us/layer")
        extra["llama3_70b_layer_symmetric_weights"] = sym
        del symw
        torch.cuda.empty_cache()
        lm = lm_head_leg(args, use_graph)
        extra["lm_head_topk_V128256"] = lm
        read_rate = plain["gate_up"]["GBps"]
        small = Layer(I.LLAMA3_8B, 6, seed=8)   # 6 x 113 MB: never re-read within 512 MB
        s8 = {}
        for M in I.M_SWEEP_8B:
            ms = time_steps(lambda c, M=M: small.step(M, c), args.steps, args.warmup, use_graph, 6)
            s8[M] = ms
            log(f"8B M={M}: {ms * 1e3:.1f} us/layer  {small.bytes / ms / 1e6:.0f} GB/s")
        dl8 = {}
        for M in (1, 8, 30, 40, 50, 60):
            layer = DecoderLayer(small, M, 2048, kv_copies=48, Hq=32, Hkv=8, D=128)
            ms = time_steps(layer.step, args.steps, args.warmup, use_graph, 48)
            dl8[M] = ms
            log(f"8B decoder layer M={M}: {ms * 1e3:.1f} us")
            del layer
        extra["llama3_8b_decoder_layer_P2048"] = {
            str(M): {"us_per_layer": ms * 1e3, "ratio_vs_M1": ms / dl8[1], "ms_per_32_layers": ms * 32} for M, ms in dl8.items()}
        bytes8 = small.bytes
        del small
        torch.cuda.empty_cache()
        m70 = model_leg("70B", I.LLAMA3_70B, 80, 64, 8, (1, 8, 24, 32, 40, 48, 60), args, use_graph)
        m8 = model_leg("8B", I.LLAMA3_8B, 32, 32, 8, (1, 8, 30, 40, 50, 60), args, use_graph)
        extra["llama3_70b_model_P2048"], extra["llama3_8b_model_P2048"] = m70, m8
        by_m = lambda leg: {int(k): v["ms_per_forward"] for k, v in leg.items() if k.isdigit()}
        extra["eq1_projection_70b"] = eq1_projection(dl, read_rate, lm_head_ms=lm["8192"]["M1"]["us"] * 1e-3,
                                                     draft_lm_head_ms=lm["8192"]["M10"]["us"] * 1e-3, model_ms=by_m(m70))
        extra["eq1_projection_8b"] = eq1_projection(dl8, read_rate, shapes=I.LLAMA3_8B, n_layers=32, tau=PAPER_TAU_8B_W4A16,
                                                    paper_ratio=PAPER_RATIO_8B_W4A16_A100,
                                                    lm_head_ms=lm["4096"]["M1"]["us"] * 1e-3,
                                                    draft_lm_head_ms=lm["4096"]["M10"]["us"] * 1e-3, model_ms=by_m(m8))
        extra["llama3_8b_layer"] = {str(M): {"us_per_layer": ms * 1e3, "weight_GBps": bytes8 / ms / 1e6,
                                            "ratio_vs_M1": ms / s8[1]} for M, ms in s8.items()}
        bytes70 = sum(weight_bytes(K, N) for (_, K, N) in I.LLAMA3_70B)
        extra["llama3_70b_layer"] = {str(M): {"us_per_layer": ms * 1e3, "p10_us": sweep_stats[M]["p10_ms"] * 1e3,
                                             "p90_us": sweep_stats[M]["p90_ms"] * 1e3, "weight_GBps": bytes70 / ms / 1e6,
                                             "frac_of_hbm_peak": bytes70 / ms / 1e6 / HBM_PEAK_GBPS,
                                             "ratio_vs_M1": ms / ms1} for M, ms in sweep.items()}
        extra["llama3_70b_per_gemm"] = {str(M): d for M, d in per_gemm.items()}
        extra["llama3_70b_per_gemm_ratio_M64_over_M1"] = {name: per_gemm[64][name]["us"] / per_gemm[1][name]["us"]
                                                          for name in per_gemm[1]}
        extra["llama3_70b_plain_read"] = dict(plain, layer_us=sum(d["us"] for d in plain.values()),
                                              gemm_layer_over_plain_read=ms1 * 1e3 / sum(d["us"] for d in plain.values()))
        flops64 = sum(2.0 * 64 * K * N for (_, K, N) in I.LLAMA3_70B)
        extra["mfma_utilisation_M64"] = flops64 / (sweep[64] * 1e-3) / MFMA_F16_PEAK_FLOPS
        extra["latency_ratio_M64_over_M1"] = sweep[64] / ms1
        extra["paper_context"] = ("whole-model A100 figures, not comparable: verification/decoding time ratio 1.58 at "
                                  "n=48 (W4A16 70B), 1.80 at n=60 (W4A16 8B); end-to-end 2.78x over autoregressive, "
                                  "1.31x over EAGLE-2")

    result = {
        "metric": f"weight-HBM GB/s of the W4A16 GEMMs of one Llama-3-70B layer at M={hm} (us/layer in ms_per_step)",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "Llama-3-70B decoder-layer linear set (qkv 8192->10240, o_proj 8192->8192, "
                               "gate_up 8192->57344, down 28672->8192), W4A16 G=128, M=" + str(hm) + "; sweep M in {1,4,8,16,32,64}",
                   "weight_copies_rotated": args.copies, "hip_graph": use_graph, "device": dev},
        "frac_of_hbm_peak": value / HBM_PEAK_GBPS,
        "timing": dict(sweep_stats[hm], note=f"median of {REPEATS} timed regions of exactly --steps steps each, HIP events on the launch stream; before them the same "
                                               f"region runs untimed for --warmup steps and at least {SETTLE_S * 1e3:.0f} ms (the GPU is up to 5 % slower for "
                                               f"some 40 ms after set-up work)"),
        "gpu_clocks": {"before": clocks_before, "after": gpu_clocks()},
        "roofline": roofline,
    }
    if not args.no_cpu and not args.quick:
        log("timing the CPU oracle ...")
        result["cpu_baseline"] = cpu_baseline()
    else:
        result["cpu_baseline"] = None
    result.update(extra)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
