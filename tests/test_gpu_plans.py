"""Every launch plan the library picks by itself on the Llama-3 layer shapes, against the CPU oracle.

The benchmark times w4a16_gemm with default knobs on the 8B and 70B layer shapes (paper section 2.2 layer,
token counts of section 2.1 / section 3).  Which kernel instantiation such a call runs is decided by the
tuned tables and the rules behind them; w4a16_plan_describe reports it.  The host test shows that the M
values used below reach every plan that any M in 1..64 reaches; the GPU tests then compare, for every
shape and every such M, sampled output columns (all rows) with the oracle -- plain, and through the fused
epilogue the decoder layer uses for that linear -- at the tolerance of tests/parity.py."""
import os
import re

import numpy as np
import pytest
import torch

from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I
from tests.parity import check_gemm, column_subproblem

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DEV = "cuda"
SENTINEL = 1234.0
SHAPES = [(3, gi) for gi in range(4)] + [(4, gi) for gi in range(4)]   # (config, linear): 8B set, 70B set
CONFIG_MS = (1, 4, 7, 8, 16, 24, 32, 40, 48, 60, 64)   # the sweeps, the sequence draft, the tree-verify step


def shape_of(cfg, gi):
    return (I.LLAMA3_8B if cfg == 3 else I.LLAMA3_70B)[gi]


def plan_ranges(N, K):
    """{plan: [M, ...]} over every supported M, default knobs"""
    plans = {}
    for M in range(1, 65):
        plans.setdefault(B.w4a16_plan_describe(M, N, K), []).append(M)
    return plans


def rows_to_test(N, K):
    ms = set(CONFIG_MS)
    for rows in plan_ranges(N, K).values():
        ms.update((rows[0], rows[-1]))
    return sorted(ms)


def test_tested_rows_reach_every_default_plan():
    for cfg, gi in SHAPES:
        _, K, N = shape_of(cfg, gi)
        every = set(plan_ranges(N, K))
        reached = {B.w4a16_plan_describe(M, N, K) for M in rows_to_test(N, K)}
        assert reached == every, (cfg, gi, every - reached)


def test_every_tuned_row_is_a_llama_shape_and_is_reached():
    """a row of the tuned tables that no default call on the tested shapes selects would be timed by nobody
    and tested by nobody: there must be none"""
    shapes = {(N, K) for cfg, gi in SHAPES for _, K, N in [shape_of(cfg, gi)]}
    csrc = os.path.join(ROOT, "paper_2505_22179_amd", "csrc")
    rows = re.findall(r"^\{([^}]*)\},", open(os.path.join(csrc, "tuned_plans.inc")).read(), flags=re.M)
    assert rows
    for row in rows:
        N, K, bucket, tw, nw, depth, S, fused, ks = (int(v) for v in row.split(","))
        assert (N, K) in shapes, row
        M = 8 if bucket == 0 else 16 * bucket
        fam, mt, ptw, pnw, pdepth, pS, pfused, _ = B.w4a16_plan_describe(M, N, K)
        want_nw = ks if ks else nw
        assert (ptw, pnw, pdepth, pS) == (tw, want_nw, depth, S), (row, B.w4a16_plan_describe(M, N, K))
    flat = re.findall(r"^\{([^}]*)\},", open(os.path.join(csrc, "tuned_flat.inc")).read(), flags=re.M)
    for row in flat:
        N, K, m_max, tw, nw, ng, S, fused = (int(v) for v in row.split(","))
        assert (N, K) in shapes, row
        assert B.w4a16_plan_describe(m_max, N, K)[:6] == (1, 1, tw, nw, ng, S), row


def sample_columns(rng, N, blocks=32):
    b = rng.choice(N // 8, size=blocks, replace=False)
    return np.sort((b[:, None] * 8 + np.arange(8)[None, :]).ravel())


@pytest.mark.gpu
@pytest.mark.parametrize("cfg,gi", SHAPES)
def test_default_plans_full_size_sampled_columns(cfg, gi):
    from oracle import reference as R
    name, K, N = shape_of(cfg, gi)
    inp = I.make_linear(I.seed_for(cfg, gi), 64, K, N, m_max=64)
    rng = np.random.default_rng(100 * cfg + gi)
    gated = name == "gate_up"
    ws = B.new_workspace(B.w4a16_workspace_bytes(64, N, K))   # exactly the advertised size
    packed = B.pack_from_numpy(inp)
    packed_paired = B.pack_from_numpy(inp, gate_up=True) if gated else None
    xd = torch.from_numpy(inp.x).to(DEV)
    res = I.make_hidden(9990 + gi, 64, N, 0) if name in ("o_proj", "down") else None
    cols = sample_columns(rng, N)
    sub = column_subproblem(inp, cols)
    if gated:
        half = N // 2
        gcols = sample_columns(rng, half, 16)
        gsub = column_subproblem(inp, np.concatenate([gcols, half + gcols]))
    for M in rows_to_test(N, K):
        plan = B.w4a16_plan_describe(M, N, K)
        print(f"cfg {cfg} {name} K={K} N={N} M={M} plan {dict(zip(B.PLAN_FIELDS, plan))}", flush=True)
        x = xd[:M].contiguous()
        y = torch.full((M + 2, N), SENTINEL, dtype=torch.float16, device=DEV)
        B.w4a16_gemm(x, packed, y, M, N, K, 128, ws)
        torch.cuda.synchronize()
        out = y.cpu().numpy()
        assert (out[M:] == np.float16(SENTINEL)).all(), "rows >= M were written"
        assert np.isfinite(out[:M].astype(np.float32)).all()
        y32, _, _ = R.w4a16_gemm(inp.x[:M], *sub, 128, want64=False)
        check_gemm(out[:M, cols], y32, f"{name} M={M}")
        if gated:      # the layer runs this linear with the SiLU gate in its store
            yg = torch.full((M + 2, half), SENTINEL, dtype=torch.float16, device=DEV)
            B.w4a16_gemm_fused(x, packed_paired, yg, M, N, K, 128, B.EPI_SILU_MUL, None, ws)
            torch.cuda.synchronize()
            outg = yg.cpu().numpy()
            assert (outg[M:] == np.float16(SENTINEL)).all()
            want, _ = R.w4a16_gemm_silu_mul(inp.x[:M], *gsub)
            check_gemm(outg[:M, gcols], want, f"{name} with gate M={M}")
        if res is not None:   # ... and these with the residual added in place
            yr = torch.full((M + 2, N), SENTINEL, dtype=torch.float16, device=DEV)
            yr[:M] = torch.from_numpy(res[:M]).to(DEV)
            B.w4a16_gemm_fused(x, packed, yr, M, N, K, 128, B.EPI_RESIDUAL, yr, ws)
            torch.cuda.synchronize()
            outr = yr.cpu().numpy()
            assert (outr[M:] == np.float16(SENTINEL)).all()
            want, _ = R.w4a16_gemm_residual(inp.x[:M], *sub, res[:M, cols])
            check_gemm(outr[:M, cols], want, f"{name} + residual M={M}")


@pytest.mark.gpu
@pytest.mark.parametrize("cfg", [3, 4])
def test_default_plans_rope_projection(cfg):
    """the q/k/v projection as the decoder layer runs it (rotary embedding and append in the store): the one
    kernel against w4a16_gemm + rope_append, bit for bit, at every tested M (each of the two is compared with
    the oracle elsewhere)"""
    name, K, N = shape_of(cfg, 0)
    Hq, Hkv, D, P = (32 if cfg == 3 else 64), 8, 128, 2048
    assert N == (Hq + 2 * Hkv) * D
    inp = I.make_linear(I.seed_for(cfg, 0) + 7, 64, K, N, m_max=64)
    ws = B.new_workspace(B.w4a16_workspace_bytes(64, N, K))
    plain, paired = B.pack_from_numpy(inp), B.pack_from_numpy(inp, head_dim=D)
    cos, sin = I.make_rope_tables(P + 64, D)
    cosd, sind = torch.from_numpy(cos).to(DEV), torch.from_numpy(sin).to(DEV)
    gen = np.random.default_rng(cfg)
    k0 = torch.from_numpy(gen.standard_normal((P + 64, Hkv, D), dtype=np.float32).astype(np.float16)).to(DEV)
    v0 = torch.from_numpy(gen.standard_normal((P + 64, Hkv, D), dtype=np.float32).astype(np.float16)).to(DEV)
    xd = torch.from_numpy(inp.x).to(DEV)
    for M in rows_to_test(N, K):
        print(f"cfg {cfg} qkv with rope M={M}", flush=True)
        parent = I.make_tree(9796, M, 6, 4)[0] if M > 6 else np.arange(-1, M - 1)
        pos = torch.from_numpy(I.tree_positions(parent, P)).to(DEV)
        x = xd[:M].contiguous()
        qkv = torch.empty((M, N), dtype=torch.float16, device=DEV)
        q2, k2, v2 = torch.zeros((M, Hq, D), dtype=torch.float16, device=DEV), k0.clone(), v0.clone()
        B.w4a16_gemm(x, plain, qkv, M, N, K, 128, ws)
        B.rope_append(qkv, pos, cosd, sind, P + 64, q2, k2, v2, M, P, Hq, Hkv, D)
        q1, k1, v1 = torch.zeros((M, Hq, D), dtype=torch.float16, device=DEV), k0.clone(), v0.clone()
        B.w4a16_gemm_rope(x, paired, M, K, 128, pos, cosd, sind, P + 64, q1, k1, v1, P, Hq, Hkv, D, ws)
        torch.cuda.synchronize()
        for a, b, what in ((q1, q2, "q"), (k1, k2, "k_cache"), (v1, v2, "v_cache")):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"{what}, M={M}"
