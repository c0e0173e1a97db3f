"""GPU: the symmetric-weight path (every zero-point 8 -- the scheme paper section 2.2 describes) against the CPU
oracle, which needs no change: such a weight is the special case z = 8 of its formula.  With W4A16_SYMMETRIC the
kernels never read the zero-points; the tests check parity at the tolerance of tests/parity.py, bit-exactness on
exact-arithmetic inputs, agreement with the unflagged call, and -- by flagging a weight whose stored zero-points
are NOT 8 -- that the flagged kernels really ignore them."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I
from tests.parity import check_gemm, column_subproblem

pytestmark = pytest.mark.gpu
DEV = "cuda"
KNOBS = ("tiles_per_wave", "waves_per_wg", "prefetch_depth", "split_k", "fused_reduce", "k_sets", "flat_groups", "even_split")


def set_knobs(**kw):
    for k in KNOBS:
        B.w4a16_set_param(k, kw.get(k, 2 if k == "fused_reduce" else 0))


@pytest.fixture(autouse=True)
def _reset_knobs():
    yield
    set_knobs()


@pytest.fixture(scope="module")
def ws():
    return B.new_workspace(64 << 20)


def run(inp, packed, ws, epi=B.EPI_NONE, residual=None, M=None):
    M = inp.M if M is None else M
    width = inp.N // 2 if (epi & 0xff) == B.EPI_SILU_MUL else inp.N
    x = torch.from_numpy(inp.x[:M]).to(DEV).contiguous()
    y = torch.full((M + 2, width), 99.0, dtype=torch.float16, device=DEV)
    res = None if residual is None else torch.from_numpy(residual[:M]).to(DEV)
    B.w4a16_gemm_fused(x, packed, y, M, inp.N, inp.K, 128, epi, res, ws)
    torch.cuda.synchronize()
    out = y.cpu().numpy()
    assert (out[M:] == np.float16(99.0)).all(), "rows >= M were written"
    return out[:M]


# kernel families that have a symmetric instantiation: K-split workgroups (any M) and the column-split kernel with
# interleaved K sets (M > 16); {} is the library's own plan
def families(M):
    fam = [{}, dict(tiles_per_wave=8, waves_per_wg=4, prefetch_depth=1, split_k=1), dict(tiles_per_wave=2, waves_per_wg=4, prefetch_depth=2, split_k=3, fused_reduce=1),
           dict(tiles_per_wave=4, waves_per_wg=4, prefetch_depth=2, split_k=2, fused_reduce=0)]
    if M <= 16:
        fam += [dict(tiles_per_wave=4, waves_per_wg=8, prefetch_depth=1, split_k=1), dict(tiles_per_wave=2, waves_per_wg=8, prefetch_depth=2, split_k=2, fused_reduce=1)]
    if M > 16:
        fam += [dict(tiles_per_wave=2, k_sets=2, prefetch_depth=1, split_k=1), dict(tiles_per_wave=4, k_sets=1, prefetch_depth=2, split_k=2),
                dict(tiles_per_wave=2, k_sets=2, prefetch_depth=2, split_k=3, fused_reduce=1)]
    if 16 < M <= 48:
        fam += [dict(tiles_per_wave=2, k_sets=3, prefetch_depth=1, split_k=3, fused_reduce=1)]
    return fam


CASES = [(1, 4096, 544), (5, 2048, 256), (8, 1536, 992), (16, 1024, 256), (17, 2048, 288), (40, 1536, 1312), (64, 2048, 1024), (60, 4096, 160)]   # N % 32 == 0: the gate needs it


@pytest.mark.parametrize("M,K,N", CASES)
def test_symmetric_parity_and_zero_points_not_read(M, K, N, ws):
    print(f"symmetric M={M} K={K} N={N}", flush=True)
    sym = I.make_linear(9100 + M + K + N, M, K, N, zero_kind="eight")
    asym = I.make_linear(9100 + M + K + N, M, K, N)          # same x, codes and scales; zero-points uniform in 0..15
    assert np.array_equal(sym.qweight, asym.qweight) and not np.array_equal(sym.qzeros, asym.qzeros)
    res = I.make_hidden(9200 + M, M, N, 0)
    y32 = R.w4a16_gemm(sym.x, sym.qweight, sym.scales, sym.qzeros, 128, want64=False)[0]
    yres = R.w4a16_gemm_residual(sym.x, sym.qweight, sym.scales, sym.qzeros, res)[0]
    ygate = R.w4a16_gemm_silu_mul(sym.x, sym.qweight, sym.scales, sym.qzeros)[0]
    p_sym, p_asym = B.pack_from_numpy(sym), B.pack_from_numpy(asym)
    g_sym, g_asym = B.pack_from_numpy(sym, gate_up=True), B.pack_from_numpy(asym, gate_up=True)
    ran = 0
    for knobs in families(M):
        set_knobs(**knobs)
        plan = B.w4a16_plan_describe(M, N, K)
        assert plan[7] == 1 or not knobs, (knobs, plan)     # every forced family here has the instantiation
        flagged = run(sym, p_sym, ws, B.EPI_NONE | B.SYMMETRIC)
        check_gemm(flagged, y32, f"symmetric, {knobs}")
        check_gemm(run(sym, p_sym, ws, B.EPI_RESIDUAL | B.SYMMETRIC, res), yres, f"symmetric + residual, {knobs}")
        check_gemm(run(sym, g_sym, ws, B.EPI_SILU_MUL | B.SYMMETRIC), ygate, f"symmetric + gate, {knobs}")
        plain = run(sym, p_sym, ws, B.EPI_NONE)
        if M > 16:
            assert np.array_equal(flagged.view(np.uint16), plain.view(np.uint16)), f"flag changes bits at M > 16, {knobs}"
        else:
            check_gemm(plain, y32, f"symmetric weight, no flag, {knobs}")
        if plan[7] == 1:   # the flagged kernel must not look at the stored zero-points at all
            assert np.array_equal(run(asym, p_asym, ws, B.EPI_NONE | B.SYMMETRIC).view(np.uint16), flagged.view(np.uint16)), knobs
            assert np.array_equal(run(asym, g_asym, ws, B.EPI_SILU_MUL | B.SYMMETRIC).view(np.uint16),
                                  run(sym, g_sym, ws, B.EPI_SILU_MUL | B.SYMMETRIC).view(np.uint16)), knobs
            ran += 1
    assert ran >= 4


@pytest.mark.parametrize("M", [1, 7, 16, 31, 64])
def test_symmetric_exact_inputs_bit_exact(M, ws):
    K, N = 3072, 392
    inp = I.make_linear(9300 + M, M, K, N, x_kind="small_int", scale_kind="pow2", zero_kind="eight")
    packed = B.pack_from_numpy(inp)
    y16 = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)[2]
    for knobs in families(M):
        set_knobs(**knobs)
        assert np.array_equal(run(inp, packed, ws, B.EPI_NONE | B.SYMMETRIC).view(np.uint16), y16.view(np.uint16)), (M, knobs)


def test_weight_is_symmetric():
    flag = torch.full((3,), 7, dtype=torch.int32, device=DEV)
    for i, (kind, N) in enumerate((("eight", 992), ("uniform", 1000), ("eight", 136))):
        inp = I.make_linear(9400 + i, 1, 512, N, zero_kind=kind)
        B.w4a16_weight_is_symmetric(B.pack_from_numpy(inp, gate_up=(i == 0)), N, 512, flag[i:])
    torch.cuda.synchronize()
    assert flag.cpu().tolist() == [1, 0, 1]      # padding columns (N = 136, 992) do not count
    inp = I.make_linear(9410, 1, 512, 136, zero_kind="eight")
    inp.zeros[3, 135] = 9                        # one zero-point of the last real column
    inp.qzeros = I.pack_cols(inp.zeros)
    B.w4a16_weight_is_symmetric(B.pack_from_numpy(inp), 136, 512, flag)
    torch.cuda.synchronize()
    assert int(flag[0]) == 0


@pytest.mark.parametrize("gi", [0, 1, 2, 3])
def test_symmetric_full_size_default_plans(gi):
    """Llama-3-70B layer shapes, default plans, M of plain decoding, the sequence draft (d = 6, 7) and a full tree"""
    name, K, N = I.LLAMA3_70B[gi]
    inp = I.make_linear(I.seed_for(4, gi) + 30, 64, K, N, m_max=64, zero_kind="eight")
    wsz = B.new_workspace(B.w4a16_workspace_bytes(64, N, K))
    packed = B.pack_from_numpy(inp)
    rng = np.random.default_rng(9500 + gi)
    blocks = rng.choice(N // 8, size=32, replace=False)
    cols = np.sort((blocks[:, None] * 8 + np.arange(8)[None, :]).ravel())
    sub = column_subproblem(inp, cols)
    for M in (1, 7, 8, 24, 64):
        print(f"symmetric full size {name} M={M} plan {B.w4a16_plan_describe(M, N, K)}", flush=True)
        y = run(inp, packed, wsz, B.EPI_NONE | B.SYMMETRIC, M=M)
        y32 = R.w4a16_gemm(inp.x[:M], *sub, 128, want64=False)[0]
        check_gemm(y[:, cols], y32, f"{name} M={M}")
