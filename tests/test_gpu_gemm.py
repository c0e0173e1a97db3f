"""GPU: w4a16_gemm through the C ABI against the CPU oracle (paper section 2.2 layer at the token
counts of section 2.1).  Tolerance: max |err| <= 1e-2 and relative Frobenius error <= 1e-3 against
the oracle's fp32 result (see tests/parity.py for the fp16-ulp caveat); bit-exact where the
arithmetic is exact in any order."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I
from tests.parity import check_gemm, column_subproblem

pytestmark = pytest.mark.gpu
DEV = "cuda"
SENTINEL = 1234.0


@pytest.fixture(scope="module")
def big_ws():
    return B.new_workspace(256 << 20)


@pytest.fixture(autouse=True)
def _reset_knobs():
    yield
    for k in ("split_k", "tiles_per_wave", "waves_per_wg", "prefetch_depth", "k_sets", "flat_groups", "even_split"):
        B.w4a16_set_param(k, 0)
    B.w4a16_set_param("fused_reduce", 2)


def run_gemm(inp, packed, ws, M=None, guard_rows=2):
    """Returns fp16 y[M, N]; also checks that rows >= M of the y buffer are left untouched."""
    M = inp.M if M is None else M
    x = torch.from_numpy(inp.x[:M]).to(DEV).contiguous()
    y = torch.full((M + guard_rows, inp.N), SENTINEL, dtype=torch.float16, device=DEV)
    B.w4a16_gemm(x, packed, y, M, inp.N, inp.K, inp.G, ws)
    torch.cuda.synchronize()
    out = y.cpu().numpy()
    assert (out[M:] == np.float16(SENTINEL)).all(), "rows >= M were written"
    return out[:M]


# (tiles_per_wave, waves_per_wg, prefetch_depth, split_k, fused_reduce); 0 = the library's heuristic.
# Every row is a kernel variant compiled for all M.
VARIANTS = [(0, 0, 0, 0, 2), (8, 4, 1, 1, 1), (8, 4, 2, 3, 1), (4, 4, 2, 2, 0), (4, 4, 1, 1, 1), (2, 4, 4, 0, 0),
            (2, 4, 2, 3, 1), (2, 4, 4, 1, 1), (2, 4, 1, 5, 0)]
# column-split workgroups (waves_per_wg = 1): compiled for M > 16 (and tw 8 at any M)
VARIANTS_NS = [(4, 1, 1, 1, 2), (4, 1, 1, 3, 2), (8, 1, 1, 1, 2), (8, 1, 1, 2, 2), (8, 1, 2, 2, 2), (8, 1, 2, 1, 2), (4, 1, 2, 2, 2)]
NS_ANY_M = [v for v in VARIANTS_NS if v[0] == 8]   # the 8-tile column-split kernels are compiled for one row tile too
VARIANTS_M16 = [(2, 8, 1, 1, 1), (2, 8, 2, 2, 1), (2, 8, 4, 3, 0), (4, 8, 2, 2, 0), (4, 4, 4, 1, 1), (8, 8, 2, 1, 1), (8, 8, 1, 3, 1)]


def compiled(macro, arity):
    """the (..) tuples of one of the kernel-variant lists in csrc/gemm.hip"""
    import os, re
    src = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2505_22179_amd", "csrc", "gemm.hip")).read()
    body = re.search(r"#define " + macro + r"\(\w\)(.*?)\n\n", src, flags=re.S).group(1)
    return {tuple(int(v) for v in m) for m in re.findall(r"\b[XYZF]\(" + ", ".join([r"(\d+)"] * arity) + r"\)", body)}


NS_COMPILED = compiled("W4_NS_VARIANTS", 3)   # (row tiles, tiles per wavefront, depth)
CS_COMPILED = compiled("W4_CS_VARIANTS", 4)   # (row tiles, tiles per wavefront, K sets, depth)


def ns_variants(M):
    mt = (M + 15) // 16
    return [v for v in VARIANTS_NS if (mt, v[0], v[2]) in NS_COMPILED]


def set_variant(tw, nw, depth, split, fused):
    B.w4a16_set_param("tiles_per_wave", tw)
    B.w4a16_set_param("waves_per_wg", nw)
    B.w4a16_set_param("prefetch_depth", depth)
    B.w4a16_set_param("split_k", split)
    B.w4a16_set_param("fused_reduce", fused)


SMALL = [
    # M, K, N  -- several column blocks, several groups per wavefront, ragged M and N tails
    (1, 128, 8), (1, 4096, 4096), (3, 1024, 136), (4, 2048, 512), (8, 1536, 1000),
    (16, 1024, 256), (17, 2048, 264), (32, 4096, 384), (33, 1024, 128), (48, 2048, 520),
    (60, 4096, 256), (64, 2048, 1024), (64, 128, 128), (7, 14336, 256),
]


@pytest.mark.parametrize("M,K,N", SMALL)
def test_parity_small(M, K, N, big_ws):
    print(f"gemm parity M={M} K={K} N={N}", flush=True)
    inp = I.make_linear(5000 + M * 7 + K + N, M, K, N)
    packed = B.pack_from_numpy(inp)
    y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
    for variant in VARIANTS + ns_variants(M):
        set_variant(*variant)
        y = run_gemm(inp, packed, big_ws)
        check_gemm(y, y32, f"M={M} K={K} N={N} (tw, nw, depth, split, fused)={variant}")


@pytest.mark.parametrize("M,K,N", [(1, 4096, 520), (7, 2176, 256), (16, 8192, 136)])
def test_parity_wide_workgroups(M, K, N, big_ws):
    """variants that exist for M <= 16 only (8 and 16 wavefronts per workgroup on wider tiles)"""
    print(f"gemm parity (wide workgroups) M={M} K={K} N={N}", flush=True)
    inp = I.make_linear(5500 + M + K + N, M, K, N)
    packed = B.pack_from_numpy(inp)
    y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
    ex = I.make_linear(5600 + M, M, K, N, x_kind="small_int", scale_kind="pow2")
    ex_packed = B.pack_from_numpy(ex)
    _, _, ex16 = R.w4a16_gemm(ex.x, ex.qweight, ex.scales, ex.qzeros, 128, want64=False)
    for variant in VARIANTS_M16:
        set_variant(*variant)
        check_gemm(run_gemm(inp, packed, big_ws), y32, f"M={M} K={K} N={N} variant={variant}")
        assert np.array_equal(run_gemm(ex, ex_packed, big_ws).view(np.uint16), ex16.view(np.uint16)), variant


# high-occupancy column-split workgroups, M > 16 only: (tiles_per_wave, k_sets, prefetch_depth, split_k)
VARIANTS_CS = [(2, 1, 2, 1), (2, 2, 2, 1), (2, 2, 2, 3), (4, 1, 2, 1), (4, 1, 2, 2), (4, 2, 2, 1),
               (2, 3, 1, 3), (2, 3, 1, 1), (2, 3, 2, 1), (4, 3, 1, 2), (2, 2, 1, 3), (4, 2, 1, 2), (4, 1, 1, 1), (8, 1, 1, 1)]


def set_cs_variant(tw, ks, depth, split):
    B.w4a16_set_param("tiles_per_wave", tw)
    B.w4a16_set_param("k_sets", ks)
    B.w4a16_set_param("prefetch_depth", depth)
    B.w4a16_set_param("split_k", split)


@pytest.mark.parametrize("M,K,N", [s for s in SMALL if s[0] > 16] + [(40, 640, 136), (64, 8192, 2056)])
def test_parity_high_occupancy(M, K, N, big_ws):
    """the variant whose workgroup interleaves several K sets per column quarter; covers K ranges
    shorter than the prefetch ring, group counts that do not divide by the number of sets, idle
    column quarters in the last workgroup, and K split across workgroups on top"""
    print(f"gemm parity (high occupancy) M={M} K={K} N={N}", flush=True)
    inp = I.make_linear(5800 + M + K + N, M, K, N)
    packed = B.pack_from_numpy(inp)
    y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
    ex = I.make_linear(5900 + M, M, K, N, x_kind="small_int", scale_kind="pow2")
    ex_packed = B.pack_from_numpy(ex)
    _, _, ex16 = R.w4a16_gemm(ex.x, ex.qweight, ex.scales, ex.qzeros, 128, want64=False)
    ran = 0
    for variant in VARIANTS_CS:
        if ((M + 15) // 16, variant[0], variant[1], variant[2]) not in CS_COMPILED:
            continue   # not every combination is compiled for every number of row tiles
        ran += 1
        set_cs_variant(*variant)
        for fused in ((0, 1) if variant[3] > 1 else (0,)):   # K splits summed by a second kernel, or by the last workgroup to arrive
            B.w4a16_set_param("fused_reduce", fused)
            check_gemm(run_gemm(inp, packed, big_ws), y32, f"M={M} K={K} N={N} (tw, ks, depth, split)={variant} fused={fused}")
            assert np.array_equal(run_gemm(ex, ex_packed, big_ws).view(np.uint16), ex16.view(np.uint16)), (variant, fused)
        if variant[1] == 3:
            continue   # the even split below is an ablation of the one- and two-set kernels only
        # (unit, group) pairs dealt evenly to one workgroup per compute unit: runs cross unit boundaries
        B.w4a16_set_param("even_split", 1)
        check_gemm(run_gemm(inp, packed, big_ws), y32, f"M={M} K={K} N={N} (tw, ks, depth)={variant[:3]} even split")
        assert np.array_equal(run_gemm(ex, ex_packed, big_ws).view(np.uint16), ex16.view(np.uint16)), (variant, "even split")
        B.w4a16_set_param("even_split", 0)
    assert ran >= 6, ran


# all-loads-up-front kernel, M <= 4 only: (tiles_per_wave, waves_per_wg, flat_groups, split_k, fused_reduce);
# it needs K / 128 == split_k * waves_per_wg * flat_groups exactly
VARIANTS_FLAT = [(2, 8, 8, 1, 1), (2, 16, 4, 1, 1), (2, 4, 7, 2, 1), (2, 8, 7, 2, 0), (4, 8, 4, 1, 1), (4, 4, 8, 3, 1),
                 (4, 8, 7, 1, 1), (8, 4, 4, 2, 0), (8, 8, 4, 1, 1)]


@pytest.mark.parametrize("M", [1, 2, 3, 4])
@pytest.mark.parametrize("N", [136, 1000])
def test_parity_flat(M, N, big_ws):
    """every wavefront requests all of its weights before computing; x rows staged in LDS"""
    print(f"gemm parity (flat) M={M} N={N}", flush=True)
    for tw, nw, ng, split, fused in VARIANTS_FLAT:
        K = split * nw * ng * 128
        inp = I.make_linear(6100 + M + N + K, M, K, N)
        packed = B.pack_from_numpy(inp)
        y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
        ex = I.make_linear(6200 + M + K, M, K, N, x_kind="small_int", scale_kind="pow2")
        ex_packed = B.pack_from_numpy(ex)
        _, _, ex16 = R.w4a16_gemm(ex.x, ex.qweight, ex.scales, ex.qzeros, 128, want64=False)
        set_variant(tw, nw, 0, split, fused)
        B.w4a16_set_param("flat_groups", ng)
        check_gemm(run_gemm(inp, packed, big_ws), y32, f"M={M} K={K} N={N} flat (tw, nw, ng, split, fused)={(tw, nw, ng, split, fused)}")
        assert np.array_equal(run_gemm(ex, ex_packed, big_ws).view(np.uint16), ex16.view(np.uint16)), (tw, nw, ng, split, fused)
    # a K that the forced variant cannot tile, or M > 4, is reported, not computed wrongly
    B.w4a16_set_param("flat_groups", 8)
    set_variant(2, 8, 0, 1, 1)
    inp = I.make_linear(6300, 5, 8192, 128)
    with pytest.raises(B.W4A16Error) as e:
        run_gemm(inp, B.pack_from_numpy(inp), big_ws)
    assert e.value.code == -4


@pytest.mark.parametrize("M,K,N", [(64, 8192, 7168), (33, 4096, 14336 + 128), (48, 1024, 57344)])
def test_parity_even_split_many_units(M, K, N, big_ws):
    """more workgroup units than compute units, or not a multiple of them: every run crosses a unit
    boundary somewhere, units have one, two or three contributors"""
    print(f"gemm parity (even split) M={M} K={K} N={N}", flush=True)
    inp = I.make_linear(6400 + M + K + N, M, K, N)
    packed = B.pack_from_numpy(inp)
    y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
    for tw, ks, depth in ((4, 2, 1), (2, 2, 1), (4, 1, 2)):
        if tw == 4 and ks == 2 and M > 32 and depth == 2:
            continue
        set_cs_variant(tw, ks, depth, 0)
        B.w4a16_set_param("even_split", 1)
        first = run_gemm(inp, packed, big_ws)
        check_gemm(first, y32, f"M={M} K={K} N={N} even split (tw, ks, depth)={(tw, ks, depth)}")
        assert np.array_equal(run_gemm(inp, packed, big_ws).view(np.uint16), first.view(np.uint16)), "not deterministic"


def test_uncompiled_variant_is_reported():
    inp = I.make_linear(5700, 40, 256, 128)
    packed = B.pack_from_numpy(inp)
    x = torch.from_numpy(inp.x).to(DEV)
    y = torch.empty((40, 128), dtype=torch.float16, device=DEV)
    set_variant(8, 16, 4, 0, 2)
    with pytest.raises(B.W4A16Error) as e:
        B.w4a16_gemm(x, packed, y, 40, 128, 256, 128, B.new_workspace(1 << 20))
    assert e.value.code == -4


@pytest.mark.parametrize("M", [1, 5, 16, 31, 48, 64])
def test_exact_inputs_bit_exact(M, big_ws):
    # x in {-2..2}, scales 2^-7: every partial sum is exact in fp32 whatever the order, so every
    # kernel variant must reproduce the oracle's fp16 output bit for bit
    K, N = 3072, 392
    print(f"gemm exact M={M}", flush=True)
    inp = I.make_linear(6000 + M, M, K, N, x_kind="small_int", scale_kind="pow2")
    packed = B.pack_from_numpy(inp)
    _, _, y16 = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
    for variant in VARIANTS + ns_variants(M):
        set_variant(*variant)
        y = run_gemm(inp, packed, big_ws)
        assert np.array_equal(y.view(np.uint16), y16.view(np.uint16)), (M, variant)


def test_run_to_run_determinism_and_ticket_reuse(big_ws):
    inp = I.make_linear(7001, 24, 8192, 2048)
    packed = B.pack_from_numpy(inp)
    first = run_gemm(inp, packed, big_ws)
    for _ in range(6):   # the tickets must come back to zero after every call
        again = run_gemm(inp, packed, big_ws)
        assert np.array_equal(again.view(np.uint16), first.view(np.uint16))
    other = I.make_linear(7002, 9, 4096, 1024)
    y32, _, _ = R.w4a16_gemm(other.x, other.qweight, other.scales, other.qzeros, 128, want64=False)
    check_gemm(run_gemm(other, B.pack_from_numpy(other), big_ws), y32, "after reuse")


def test_rows_do_not_influence_each_other(big_ws):
    inp = I.make_linear(7003, 40, 2048, 512)
    packed = B.pack_from_numpy(inp)
    base = run_gemm(inp, packed, big_ws)
    inp.x[7] = np.float16(3.0)
    inp.x[39] *= np.float16(-1)
    pert = run_gemm(inp, packed, big_ws)
    keep = [m for m in range(40) if m not in (7, 39)]
    assert np.array_equal(pert[keep].view(np.uint16), base[keep].view(np.uint16))
    assert not np.array_equal(pert[7], base[7])


def test_m_prefix_consistency(big_ws):
    # the first rows of a 64-row call match a smaller call within tolerance of the same oracle rows
    inp = I.make_linear(7004, 64, 4096, 512)
    packed = B.pack_from_numpy(inp)
    y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, 128, want64=False)
    for M in (1, 2, 15, 16, 47, 63, 64):
        check_gemm(run_gemm(inp, packed, big_ws, M=M), y32[:M], f"prefix M={M}")


def test_workspace_too_small_is_rejected():
    inp = I.make_linear(7005, 1, 4096, 4096)
    packed = B.pack_from_numpy(inp)
    x = torch.from_numpy(inp.x).to(DEV)
    y = torch.empty((1, 4096), dtype=torch.float16, device=DEV)
    tiny = torch.empty(16384, dtype=torch.uint8, device=DEV)
    B.w4a16_set_param("split_k", 2)
    with pytest.raises(B.W4A16Error) as e:
        B.w4a16_gemm(x, packed, y, 1, 4096, 4096, 128, tiny)
    assert e.value.code == -5


@pytest.mark.parametrize("M", [1, 4, 16, 32])
def test_tiny_activations(M, big_ws):
    """x ~ N(0, 1e-4^2), many of them subnormal in fp16: every operand of the matrix instruction is exact, so the
    relative error is that of rounding y, as for activations of ordinary size (a kernel that scaled x down in
    fp16 on the way -- an earlier form of the few-row kernels divided half of it by 16 -- shows 2e-3 here)"""
    K, N = 4096, 1024
    inp = I.make_linear(4321 + M, M, K, N)
    inp.x = (np.random.default_rng(99).standard_normal((M, K)) * 1e-4).astype(np.float16)
    packed = B.pack_from_numpy(inp)
    got = run_gemm(inp, packed, big_ws).astype(np.float64)
    y32, _, _ = R.matmul(inp.x, R.dequant(inp.qweight, inp.scales, inp.qzeros, 128), want64=False)
    err = np.abs(got - y32).max()
    rel = np.linalg.norm(got - y32) / np.linalg.norm(y32)
    print(f"tiny x, M={M}: max abs err {err:.3g}, rel fro {rel:.3g}", flush=True)
    assert err <= 1e-6 and rel <= 3e-4


@pytest.mark.parametrize("M", [1, 16, 32, 64])
def test_large_activations(M, big_ws):
    """x ~ N(0, 500^2), outputs in the thousands: the relative criterion applies (half an fp16 ulp of such a y is
    already above 1e-2).  Element by element: half an ulp of the rounding plus the fp32 accumulation noise, which
    scales with the row (in the one-row-tile kernels the cancelled code bias costs about ten bits of it)"""
    K, N = 4096, 1024
    inp = I.make_linear(4400 + M, M, K, N)
    inp.x = (np.random.default_rng(7).standard_normal((M, K)) * 500.0).astype(np.float16)
    packed = B.pack_from_numpy(inp)
    got = run_gemm(inp, packed, big_ws).astype(np.float64)
    y32, _, _ = R.matmul(inp.x, R.dequant(inp.qweight, inp.scales, inp.qzeros, 128), want64=False)
    assert np.isfinite(got).all()
    rel = np.linalg.norm(got - y32) / np.linalg.norm(y32)
    ulp = np.spacing(np.abs(y32).astype(np.float16)).astype(np.float64)
    rms = np.sqrt((y32.astype(np.float64) ** 2).mean(axis=1, keepdims=True))
    excess = (np.abs(got - y32) - 0.5 * ulp) / rms
    print(f"large x, M={M}: rel fro {rel:.3g}, error beyond half an ulp {excess.max():.3g} of the row rms", flush=True)
    assert rel <= 3e-4 and excess.max() <= 5e-4


@pytest.mark.parametrize("lo,hi", [(1e-7, 5e-5), (10.0, 200.0)])
@pytest.mark.parametrize("M", [1, 16, 32, 64])
def test_scale_extremes(M, lo, hi, big_ws):
    """scales that are all subnormal in fp16, and scales in the hundreds: exact in the dequantisation export, and
    the product as accurate as with the benchmark's scales (they enter as fp32 factors of fp32 group sums)"""
    K, N = 4096, 1024
    inp = I.make_linear(4500 + M, M, K, N)
    inp.scales = np.random.default_rng(5).uniform(lo, hi, inp.scales.shape).astype(np.float16)
    if hi > 1:
        inp.x = (inp.x.astype(np.float32) * 0.01).astype(np.float16)   # keeps y inside the fp16 range
    packed = B.pack_from_numpy(inp)
    W = torch.empty((K, N), dtype=torch.float32, device=DEV)
    B.w4a16_dequant(packed, W, N, K)
    got = run_gemm(inp, packed, big_ws).astype(np.float64)
    Wref = R.dequant(inp.qweight, inp.scales, inp.qzeros, 128)
    assert np.array_equal(W.cpu().numpy().view(np.uint32), Wref.view(np.uint32))
    y32, _, _ = R.matmul(inp.x, Wref, want64=False)
    assert np.isfinite(got).all()
    rel = np.linalg.norm(got - y32) / np.linalg.norm(y32)
    assert rel <= 3e-4, rel


def test_vocabulary_sized_linear(big_ws):
    """N = 128256 (a quantised LM head on the Llama-3 vocabulary; not a multiple of 128): 8016 column tiles, the
    widest grid any shape here launches.  The oracle recomputes 1016 sampled columns, the first and the last included."""
    K, N = 4096, 128256
    inp = I.make_linear(31337, 64, K, N)
    packed = B.pack_from_numpy(inp)
    rng = np.random.default_rng(1)
    cols = np.unique(np.concatenate([rng.choice(N, 1000, replace=False), np.arange(8), np.arange(N - 16, N)]))
    cols = cols[len(cols) % 8:]
    Wsub = R.dequant(*column_subproblem(inp, cols), 128)
    for M in (1, 16, 40, 64):
        got = run_gemm(inp, packed, big_ws, M=M)[:, cols]
        y32, _, _ = R.matmul(inp.x[:M], Wsub, want64=False)
        check_gemm(got, y32, f"N={N} M={M}")
