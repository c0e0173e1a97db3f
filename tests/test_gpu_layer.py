"""GPU: the layer glue through the C ABI against the CPU oracle -- fused residual / SiLU-gate
epilogues of the linear (every kernel family and reduction mode), the paired gate/up packing (bit
for bit through the dequantisation export), rms_norm, rope_append, and a whole decoder layer chained
from the library's entry points.

Tolerances.  Fused linears: the linear's own (max |err| <= 1e-2 up to half an fp16 ulp, relative
Frobenius error <= 1e-3) against the oracle's fp64 result.  rms_norm and rope_append evaluate a
handful of fp32 operations per element before one rounding: the result may differ from the
correctly rounded fp64 value only where that value lies within fp32 noise of a rounding boundary,
so every element must be within one fp16 ulp and at most 0.1 % of them may differ at all."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I
from tests.parity import check_gemm, fp16_ulp

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


def set_knobs(tw=0, nw=0, depth=0, split=0, fused=2, ks=0, ng=0, even=0):
    for k, v in (("tiles_per_wave", tw), ("waves_per_wg", nw), ("prefetch_depth", depth), ("split_k", split),
                 ("fused_reduce", fused), ("k_sets", ks), ("flat_groups", ng), ("even_split", even)):
        B.w4a16_set_param(k, v)


def close_to_rounded(got16, want64, what):
    """one rounding of a few fp32 operations: within one ulp everywhere, identical almost everywhere"""
    want16 = want64.astype(np.float16)
    err = np.abs(got16.astype(np.float64) - want64)
    assert (err <= 1.0 * fp16_ulp(want64) + 1e-12).all(), f"{what}: {err.max()}"
    differ = (got16.view(np.uint16) != want16.view(np.uint16)).mean()
    assert differ <= 1e-3, f"{what}: {differ:.2%} of the elements differ from the correctly rounded value"


# ---- paired packing ------------------------------------------------------------------------------

@pytest.mark.parametrize("K,N", [(128, 32), (256, 96), (384, 320), (1024, 4096)])
def test_pack_gate_up_is_pack_of_permuted_columns(K, N):
    inp = I.make_linear(8100 + K + N, 1, K, N)
    packed = B.pack_from_numpy(inp, gate_up=True)
    W = torch.empty((K, N), dtype=torch.float32, device=DEV)
    B.w4a16_dequant(packed, W, N, K)
    torch.cuda.synchronize()
    perm = np.empty(N, dtype=np.int64)
    for n in range(N):          # packed tile 2j = gate tile j, packed tile 2j+1 = up tile j
        tile, c = divmod(n, 16)
        perm[n] = (tile % 2) * (N // 2) + (tile // 2) * 16 + c
    assert sorted(perm.tolist()) == list(range(N))
    Wref = R.dequant(inp.qweight, inp.scales, inp.qzeros, 128)[:, perm]
    assert np.array_equal(W.cpu().numpy().view(np.uint32), np.ascontiguousarray(Wref).view(np.uint32))
    # and the unpack export returns the permuted canonical tensors
    qw = torch.empty((K // 8, N), dtype=torch.int32, device=DEV)
    sc = torch.empty((K // 128, N), dtype=torch.float16, device=DEV)
    qz = torch.empty((K // 128, N // 8), dtype=torch.int32, device=DEV)
    B.w4a16_unpack(packed, qw, sc, qz, N, K)
    torch.cuda.synchronize()
    assert np.array_equal(qw.cpu().numpy(), inp.qweight[:, perm])
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), inp.scales[:, perm].view(np.uint16))


@pytest.mark.parametrize("K,N,D", [(128, 64, 32), (256, 384, 128), (384, 320, 64), (1024, 1280, 128)])
def test_pack_heads_is_pack_of_permuted_columns(K, N, D):
    inp = I.make_linear(8150 + K + N, 1, K, N)
    packed = B.pack_from_numpy(inp, head_dim=D)
    W = torch.empty((K, N), dtype=torch.float32, device=DEV)
    B.w4a16_dequant(packed, W, N, K)
    torch.cuda.synchronize()
    perm = np.empty(N, dtype=np.int64)
    for n in range(N):          # inside a head: packed tile 2j = tile j of the first half, 2j+1 = tile j of the second
        head, within = divmod(n, D)
        tile, c = divmod(within, 16)
        perm[n] = head * D + (tile % 2) * (D // 2) + (tile // 2) * 16 + c
    assert sorted(perm.tolist()) == list(range(N))
    Wref = R.dequant(inp.qweight, inp.scales, inp.qzeros, 128)[:, perm]
    assert np.array_equal(W.cpu().numpy().view(np.uint32), np.ascontiguousarray(Wref).view(np.uint32))


# ---- fused epilogues -----------------------------------------------------------------------------

# knob settings that reach every kernel family and every way the K splits are summed
def kernel_families(M):
    fam = [("default", {}), ("ksplit S=1", dict(tw=4, nw=4, depth=2, split=1, fused=1)),
           ("ksplit last-arriver", dict(tw=2, nw=4, depth=2, split=3, fused=1)),
           ("ksplit two kernels", dict(tw=8, nw=4, depth=1, split=2, fused=0))]
    if M <= 4:
        fam += [("flat S=1", dict(tw=2, nw=8, ng=1, split=1, fused=1)), ("flat last-arriver", dict(tw=4, nw=4, ng=1, split=2, fused=1)),
                ("flat two kernels", dict(tw=8, nw=4, ng=1, split=2, fused=0))]
    if M <= 16:
        fam += [("column split, two groups in flight", dict(tw=8, nw=1, depth=2, split=2))]
    if 16 < M <= 48:
        fam += [("high occupancy three sets last-arriver", dict(tw=2, ks=3, depth=1, split=3, fused=1)),
                ("high occupancy three sets S=1", dict(tw=2, ks=3, depth=1, split=1))]
    if M > 16:
        fam += [("column split S=1", dict(tw=4, nw=1, depth=1, split=1)), ("column split S=3", dict(tw=8, nw=1, depth=1, split=3)),
                ("high occupancy S=1", dict(tw=2, ks=2, depth=2, split=1)), ("high occupancy S=2", dict(tw=4, ks=1, depth=2, split=2)),
                ("high occupancy last-arriver", dict(tw=2, ks=2, depth=2, split=3, fused=1)),
                ("high occupancy even split", dict(tw=2, ks=1, depth=2, even=1))]
    return fam


CASES = [(1, 4096, 512), (3, 2048, 1056), (4, 4096, 288), (16, 1024, 256), (17, 2048, 544), (40, 1536, 1312),
         (64, 2048, 1024), (60, 4096, 160)]


def run_fused(inp, packed, ws, epi, residual=None, in_place=False):
    M, N, K = inp.M, inp.N, inp.K
    width = N // 2 if epi == B.EPI_SILU_MUL else N
    x = torch.from_numpy(inp.x).to(DEV)
    y = torch.full((M + 2, width), SENTINEL, dtype=torch.float16, device=DEV)
    res = None
    if residual is not None:
        if in_place:
            y[:M] = torch.from_numpy(residual).to(DEV)
            res = y
        else:
            res = torch.from_numpy(residual).to(DEV)
    B.w4a16_gemm_fused(x, packed, y, M, N, K, 128, epi, res, ws)
    torch.cuda.synchronize()
    out = y.cpu().numpy()
    assert (out[M:] == np.float16(SENTINEL)).all(), "rows >= M were written"
    return out[:M]


def each_family(M, K):
    for name, knobs in kernel_families(M):
        knobs = dict(knobs)
        if knobs.get("ng"):
            groups = K // 128
            per = knobs["split"] * knobs["nw"]
            if groups % per or groups // per not in (4, 7, 8):
                continue
            knobs["ng"] = groups // per
        set_knobs(**knobs)
        yield name


@pytest.mark.parametrize("M,K,N", CASES)
def test_residual_epilogue(M, K, N, big_ws):
    print(f"fused residual M={M} K={K} N={N}", flush=True)
    inp = I.make_linear(8200 + M + K + N, M, K, N)
    r = I.make_hidden(8300 + M, M, N)
    packed = B.pack_from_numpy(inp)
    y64, _ = R.w4a16_gemm_residual(inp.x, inp.qweight, inp.scales, inp.qzeros, r)
    ran = []
    for name in each_family(M, K):
        check_gemm(run_fused(inp, packed, big_ws, B.EPI_RESIDUAL, r), y64, f"residual, {name}")
        check_gemm(run_fused(inp, packed, big_ws, B.EPI_RESIDUAL, r, in_place=True), y64, f"residual in place, {name}")
        ran.append(name)
    assert len(ran) >= 4, ran


@pytest.mark.parametrize("M,K,N", CASES)
def test_silu_mul_epilogue(M, K, N, big_ws):
    print(f"fused silu*mul M={M} K={K} N={N}", flush=True)
    inp = I.make_linear(8400 + M + K + N, M, K, N)
    packed = B.pack_from_numpy(inp, gate_up=True)
    y64, _ = R.w4a16_gemm_silu_mul(inp.x, inp.qweight, inp.scales, inp.qzeros)
    ran = []
    for name in each_family(M, K):
        check_gemm(run_fused(inp, packed, big_ws, B.EPI_SILU_MUL), y64, f"silu*mul, {name}")
        ran.append(name)
    assert len(ran) >= 4, ran


def test_flat_family_is_reached(big_ws):
    """the all-loads-up-front kernels need K = split * waves * groups * 128: shapes chosen for them"""
    for M, K, N, knobs in ((2, 4096, 288, dict(tw=2, nw=8, ng=4, split=1, fused=1)),
                           (4, 7168, 544, dict(tw=4, nw=4, ng=7, split=2, fused=1)),
                           (1, 4096, 1056, dict(tw=8, nw=4, ng=4, split=2, fused=0))):
        inp = I.make_linear(8500 + M + K, M, K, N)
        r = I.make_hidden(8600 + M, M, N)
        y64r, _ = R.w4a16_gemm_residual(inp.x, inp.qweight, inp.scales, inp.qzeros, r)
        y64g, _ = R.w4a16_gemm_silu_mul(inp.x, inp.qweight, inp.scales, inp.qzeros)
        set_knobs(**knobs)
        check_gemm(run_fused(inp, B.pack_from_numpy(inp), big_ws, B.EPI_RESIDUAL, r), y64r, f"flat residual {knobs}")
        check_gemm(run_fused(inp, B.pack_from_numpy(inp, gate_up=True), big_ws, B.EPI_SILU_MUL), y64g, f"flat gate {knobs}")


def test_epilogue_none_is_the_plain_gemm_bit_for_bit(big_ws):
    inp = I.make_linear(8700, 24, 2048, 512)
    packed = B.pack_from_numpy(inp)
    x = torch.from_numpy(inp.x).to(DEV)
    a = torch.empty((24, 512), dtype=torch.float16, device=DEV)
    b = torch.empty_like(a)
    B.w4a16_gemm(x, packed, a, 24, 512, 2048, 128, big_ws)
    B.w4a16_gemm_fused(x, packed, b, 24, 512, 2048, 128, B.EPI_NONE, None, big_ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_gate_saturation():
    """large negative gates give -0 or tiny values, large positive ones pass the up value through"""
    K, N = 128, 32
    inp = I.make_linear(8800, 2, K, N, x_kind="small_int", scale_kind="pow2")
    x = np.zeros((2, K), dtype=np.float16)
    x[0, :8] = 60.0      # eight rows of codes: |gate| up to a few tens, far into both tails of the sigmoid
    x[1, :8] = -60.0
    inp.x = x
    y64, _ = R.w4a16_gemm_silu_mul(x, inp.qweight, inp.scales, inp.qzeros)
    packed = B.pack_from_numpy(inp, gate_up=True)
    got = run_fused(inp, packed, B.new_workspace(1 << 20), B.EPI_SILU_MUL)
    assert np.isfinite(got.astype(np.float32)).all()
    check_gemm(got, y64, "saturated gates")


# ---- rms_norm ------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,K", [(1, 8), (1, 8192), (7, 4096), (64, 8192), (5, 16384), (3, 1000), (2, 2056)])
def test_rms_norm(M, K):
    print(f"rms_norm M={M} K={K}", flush=True)
    x = I.make_hidden(8900 + M + K, M, K)
    g = I.make_gamma(8950 + K, K)
    y64, _ = R.rms_norm(x, g, 1e-5)
    xd = torch.from_numpy(x).to(DEV)
    gd = torch.from_numpy(g).to(DEV)
    y = torch.full((M + 1, K), SENTINEL, dtype=torch.float16, device=DEV)
    B.rms_norm(xd, gd, y, M, K, 1e-5)
    torch.cuda.synchronize()
    out = y.cpu().numpy()
    assert (out[M:] == np.float16(SENTINEL)).all()
    close_to_rounded(out[:M], y64, f"rms_norm M={M} K={K}")
    B.rms_norm(xd, gd, xd, M, K, 1e-5)   # in place
    torch.cuda.synchronize()
    assert np.array_equal(xd.cpu().numpy().view(np.uint16), out[:M].view(np.uint16))


def test_rms_norm_zero_row_and_eps():
    K = 512
    x = np.zeros((2, K), dtype=np.float16)
    x[1, 3] = 1.0
    g = np.ones(K, dtype=np.float16)
    y = torch.empty((2, K), dtype=torch.float16, device=DEV)
    B.rms_norm(torch.from_numpy(x).to(DEV), torch.from_numpy(g).to(DEV), y, 2, K, 1e-6)
    torch.cuda.synchronize()
    out = y.cpu().numpy()
    assert (out[0] == 0).all()
    y64, _ = R.rms_norm(x, g, 1e-6)
    close_to_rounded(out, y64, "zero row")


# ---- rope_append ---------------------------------------------------------------------------------

@pytest.mark.parametrize("M,P,Hq,Hkv,D", [(60, 100, 64, 8, 128), (1, 0, 32, 8, 128), (5, 7, 4, 2, 16), (64, 2048, 8, 1, 64)])
def test_rope_append(M, P, Hq, Hkv, D):
    print(f"rope_append M={M} P={P} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    rng = np.random.default_rng(9000 + M + P)
    n_pos = P + 16
    qkv = rng.standard_normal((M, (Hq + 2 * Hkv) * D), dtype=np.float32).astype(np.float16)
    parent, _, _ = I.make_tree(9100 + M, M, 6, 4) if M > 1 else (np.array([-1]), None, None)
    pos = I.tree_positions(parent, P)
    cos, sin = I.make_rope_tables(n_pos, D)
    kc = rng.standard_normal((P + M + 3, Hkv, D), dtype=np.float32).astype(np.float16)
    vc = rng.standard_normal((P + M + 3, Hkv, D), dtype=np.float32).astype(np.float16)
    q64, _, k_want, v_want = R.rope_append(qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    q = torch.full((M + 1, Hq, D), SENTINEL, dtype=torch.float16, device=DEV)
    kd, vd = dev(kc), dev(vc)
    B.rope_append(dev(qkv), dev(pos), dev(cos), dev(sin), n_pos, q, kd, vd, M, P, Hq, Hkv, D)
    torch.cuda.synchronize()
    qo, ko, vo = q.cpu().numpy(), kd.cpu().numpy(), vd.cpu().numpy()
    assert (qo[M:] == np.float16(SENTINEL)).all()
    close_to_rounded(qo[:M], q64, "rotated q")
    # keys: compare against the fp64 rotation before its rounding
    a = qkv.astype(np.float64).reshape(M, Hq + 2 * Hkv, D)[:, Hq:Hq + Hkv]
    h = D // 2
    c, s = cos.astype(np.float64)[pos][:, None, :], sin.astype(np.float64)[pos][:, None, :]
    k64 = np.concatenate([a[..., :h] * c - a[..., h:] * s, a[..., h:] * c + a[..., :h] * s], axis=-1)
    assert np.array_equal(k64.astype(np.float16), k_want[P:P + M])      # the oracle's own keys, recomputed
    close_to_rounded(ko[P:P + M], k64, "rotated k")
    assert np.array_equal(vo.view(np.uint16), v_want.view(np.uint16)), "values must be copied bit for bit"
    assert np.array_equal(ko[:P].view(np.uint16), kc[:P].view(np.uint16)) and np.array_equal(ko[P + M:].view(np.uint16), kc[P + M:].view(np.uint16))


@pytest.mark.parametrize("D,table_offset", [(10, 0), (16, 1), (128, 3)])
def test_rope_append_general_form(D, table_offset):
    """Head dimensions that are not multiples of 8, and tables that are only 4-byte aligned, take the
    element-wise kernel: same results to the same bar."""
    M, P, Hq, Hkv = 5, 6, 3, 1
    print(f"rope_append general form D={D} table offset {table_offset} floats", flush=True)
    rng = np.random.default_rng(9300 + D)
    n_pos = P + 8
    qkv = rng.standard_normal((M, (Hq + 2 * Hkv) * D), dtype=np.float32).astype(np.float16)
    pos = np.array([6, 7, 7, 8, 13], dtype=np.int32)
    cos, sin = I.make_rope_tables(n_pos, D)
    kc = rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16)
    vc = rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16)
    q64, _, k_want, v_want = R.rope_append(qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)

    def shifted(t):   # the same values at an address table_offset floats past a 16-byte boundary
        buf = torch.empty(t.size + table_offset, dtype=torch.float32, device=DEV)
        buf[table_offset:] = dev(t).reshape(-1)
        return buf[table_offset:]

    q = torch.full((M, Hq, D), SENTINEL, dtype=torch.float16, device=DEV)
    kd, vd = dev(kc), dev(vc)
    B.rope_append(dev(qkv), dev(pos), shifted(cos), shifted(sin), n_pos, q, kd, vd, M, P, Hq, Hkv, D)
    torch.cuda.synchronize()
    close_to_rounded(q.cpu().numpy(), q64, "rotated q")
    a = qkv.astype(np.float64).reshape(M, Hq + 2 * Hkv, D)[:, Hq:Hq + Hkv]
    h = D // 2
    c, s = cos.astype(np.float64)[pos][:, None, :], sin.astype(np.float64)[pos][:, None, :]
    k64 = np.concatenate([a[..., :h] * c - a[..., h:] * s, a[..., h:] * c + a[..., :h] * s], axis=-1)
    close_to_rounded(kd.cpu().numpy()[P:], k64, "rotated k")
    assert np.array_equal(vd.cpu().numpy().view(np.uint16), v_want.view(np.uint16))
    assert np.array_equal(kd.cpu().numpy()[:P].view(np.uint16), kc[:P].view(np.uint16))


def test_rope_position_outside_the_tables_is_skipped():
    M, P, Hq, Hkv, D = 3, 2, 2, 1, 16
    rng = np.random.default_rng(9200)
    qkv = rng.standard_normal((M, (Hq + 2 * Hkv) * D), dtype=np.float32).astype(np.float16)
    cos, sin = I.make_rope_tables(8, D)
    pos = np.array([1, 8, -1], dtype=np.int32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    q = torch.full((M, Hq, D), SENTINEL, dtype=torch.float16, device=DEV)
    kd = torch.full((P + M, Hkv, D), SENTINEL, dtype=torch.float16, device=DEV)
    vd = torch.full((P + M, Hkv, D), SENTINEL, dtype=torch.float16, device=DEV)
    B.rope_append(dev(qkv), dev(pos), dev(cos), dev(sin), 8, q, kd, vd, M, P, Hq, Hkv, D)
    torch.cuda.synchronize()
    qo, ko, vo = q.cpu().numpy(), kd.cpu().numpy(), vd.cpu().numpy()
    assert (qo[1:] == np.float16(SENTINEL)).all() and (ko[P + 1:] == np.float16(SENTINEL)).all()
    assert not (qo[0] == np.float16(SENTINEL)).any() and not (ko[P] == np.float16(SENTINEL)).any()
    assert np.array_equal(vo[P:], qkv.reshape(M, Hq + 2 * Hkv, D)[:, Hq + Hkv:])


# ---- the q/k/v projection with the rotary embedding and the append in its store ----------------------

ROPE_CASES = [(1, 1024, 4, 2, 64, 0), (5, 512, 2, 1, 128, 9), (17, 2048, 3, 1, 32, 40), (40, 1024, 8, 2, 64, 3), (64, 2048, 4, 4, 128, 100),
              (3, 4096, 6, 2, 128, 7)]


def gemm_rope_both_ways(inp, M, K, Hq, Hkv, D, P, pos, ws, plain, heads):
    """(q, k_cache, v_cache) from w4a16_gemm + rope_append and from w4a16_gemm_rope, same knobs"""
    N = (Hq + 2 * Hkv) * D
    rng = np.random.default_rng(9777)
    cos, sin = I.make_rope_tables(P + 16, D)
    kc = rng.standard_normal((P + M + 2, Hkv, D), dtype=np.float32).astype(np.float16)
    vc = rng.standard_normal((P + M + 2, Hkv, D), dtype=np.float32).astype(np.float16)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    x, posd, cosd, sind = dev(inp.x), dev(pos), dev(cos), dev(sin)
    out = []
    for fused in (False, True):
        q = torch.full((M + 1, Hq, D), SENTINEL, dtype=torch.float16, device=DEV)
        kd, vd = dev(kc), dev(vc)
        if fused:
            B.w4a16_gemm_rope(x, heads, M, K, 128, posd, cosd, sind, P + 16, q, kd, vd, P, Hq, Hkv, D, ws)
        else:
            qkv = torch.empty((M, N), dtype=torch.float16, device=DEV)
            B.w4a16_gemm(x, plain, qkv, M, N, K, 128, ws)
            B.rope_append(qkv, posd, cosd, sind, P + 16, q, kd, vd, M, P, Hq, Hkv, D)
        torch.cuda.synchronize()
        out.append((q.cpu().numpy(), kd.cpu().numpy(), vd.cpu().numpy()))
    return out, (cos, sin, kc, vc)


@pytest.mark.parametrize("M,K,Hq,Hkv,D,P", ROPE_CASES)
def test_gemm_rope_is_gemm_then_rope_append(M, K, Hq, Hkv, D, P, big_ws):
    """every kernel family and reduction mode: q, the cache rows and everything around them bit for bit"""
    print(f"projection + rotary + append in one kernel M={M} K={K} Hq={Hq} Hkv={Hkv} D={D} P={P}", flush=True)
    N = (Hq + 2 * Hkv) * D
    inp = I.make_linear(9700 + M + K + N, M, K, N)
    plain, heads = B.pack_from_numpy(inp), B.pack_from_numpy(inp, head_dim=D)
    pos = (P + np.arange(M) % 7).astype(np.int32)
    if M >= 3:
        pos[1], pos[2] = -1, P + 16   # outside the tables: that row's q and k stay untouched, its v is appended
    ran = []
    for name in each_family(M, K):
        (two, one), _ = gemm_rope_both_ways(inp, M, K, Hq, Hkv, D, P, pos, big_ws, plain, heads)
        for a, b, what in zip(two, one, ("q", "k_cache", "v_cache")):
            assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), f"{what}, {name}"
        ran.append(name)
    assert len(ran) >= 4, ran
    if M >= 3:
        assert (one[0][1:3] == np.float16(SENTINEL)).all()


def test_gemm_rope_against_the_oracle(big_ws):
    M, K, Hq, Hkv, D, P = 12, 1024, 4, 2, 64, 30
    N = (Hq + 2 * Hkv) * D
    inp = I.make_linear(9790, M, K, N)
    parent, _, _ = I.make_tree(9791, M, 4, 3)
    pos = I.tree_positions(parent, P)
    (_, (q, kd, vd)), (cos, sin, kc, vc) = gemm_rope_both_ways(inp, M, K, Hq, Hkv, D, P, pos, big_ws, B.pack_from_numpy(inp),
                                                            B.pack_from_numpy(inp, head_dim=D))
    _, y64, y16 = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros)
    q64, _, k_want, v_want = R.rope_append(y16, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    # one more fp16 rounding than the linear alone (the projection's own), then rope_append's bar
    assert (np.abs(q[:M].astype(np.float64) - q64) <= 1.5 * fp16_ulp(q64) + 1e-2).all()
    rel = np.linalg.norm(q[:M].astype(np.float64) - q64) / np.linalg.norm(q64)
    assert rel <= 1e-3, rel
    assert (np.abs(kd[P:P + M].astype(np.float64) - k_want[P:P + M].astype(np.float64)) <= 1e-2 + 1.5 * fp16_ulp(k_want[P:P + M].astype(np.float64))).all()
    check_gemm(vd[P:P + M].reshape(M, Hkv * D), y64.reshape(M, Hq + 2 * Hkv, D)[:, Hq + Hkv:].reshape(M, Hkv * D), "appended values")
    assert np.array_equal(kd[:P].view(np.uint16), kc[:P].view(np.uint16)) and np.array_equal(kd[P + M:].view(np.uint16), kc[P + M:].view(np.uint16))


@pytest.mark.parametrize("M", [1, 7, 60])
def test_gemm_rope_model_shapes(M):
    """Llama-3-70B and 8B q/k/v projections, committed launch plans: the one kernel against the two"""
    for K, Hq, Hkv, D in ((8192, 64, 8, 128), (4096, 32, 8, 128)):
        N = (Hq + 2 * Hkv) * D
        print(f"   K={K} N={N} M={M}", flush=True)
        inp = I.make_linear(9795 + M + K, M, K, N)
        ws = B.new_workspace(B.w4a16_workspace_bytes(M, N, K))
        parent = I.make_tree(9796, M, 6, 4)[0] if M > 6 else np.arange(-1, M - 1)
        pos = I.tree_positions(parent, 2048)
        (two, one), _ = gemm_rope_both_ways(inp, M, K, Hq, Hkv, D, 2048, pos, ws, B.pack_from_numpy(inp), B.pack_from_numpy(inp, head_dim=D))
        for a, b, what in zip(two, one, ("q", "k_cache", "v_cache")):
            assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), f"{what}, K={K}"


# ---- a whole decoder layer from the library's entry points -----------------------------------------

def test_decoder_layer_chain(big_ws):
    """norm -> qkv -> rope/append -> tree attention -> o_proj + residual -> norm -> gate/up with the
    SiLU gate -> down + residual, every step fed with the previous step's GPU output and compared
    with the oracle's step on the same input (strict), and the end of the chain with the oracle's own
    chain (loose: roundings of intermediate fp16 tensors may fall differently and propagate)."""
    M, P, Hq, Hkv, D, H, Iff = 24, 150, 8, 2, 128, 1024, 2816
    rng = np.random.default_rng(9300)
    lin = {name: I.make_linear(9310 + i, M, K, N) for i, (name, K, N) in
           enumerate((("qkv", H, (Hq + 2 * Hkv) * D), ("o", Hq * D, H), ("gate_up", H, 2 * Iff), ("down", Iff, H)))}
    packed = {n: B.pack_from_numpy(v, gate_up=(n == "gate_up")) for n, v in lin.items()}
    canon = {n: (v.qweight, v.scales, v.qzeros) for n, v in lin.items()}
    h0 = I.make_hidden(9320, M, H)
    g1, g2 = I.make_gamma(9321, H), I.make_gamma(9322, H)
    parent, _, mask = I.make_tree(9323, M, 5, 3)
    pos = I.tree_positions(parent, P)
    cos, sin = I.make_rope_tables(P + 16, D)
    kc = (rng.standard_normal((P + M, Hkv, D), dtype=np.float32)).astype(np.float16)
    vc = (rng.standard_normal((P + M, Hkv, D), dtype=np.float32)).astype(np.float16)
    scale = 1.0 / np.sqrt(D)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device=DEV)
    host = lambda t: t.cpu().numpy()

    def gpu_layer():
        h = dev(h0)
        n1, qkv, q, att, n2, act = f16(M, H), f16(M, (Hq + 2 * Hkv) * D), f16(M, Hq, D), f16(M, Hq, D), f16(M, H), f16(M, Iff)
        kd, vd = dev(kc), dev(vc)
        aws = B.new_workspace(B.tree_verify_attn_workspace_bytes(M, P, Hq, Hkv, D))
        B.rms_norm(h, dev(g1), n1, M, H, 1e-5)
        B.w4a16_gemm(n1, packed["qkv"], qkv, M, (Hq + 2 * Hkv) * D, H, 128, big_ws)
        B.rope_append(qkv, dev(pos), dev(cos), dev(sin), P + 16, q, kd, vd, M, P, Hq, Hkv, D)
        B.tree_verify_attn(q, kd, vd, dev(mask), att, M, P, Hq, Hkv, D, scale, aws)
        h1 = h.clone()
        B.w4a16_gemm_fused(att.view(M, Hq * D), packed["o"], h1, M, H, Hq * D, 128, B.EPI_RESIDUAL, h1, big_ws)
        B.rms_norm(h1, dev(g2), n2, M, H, 1e-5)
        B.w4a16_gemm_fused(n2, packed["gate_up"], act, M, 2 * Iff, H, 128, B.EPI_SILU_MUL, None, big_ws)
        h2 = h1.clone()
        B.w4a16_gemm_fused(act, packed["down"], h2, M, H, Iff, 128, B.EPI_RESIDUAL, h2, big_ws)
        torch.cuda.synchronize()
        return tuple(host(t) for t in (n1, qkv, q, kd, vd, att, h1, n2, act, h2))

    n1, qkv, q, kd, vd, att, h1, n2, act, h2 = gpu_layer()

    # the same layer as ONE call: every kernel is the same, so the hidden state and the cache must agree bit for bit
    hd, kd1, vd1 = dev(h0), dev(kc), dev(vc)
    g1d, g2d = dev(g1), dev(g2)
    weights = B.layer_weights(packed["qkv"], packed["o"], packed["gate_up"], packed["down"], g1d, g2d, H, Hq, Hkv, D, Iff, 1e-5)
    bufs = [f16(M, H), f16(M, (Hq + 2 * Hkv) * D), f16(M, Hq, D), f16(M, Hq, D), f16(M, Iff)]
    aws = B.new_workspace(B.tree_verify_attn_workspace_bytes(M, P, Hq, Hkv, D))
    scratch = B.layer_scratch(*bufs, big_ws, aws)
    posd, cosd, sind, maskd = dev(pos), dev(cos), dev(sin), dev(mask)
    B.w4a16_decoder_layer(weights, hd, M, P, posd, cosd, sind, P + 16, maskd, kd1, vd1, scratch)
    torch.cuda.synchronize()
    assert np.array_equal(host(hd).view(np.uint16), h2.view(np.uint16)), "one-call layer differs from the chained calls"
    assert np.array_equal(host(kd1).view(np.uint16), kd.view(np.uint16)) and np.array_equal(host(vd1).view(np.uint16), vd.view(np.uint16))
    # and with the rotary embedding and the append inside the q/k/v projection (no qkv scratch): the same bits again
    hd, kd1, vd1 = dev(h0), dev(kc), dev(vc)
    weights = B.layer_weights(B.pack_from_numpy(lin["qkv"], head_dim=D), packed["o"], packed["gate_up"], packed["down"], g1d, g2d,
                              H, Hq, Hkv, D, Iff, 1e-5, qkv_heads_packed=True)
    scratch = B.layer_scratch(bufs[0], None, *bufs[2:], big_ws, aws)
    B.w4a16_decoder_layer(weights, hd, M, P, posd, cosd, sind, P + 16, maskd, kd1, vd1, scratch)
    torch.cuda.synchronize()
    assert np.array_equal(host(hd).view(np.uint16), h2.view(np.uint16)), "layer with the fused projection differs"
    assert np.array_equal(host(kd1).view(np.uint16), kd.view(np.uint16)) and np.array_equal(host(vd1).view(np.uint16), vd.view(np.uint16))
    # step by step, each oracle step on the GPU's input to that step
    close_to_rounded(n1, R.rms_norm(h0, g1, 1e-5)[0], "norm 1")
    check_gemm(qkv, R.w4a16_gemm(n1, *canon["qkv"])[1], "qkv")
    q64, _, k_want, v_want = R.rope_append(qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    close_to_rounded(q, q64, "rope q")
    assert np.array_equal(vd.view(np.uint16), v_want.view(np.uint16))
    assert (np.abs(kd.astype(np.float64) - k_want.astype(np.float64)) <= fp16_ulp(k_want.astype(np.float64))).all()
    a64, _ = R.tree_verify_attn(q, kd, vd, mask, scale)
    err = np.abs(att.astype(np.float64) - a64)
    assert err.max() <= 1e-2 and np.linalg.norm(err) / np.linalg.norm(a64) <= 1e-3
    check_gemm(h1, R.w4a16_gemm_residual(att.reshape(M, Hq * D), *canon["o"], h0)[0], "o_proj + residual")
    close_to_rounded(n2, R.rms_norm(h1, g2, 1e-5)[0], "norm 2")
    check_gemm(act, R.w4a16_gemm_silu_mul(n2, *canon["gate_up"])[0], "gate_up with gate")
    check_gemm(h2, R.w4a16_gemm_residual(act, *canon["down"], h1)[0], "down + residual")
    # the oracle's own chain
    o_n1 = R.rms_norm(h0, g1, 1e-5)[1]
    o_qkv = R.w4a16_gemm(o_n1, *canon["qkv"])[2]
    _, o_q, o_k, o_v = R.rope_append(o_qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    o_att = R.tree_verify_attn(o_q, o_k, o_v, mask, scale)[1]
    o_h1 = R.w4a16_gemm_residual(o_att.reshape(M, Hq * D), *canon["o"], h0)[1]
    o_n2 = R.rms_norm(o_h1, g2, 1e-5)[1]
    o_act = R.w4a16_gemm_silu_mul(o_n2, *canon["gate_up"])[1]
    o_h2 = R.w4a16_gemm_residual(o_act, *canon["down"], o_h1)[0]
    rel = np.linalg.norm(h2.astype(np.float64) - o_h2) / np.linalg.norm(o_h2)
    print(f"decoder layer chain: relative Frobenius error of the layer output {rel:.3g}", flush=True)
    assert rel <= 3e-3


# ---- full-size shapes in the launch configuration the benchmark times --------------------------------

@pytest.mark.parametrize("M", [1, 8, 60])
def test_fused_epilogues_full_size_sampled_columns(M):
    """Llama-3-70B gate_up with the gate and down with the residual, default launch plans; the oracle
    recomputes sampled output columns (all rows) from the same canonical tensors"""
    from tests.parity import column_subproblem
    print(f"fused epilogues full size M={M}", flush=True)
    rng = np.random.default_rng(9900 + M)
    # gate_up: output column n needs weight columns n (gate) and I + n (up)
    _, K, N = I.LLAMA3_70B[2]
    half = N // 2
    inp = I.make_linear(I.seed_for(4, 2) + 50, M, K, N)
    ws = B.new_workspace(B.w4a16_workspace_bytes(M, N, K))
    got = run_fused(inp, B.pack_from_numpy(inp, gate_up=True), ws, B.EPI_SILU_MUL)
    blocks = rng.choice(half // 8, size=16, replace=False)
    cols = np.sort((blocks[:, None] * 8 + np.arange(8)[None, :]).ravel())
    qw, sc, qz = column_subproblem(inp, np.concatenate([cols, half + cols]))
    want, _ = R.w4a16_gemm_silu_mul(inp.x, qw, sc, qz)
    check_gemm(got[:, cols], want, f"gate_up with gate, M={M}")
    del inp, got
    # down + residual, in place
    _, K, N = I.LLAMA3_70B[3]
    inp = I.make_linear(I.seed_for(4, 3) + 50, M, K, N)
    res = I.make_hidden(9950 + M, M, N, 0)
    ws = B.new_workspace(B.w4a16_workspace_bytes(M, N, K))
    got = run_fused(inp, B.pack_from_numpy(inp), ws, B.EPI_RESIDUAL, res, in_place=True)
    blocks = rng.choice(N // 8, size=32, replace=False)
    cols = np.sort((blocks[:, None] * 8 + np.arange(8)[None, :]).ravel())
    qw, sc, qz = column_subproblem(inp, cols)
    want, _ = R.w4a16_gemm_residual(inp.x, qw, sc, qz, res[:, cols])
    check_gemm(got[:, cols], want, f"down + residual, M={M}")
