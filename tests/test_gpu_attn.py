"""GPU: tree_verify_attn through the C ABI against the fp64 oracle (paper section 2.1).
Tolerance: max |err| <= 1e-2 and relative Frobenius error <= 1e-3."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.fixture(autouse=True)
def _reset_knobs():
    yield
    B.w4a16_set_param("attn_splits", 0)
    B.w4a16_set_param("attn_pack", 0)
    B.w4a16_set_param("attn_row_tiles", 0)
    B.w4a16_set_param("attn_fused_merge", 0)


def run_attn(a: I.AttnInputs, ws=None):
    q, k, v = (torch.from_numpy(t).to(DEV) for t in (a.q, a.k, a.v))
    mask = torch.from_numpy(a.mask).to(DEV)
    out = torch.full((a.M + 1, a.Hq, a.D), 77.0, dtype=torch.float16, device=DEV)
    if ws is None:
        ws = B.new_workspace(B.tree_verify_attn_workspace_bytes(a.M, a.P, a.Hq, a.Hkv, a.D))
    B.tree_verify_attn(q, k, v, mask, out, a.M, a.P, a.Hq, a.Hkv, a.D, a.scale, ws)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert (o[a.M:] == np.float16(77.0)).all()
    return o[:a.M]


def check(out16, ref64, what):
    err = np.abs(out16.astype(np.float64) - ref64)
    rel = np.linalg.norm(out16.astype(np.float64) - ref64) / np.linalg.norm(ref64)
    assert err.max() <= 1e-2, f"{what}: max abs {err.max():.3g}"
    assert rel <= 1e-3, f"{what}: rel fro {rel:.3g}"
    return float(err.max()), float(rel)


CASES = [
    # M, P, Hq, Hkv, tree
    (60, 2048, 64, 8, "random"),     # the tree-verify configuration
    (60, 2048, 64, 8, "chain"),
    (7, 2048, 64, 8, "chain"),       # sequence-draft verification
    (1, 2048, 64, 8, "identity"),    # plain decode
    (64, 100, 8, 8, "random"),
    (17, 0, 16, 4, "random"),        # no prefix: only the tree itself
    (1, 0, 8, 1, "identity"),        # a single key
    (33, 31, 8, 2, "identity"),
    (48, 5, 4, 1, "random"),
    (8, 1000, 64, 8, "random"),      # 8 rows x 8 heads of a KV group fill one 64-row tile exactly
    (5, 70, 24, 3, "random"),        # 40 of 64 tile rows in use, three KV heads
    (16, 333, 16, 4, "chain"),       # 4 heads x 16 rows
    (3, 2, 12, 2, "chain"),          # fewer keys than one step
    (12, 300, 32, 4, "random"),      # groups of 8 heads, two heads per 24-row tile
    (7, 129, 12, 2, "chain"),        # groups of 6 heads: three per 21-row tile (42 rows would need the tall tile)
    (8, 10001, 16, 2, "random"),     # long prefixes: many rounds per key range, a ragged last step
    (3, 65536, 8, 8, "chain"),
]


@pytest.mark.parametrize("M,P,Hq,Hkv,tree", CASES)
def test_attn_parity(M, P, Hq, Hkv, tree):
    print(f"attn parity M={M} P={P} Hq={Hq} Hkv={Hkv} {tree}", flush=True)
    depth = 6 if M > 6 else max(M - 1, 0)
    a = I.make_attn(8000 + M + P + Hq, M, P, Hq, Hkv, 128, tree=tree, depth=depth)
    ref64, _ = R.tree_verify_attn(a.q, a.k, a.v, a.mask, a.scale)
    for pack in ((0, 1, 2) if Hq > Hkv else (0,)):   # heads of a KV group sharing a tile (by size, never, whole group)
        B.w4a16_set_param("attn_pack", pack)
        for row_tiles in (0, 2, 4):   # by tile height; 32 rows per wavefront (one or two row groups); all 64
            B.w4a16_set_param("attn_row_tiles", row_tiles)
            for splits in (0, 1, 3, 6, 16):
                B.w4a16_set_param("attn_splits", splits)
                B.w4a16_set_param("attn_fused_merge", 2)   # the last workgroup of a tile merges its key ranges
                got = run_attn(a)
                stats = check(got, ref64, f"M={M} P={P} {tree} splits={splits} pack={pack} row_tiles={row_tiles}")
                B.w4a16_set_param("attn_fused_merge", 1)   # a second kernel does: the same arithmetic in the same order
                two = run_attn(a)
                assert np.array_equal(two.view(np.uint16), got.view(np.uint16)), (splits, pack, row_tiles)
                B.w4a16_set_param("attn_fused_merge", 0)   # chosen by size
                assert np.array_equal(run_attn(a).view(np.uint16), got.view(np.uint16)), (splits, pack, row_tiles)
    print("   ", stats, flush=True)


def test_attn_determinism_and_workspace_reuse():
    a = I.make_attn(8100, 60, 2048, 64, 8, 128)
    ws = B.new_workspace(B.tree_verify_attn_workspace_bytes(a.M, a.P, a.Hq, a.Hkv, a.D))
    first = run_attn(a, ws)
    for _ in range(4):
        assert np.array_equal(run_attn(a, ws).view(np.uint16), first.view(np.uint16))
    # the fused merge leaves its tickets at zero: the same workspace serves calls of other shapes in between
    b = I.make_attn(8101, 8, 500, 64, 8, 128)
    ref_b, _ = R.tree_verify_attn(b.q, b.k, b.v, b.mask, b.scale)
    for _ in range(2):
        check(run_attn(b, ws), ref_b, "shared workspace, second shape")
        assert np.array_equal(run_attn(a, ws).view(np.uint16), first.view(np.uint16))


def test_masked_draft_keys_have_no_influence():
    a = I.make_attn(8200, 40, 300, 16, 2, 128)
    base = run_attn(a)
    j = 25
    a.k[a.P + j] += np.float16(2.0)
    a.v[a.P + j] -= np.float16(1.0)
    pert = run_attn(a)
    for i in range(a.M):
        same = np.array_equal(pert[i].view(np.uint16), base[i].view(np.uint16))
        assert same == (a.mask[i, j] == 0), i


@pytest.mark.parametrize("gain", [6.0, 24.0])
def test_peaked_softmax(gain):
    """queries scaled up so that a handful of keys carry each row (logit spread of tens): the running-maximum
    rescaling across key steps, key ranges and the merge has to hold where exp() spans its whole range"""
    a = I.make_attn(8300 + int(gain), 60, 700, 16, 2, 128)
    a.q = (a.q.astype(np.float32) * gain).astype(np.float16)
    ref64, _ = R.tree_verify_attn(a.q, a.k, a.v, a.mask, a.scale)
    for splits in (0, 1, 5):
        B.w4a16_set_param("attn_splits", splits)
        for row_tiles in (0, 2):
            B.w4a16_set_param("attn_row_tiles", row_tiles)
            check(run_attn(a), ref64, f"peaked softmax x{gain} splits={splits} row_tiles={row_tiles}")


def test_constant_values_come_back_exactly():
    """V = c for every key: any convex combination of it is c, whatever the weights"""
    a = I.make_attn(8400, 33, 515, 8, 2, 128)
    a.v[...] = np.float16(0.375)
    for splits in (0, 4):
        B.w4a16_set_param("attn_splits", splits)
        got = run_attn(a).astype(np.float32)
        assert np.abs(got - 0.375).max() <= 2.0 ** -11 * 0.375 * 2, np.abs(got - 0.375).max()
