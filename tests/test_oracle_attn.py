"""Pins for the tree-verify attention oracle (paper section 2.1: all n draft-tree tokens are
scored by the target model in one pass; each sees the committed prefix, itself and its ancestors)
and for the draft-tree generator.  Expected values come from torch's CPU attention routine,
closed forms and invariants, never from the oracle itself."""
import numpy as np
import torch

from oracle import reference as R
from paper_2505_22179_amd import inputs as I


def _torch_sdpa(a: I.AttnInputs, full_mask: np.ndarray) -> np.ndarray:
    """library routine: dense boolean mask [M, P+M], GQA by repeating KV heads"""
    rep = a.Hq // a.Hkv
    q = torch.from_numpy(a.q.astype(np.float64)).permute(1, 0, 2)                      # [Hq, M, D]
    k = torch.from_numpy(a.k.astype(np.float64)).permute(1, 0, 2).repeat_interleave(rep, 0)
    v = torch.from_numpy(a.v.astype(np.float64)).permute(1, 0, 2).repeat_interleave(rep, 0)
    out = torch.nn.functional.scaled_dot_product_attention(
        q, k, v, attn_mask=torch.from_numpy(full_mask.astype(bool))[None], scale=a.scale)
    return out.permute(1, 0, 2).numpy()


def test_chain_tree_is_causal_attention():
    a = I.make_attn(1, M=9, P=37, Hq=8, Hkv=2, D=16, tree="chain")
    out64, _ = R.tree_verify_attn(a.q, a.k, a.v, a.mask, a.scale)
    T = a.P + a.M
    causal = np.tril(np.ones((T, T), dtype=bool))[a.P:, :]   # bottom rows of the causal matrix
    want = _torch_sdpa(a, causal)
    assert np.abs(out64 - want).max() < 1e-12
    # the same thing through torch's own is_causal path on the full sequence (prefix rows discarded)
    rep = a.Hq // a.Hkv
    qfull = torch.zeros(a.Hq, T, a.D, dtype=torch.float64)
    qfull[:, a.P:] = torch.from_numpy(a.q.astype(np.float64)).permute(1, 0, 2)
    k = torch.from_numpy(a.k.astype(np.float64)).permute(1, 0, 2).repeat_interleave(rep, 0)
    v = torch.from_numpy(a.v.astype(np.float64)).permute(1, 0, 2).repeat_interleave(rep, 0)
    o = torch.nn.functional.scaled_dot_product_attention(qfull, k, v, is_causal=True, scale=a.scale)
    assert np.abs(out64 - o[:, a.P:].permute(1, 0, 2).numpy()).max() < 1e-12


def test_random_tree_against_library_with_dense_mask():
    a = I.make_attn(2, M=20, P=50, Hq=8, Hkv=4, D=32, tree="random", depth=4, max_children=3)
    out64, out16 = R.tree_verify_attn(a.q, a.k, a.v, a.mask, a.scale)
    full = np.concatenate([np.ones((a.M, a.P), dtype=bool), a.mask.astype(bool)], axis=1)
    assert np.abs(out64 - _torch_sdpa(a, full)).max() < 1e-12
    assert np.array_equal(out16, out64.astype(np.float16))


def test_identity_mask_rows_are_independent_decodes():
    a = I.make_attn(3, M=5, P=11, Hq=4, Hkv=2, D=8, tree="identity")
    out64, _ = R.tree_verify_attn(a.q, a.k, a.v, a.mask, a.scale)
    for i in range(a.M):
        keys = list(range(a.P)) + [a.P + i]
        for h in range(a.Hq):
            kh = h // 2
            lg = torch.from_numpy(a.k[keys, kh].astype(np.float64) @ a.q[i, h].astype(np.float64) * a.scale)
            p = torch.softmax(lg, 0).numpy()
            assert np.abs(out64[i, h] - p @ a.v[keys, kh].astype(np.float64)).max() < 1e-13


def test_constant_v_and_zero_q_closed_forms():
    a = I.make_attn(4, M=7, P=13, Hq=4, Hkv=2, D=8, tree="random", depth=3, max_children=2)
    vconst = np.broadcast_to(np.linspace(-1, 1, a.D).astype(np.float16), a.v.shape).copy()
    out64, _ = R.tree_verify_attn(a.q, a.k, vconst, a.mask, a.scale)
    assert np.abs(out64 - vconst[0, 0].astype(np.float64)).max() < 1e-14
    # q = 0 gives uniform weights: the output is the mean of the visible V rows
    out64, _ = R.tree_verify_attn(np.zeros_like(a.q), a.k, a.v, a.mask, a.scale)
    for i in range(a.M):
        vis = list(range(a.P)) + [a.P + j for j in range(a.M) if a.mask[i, j]]
        for h in range(a.Hq):
            assert np.abs(out64[i, h] - a.v[vis, h // 2].astype(np.float64).mean(axis=0)).max() < 1e-14


def test_masked_keys_have_no_influence():
    a = I.make_attn(5, M=12, P=9, Hq=2, Hkv=1, D=8, tree="random", depth=4, max_children=3)
    base, _ = R.tree_verify_attn(a.q, a.k, a.v, a.mask, a.scale)
    for j in (3, 7, 11):
        k2, v2 = a.k.copy(), a.v.copy()
        k2[a.P + j] += np.float16(3.0)
        v2[a.P + j] -= np.float16(2.0)
        out, _ = R.tree_verify_attn(a.q, k2, v2, a.mask, a.scale)
        for i in range(a.M):
            same = np.array_equal(out[i], base[i])
            assert same == (a.mask[i, j] == 0), (i, j)


def test_scale_is_applied_to_logits():
    # one prefix key plus self: the two weights are sigmoid(+-scale * (q.k0 - q.k1))
    a = I.make_attn(6, M=1, P=1, Hq=1, Hkv=1, D=4, tree="identity")
    out64, _ = R.tree_verify_attn(a.q, a.k, a.v, a.mask, 0.37)
    qv = a.q[0, 0].astype(np.float64)
    d = 0.37 * (a.k[0, 0].astype(np.float64) @ qv - a.k[1, 0].astype(np.float64) @ qv)
    w0 = 1 / (1 + np.exp(-d))
    want = w0 * a.v[0, 0].astype(np.float64) + (1 - w0) * a.v[1, 0].astype(np.float64)
    assert np.abs(out64[0, 0] - want).max() < 1e-14


def test_tree_generator_structure():
    for seed in range(5):
        parent, dep, mask = I.make_tree(seed, 60, 6, 4)
        assert parent[0] == -1 and (parent[1:] < np.arange(1, 60)).all() and (parent[1:] >= 0).all()
        assert dep.max() == 6 and dep[0] == 0
        assert np.bincount(parent[1:], minlength=60).max() <= 4
        assert np.array_equal(mask, np.tril(mask)) and (np.diag(mask) == 1).all()
        assert np.array_equal(mask.sum(axis=1), dep + 1)
        assert (mask[:, 0] == 1).all()
        for i in range(1, 60):   # row i = row of its parent plus the diagonal
            want = mask[parent[i]].copy()
            want[i] = 1
            assert np.array_equal(mask[i], want)
