"""GPU: tree_accept through the C ABI against the CPU oracle -- integer work, so everything is
compared bit for bit (accepted path, count, next token, and every byte of the K/V cache)."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run(parent, token, target, k=None, v=None, P=0):
    M = len(parent)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)
    path = torch.full((M + 4,), 777, dtype=torch.int32, device=DEV)     # 4 guard words
    result = torch.full((4,), 777, dtype=torch.int32, device=DEV)
    if k is None:
        B.tree_accept(d(parent), d(token), d(target), M, path, result)
        kk = vv = None
    else:
        kk, vv = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
        B.tree_accept(d(parent), d(token), d(target), M, path, result, kk, vv, P, k.shape[1], k.shape[2])
    torch.cuda.synchronize()
    path, result = path.cpu().numpy(), result.cpu().numpy()
    assert (path[M:] == 777).all() and (result[2:] == 777).all(), "wrote past its outputs"
    n = int(result[0])
    assert (path[n:M] == -1).all()
    return list(path[:n]), int(result[1]), (kk.cpu().numpy() if kk is not None else None), (vv.cpu().numpy() if vv is not None else None)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("M,depth,p_accept", [(60, 6, 0.8), (64, 12, 0.97), (1, 6, 0.5), (7, 6, 0.9), (33, 4, 0.2)])
def test_accept_and_compact_match_oracle(seed, M, depth, p_accept):
    print(f"tree_accept M={M} depth={depth} seed={seed}", flush=True)
    parent, _, _ = I.make_tree(300 + seed, M, depth, 4) if M > 1 else (np.array([-1]), None, None)
    token, target = I.make_verify(400 + seed, parent, p_accept=p_accept)
    P, Hkv, D = 37 + seed, 8, 128
    rng = np.random.default_rng(500 + seed)
    k = rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16)
    v = rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16)
    want_path, want_next = R.tree_accept(parent, token, target)
    want_k, want_v = R.kv_compact(k, v, want_path, P)
    path, nxt, k2, v2 = run(parent, token, target, k, v, P)
    assert path == want_path and nxt == want_next
    assert np.array_equal(k2.view(np.uint16), want_k.view(np.uint16)) and np.array_equal(v2.view(np.uint16), want_v.view(np.uint16))
    # without a cache the walk alone gives the same answer
    assert run(parent, token, target)[:2] == (want_path, want_next)


def test_accept_full_chain_and_small_rows():
    M = 64
    parent, _, _ = I.chain_tree(M)
    token = np.arange(10, 10 + M, dtype=np.int32)
    target = np.concatenate([token[1:], [5]]).astype(np.int32)      # every draft token is right
    k = np.arange((3 + M) * 1 * 8, dtype=np.float32).reshape(3 + M, 1, 8).astype(np.float16)   # 16-byte rows
    v = -k
    path, nxt, k2, v2 = run(parent, token, target, k, v, 3)
    assert path == list(range(M)) and nxt == 5
    assert np.array_equal(k2, k) and np.array_equal(v2, v)          # the identity path moves nothing


def test_accept_duplicate_siblings_and_malformed_parent():
    assert run([-1, 0, 0, 1, 2], [0, 5, 5, 6, 6], [5, 9, 6, 0, 0])[:2] == ([0, 1], 9)
    # a parent entry that points forwards makes its node unreachable; the call still terminates in bounds
    assert run([-1, 3, 0, 0], [0, 8, 7, 7], [7, 1, 2, 8])[:2] == ([0, 2], 2)


def test_accept_is_deterministic_and_graph_capturable():
    parent, _, _ = I.make_tree(11, 60, 6, 4)
    token, target = I.make_verify(12, parent, p_accept=0.9)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)
    dp, dt, dg = d(parent), d(token), d(target)
    path = torch.zeros(60, dtype=torch.int32, device=DEV)
    result = torch.zeros(2, dtype=torch.int32, device=DEV)
    B.tree_accept(dp, dt, dg, 60, path, result)
    torch.cuda.synchronize()
    first = (path.clone(), result.clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.tree_accept(dp, dt, dg, 60, path, result)
    for _ in range(3):
        path.zero_(); result.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(path, first[0]) and torch.equal(result, first[1])
