"""Pins for the greedy tree-acceptance and KV-compaction oracle (paper section 2.1 draft-then-verify,
section 4 tree-to-sequence verification).  The paper prints no worked example, so the pins are
brute force over all root paths, closed forms on chains, planted paths and library gathers."""
import numpy as np
import pytest

from oracle import reference as R
from paper_2505_22179_amd import inputs as I


def brute_force_path(parent, token, target):
    """Longest root path all of whose nodes were drafted correctly, by enumerating every node's
    root path.  With distinct sibling tokens at most one child of a node can match, so the longest
    fully matching path is unique and must be what the greedy walk returns."""
    n = len(parent)
    best = [0]
    for leaf in range(n):
        chain = []
        j = leaf
        while j >= 0:
            chain.append(j)
            j = int(parent[j])
        chain.reverse()
        if all(int(token[c]) == int(target[int(parent[c])]) for c in chain[1:]) and len(chain) > len(best):
            best = chain
    return best


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("n,depth,p_accept", [(60, 6, 0.8), (64, 10, 0.95), (7, 6, 0.9), (33, 4, 0.3)])
def test_accept_matches_brute_force(seed, n, depth, p_accept):
    parent, _, _ = I.make_tree(900 + seed, n, depth, 4)
    token, target = I.make_verify(1900 + seed, parent, p_accept=p_accept)
    path, nxt = R.tree_accept(parent, token, target)
    assert path == brute_force_path(parent, token, target)
    assert nxt == int(target[path[-1]])
    assert path[0] == 0 and all(int(parent[b]) == a for a, b in zip(path, path[1:]))


def test_accept_chain_closed_form():
    # a chain accepts exactly its leading run of correct tokens
    n = 20
    parent, _, _ = I.chain_tree(n)
    token = np.arange(100, 100 + n, dtype=np.int32)
    for run in (0, 1, 7, n - 1):
        target = np.full(n, -5, dtype=np.int32)
        target[:run] = token[1:run + 1]
        path, nxt = R.tree_accept(parent, token, target)
        assert path == list(range(run + 1)) and nxt == int(target[run])


def test_accept_nothing_and_single_node():
    parent, _, _ = I.make_tree(3, 30, 5, 4)
    token, _ = I.make_verify(4, parent)
    target = np.full(30, -1, dtype=np.int32)   # no draft token is -1
    assert R.tree_accept(parent, token, target) == ([0], -1)
    assert R.tree_accept([-1], [9], [42]) == ([0], 42)


def test_accept_planted_path_and_wrong_branch():
    #        0
    #      / | \
    #     1  2  3        node 2's subtree holds the planted path 0-2-5-6
    #    /   |\
    #   4    5 7
    #        |
    #        6
    parent = [-1, 0, 0, 0, 1, 2, 5, 2]
    token = [0, 11, 12, 13, 14, 15, 16, 17]
    target = [12, 14, 15, 99, 99, 16, 77, 99]
    assert R.tree_accept(parent, token, target) == ([0, 2, 5, 6], 77)
    # node 4 would match its parent's target, but its parent (1) is not accepted: it must not count
    target2 = [13, 14, 15, 99, 99, 16, 77, 99]
    assert R.tree_accept(parent, token, target2) == ([0, 3], 99)


def test_accept_duplicate_siblings_take_lowest_index():
    parent = [-1, 0, 0, 1, 2]
    token = [0, 5, 5, 6, 6]
    target = [5, 9, 6, 0, 0]      # both children of the root match; only the second one's child matches
    assert R.tree_accept(parent, token, target) == ([0, 1], 9)


def test_kv_compact_is_a_gather_and_touches_nothing_else():
    rng = np.random.default_rng(5)
    P, M, Hkv, D = 9, 12, 2, 8
    k = rng.standard_normal((P + M, Hkv, D)).astype(np.float16)
    v = rng.standard_normal((P + M, Hkv, D)).astype(np.float16)
    path = [0, 3, 4, 9]
    k2, v2 = R.kv_compact(k, v, path, P)
    assert np.array_equal(k2[P:P + 4], k[P + np.array(path)]) and np.array_equal(v2[P:P + 4], v[P + np.array(path)])
    assert np.array_equal(k2[:P], k[:P]) and np.array_equal(k2[P + 4:], k[P + 4:])
    assert np.array_equal(v2[:P], v[:P]) and np.array_equal(v2[P + 4:], v[P + 4:])
    # the identity path changes nothing; inputs are never modified
    k3, v3 = R.kv_compact(k, v, [0, 1, 2], P)
    assert np.array_equal(k3, k) and np.array_equal(v3, v)
    # the same result as moving rows one after the other in place, in path order
    kin = k.copy()
    for j, node in enumerate(path):
        kin[P + j] = kin[P + node]
    assert np.array_equal(kin, k2)


def test_verify_generator_structure():
    parent, _, _ = I.make_tree(77, 60, 6, 4)
    token, target = I.make_verify(78, parent)
    for p in range(60):
        kids = [i for i in range(1, 60) if parent[i] == p]
        assert len({int(token[i]) for i in kids}) == len(kids)   # distinct sibling tokens
    lens = [len(R.tree_accept(parent, *I.make_verify(s, parent, p_accept=0.8))[0]) for s in range(200)]
    assert 1.5 < np.mean(lens) < 5.5 and max(lens) <= 7
