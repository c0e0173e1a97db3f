"""GPU: lm_head_topk through the C ABI against the fp64 oracle.

Tolerances.  Logits are fp32 sums of K exact fp16 x fp16 products: |err| <= 1e-3 and relative Frobenius
error <= 1e-4 against fp64 (the observed error is orders below).  Log-probabilities add a log-sum-exp in
fp32: |err| <= 2e-3.  The top-k order is an integer decision taken on floating-point values, so where two
logits are closer than the logit tolerance either order is correct: the test compares what is unique
(tokens separated from the k-th by more than the tolerance must match exactly, in order) and checks that
the rest is valid (every reported token's true logit reaches the true k-th logit within the tolerance,
reported order non-increasing within it).  Exact ties (identical weight rows) must come out in ascending
token order, bit-identical logits included."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = 1e-3


def run(x, W, top_k):
    M, K = x.shape
    V = W.shape[0]
    xd, Wraw = torch.from_numpy(x).to(DEV), torch.from_numpy(W).to(DEV)
    Wd = torch.empty(B.lm_head_packed_bytes(V, K), dtype=torch.uint8, device=DEV)
    B.lm_head_pack(Wraw, Wd, V, K)
    del Wraw
    logits = torch.full((M + 1, V), 7.0, dtype=torch.float32, device=DEV)
    idx = torch.full((M + 1, top_k), -5, dtype=torch.int32, device=DEV)
    lp = torch.full((M + 1, top_k), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(B.lm_head_workspace_bytes(M, V, K, top_k), dtype=torch.uint8, device=DEV)
    B.lm_head_topk(xd, Wd, M, V, K, top_k, logits, idx, lp, ws)
    torch.cuda.synchronize()
    L, Ix, P = logits.cpu().numpy(), idx.cpu().numpy(), lp.cpu().numpy()
    assert (L[M:] == 7.0).all() and (Ix[M:] == -5).all() and (P[M:] == 7.0).all(), "rows >= M were written"
    return L[:M], Ix[:M], P[:M]


def check(x, W, top_k, what):
    L, Ix, P = run(x, W, top_k)
    ref, ridx, rlp = R.lm_head_topk(x, W, min(top_k + 1, W.shape[0]))
    err = np.abs(L - ref)
    assert err.max() <= TOL, f"{what}: logits max abs err {err.max():.3g}"
    assert np.linalg.norm(L - ref) <= 1e-4 * max(np.linalg.norm(ref), 1e-30) + 1e-7, what
    M = x.shape[0]
    mx = ref.max(axis=1)
    lse = mx + np.log(np.exp(ref - mx[:, None]).sum(axis=1))
    for m in range(M):
        got = Ix[m].tolist()
        assert len(set(got)) == top_k and all(0 <= t < W.shape[0] for t in got), f"{what}: row {m} tokens {got}"
        true = ref[m, got]
        kth = ref[m, ridx[m, top_k - 1]]
        assert (true >= kth - 2 * TOL).all(), f"{what}: row {m} reports a token below the true top-k"
        assert (np.diff(true) <= 2 * TOL).all(), f"{what}: row {m} order"
        assert np.abs(P[m] - (true - lse[m])).max() <= 2e-3, f"{what}: row {m} log-probabilities"
        # unique part: oracle picks separated from their neighbours by more than the tolerance
        srt = ref[m, ridx[m]]
        for j in range(top_k):
            lo_gap = srt[j] - srt[j + 1] if j + 1 < len(srt) else np.inf
            hi_gap = srt[j - 1] - srt[j] if j > 0 else np.inf
            if lo_gap > 4 * TOL and hi_gap > 4 * TOL:
                assert got[j] == ridx[m, j], f"{what}: row {m} position {j}: {got[j]} vs {ridx[m, j]}"
    return float(err.max())


@pytest.mark.parametrize("M,K,V,top_k", [
    (1, 128, 16, 3), (3, 384, 1001, 7), (16, 512, 4096, 10), (10, 1024, 5000, 1), (7, 2048, 2049, 64),
    (2, 4096, 32000, 32), (16, 8192, 6000, 10), (17, 1024, 3000, 4), (40, 2048, 4104, 10), (48, 384, 2000, 3),
    (64, 4096, 8000, 10), (60, 8192, 2048, 1),
])
def test_lm_head_parity(M, K, V, top_k):
    print(f"lm_head M={M} K={K} V={V} top_k={top_k}", flush=True)
    x, W = I.make_lm_head(9500 + M + K + V, M, K, V)
    try:
        for tiles_per_wave in (0, 1, 2) + ((4,) if M > 16 else ()):
            B.w4a16_set_param("lm_tiles", tiles_per_wave)
            e = check(x, W, top_k, f"M={M} K={K} V={V} k={top_k} tiles per wavefront {tiles_per_wave}")
    finally:
        B.w4a16_set_param("lm_tiles", 0)
    print(f"    logits max abs err {e:.3g}", flush=True)


def test_lm_head_full_vocabulary():
    """the benchmark's configuration: Llama-3 vocabulary, hidden size 4096, ten beams, top 10"""
    M, K, V, top_k = 10, 4096, 128256, 10
    print("lm_head full vocabulary", flush=True)
    x, W = I.make_lm_head(9600, M, K, V)
    check(x, W, top_k, "full vocabulary")


def test_exact_ties_come_out_in_token_order():
    M, K, V = 2, 256, 3000
    x, W = I.make_lm_head(9700, M, K, V)
    W[2500] = W[77]
    W[1031] = W[77]
    x[0] = (W[77].astype(np.float32) * 30).astype(np.float16)   # token 77 and its copies win row 0
    L, Ix, P = run(x, W, 5)
    assert Ix[0, :3].tolist() == [77, 1031, 2500]
    assert L[0, 77] == L[0, 1031] == L[0, 2500] and P[0, 0] == P[0, 1] == P[0, 2]


def test_determinism():
    x, W = I.make_lm_head(9800, 5, 1024, 20000)
    a = run(x, W, 10)
    b = run(x, W, 10)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
