"""GPU: w4a16_gemm_static -- the entry point for callers that cannot allocate a workspace -- against
w4a16_gemm on the same inputs.  Both run the same kernels, so the outputs must agree bit for bit (and
w4a16_gemm is compared with the oracle in the other GPU tests).  Two calls in a row share the built-in scratch
array, the second smaller than the first, so whatever the first left behind must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"
SENTINEL = 1234.0


def both_ways(inp, M):
    x = torch.from_numpy(inp.x[:M]).to(DEV).contiguous()
    packed = B.pack_from_numpy(inp)
    ws = B.new_workspace(B.w4a16_workspace_bytes(M, inp.N, inp.K))
    want = torch.full((M + 2, inp.N), SENTINEL, dtype=torch.float16, device=DEV)
    B.w4a16_gemm(x, packed, want, M, inp.N, inp.K, 128, ws)
    got = torch.full((M + 2, inp.N), SENTINEL, dtype=torch.float16, device=DEV)
    B.w4a16_gemm_static(x, packed, got, M, inp.N, inp.K)
    return got, want


def test_static_scratch_matches_workspace_entry_on_consecutive_calls():
    # (M, K, N): default plans that split K across workgroups -- last-arriver sums (tickets) and two-kernel sums
    calls = [(40, 14336, 4096), (8, 14336, 4096), (64, 4096, 6144), (3, 8192, 1024), (1, 128, 8)]
    used_scratch = 0
    results = []
    for M, K, N in calls:   # enqueued back to back on one stream, no synchronisation in between
        print(f"static scratch M={M} K={K} N={N} plan {B.w4a16_plan_describe(M, N, K)}", flush=True)
        used_scratch += B.w4a16_plan_describe(M, N, K)[5] != 1
        results.append(both_ways(I.make_linear(7700 + M + K + N, M, K, N), M))
    torch.cuda.synchronize()
    assert used_scratch >= 3
    for (M, K, N), (got, want) in zip(calls, results):
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (M, K, N)
        assert (got[M:] == SENTINEL).all()


def test_static_scratch_rejects_what_it_cannot_hold():
    lib = B.load()
    a = 0x1000
    assert lib.w4a16_gemm_static(a, a, a, 0, 4096, 4096, 128, None) == -1
    assert lib.w4a16_gemm_static(a, a, a, 65, 4096, 4096, 128, None) == -4
    assert lib.w4a16_gemm_static(None, a, a, 1, 4096, 4096, 128, None) == -2
    assert lib.w4a16_gemm_static(a, a, a + 2, 1, 4096, 4096, 128, None) == -3
    # a forced 16-way K split of a wide weight at 64 rows needs 16 x 64 x 131072 x 4 bytes of partial sums
    B.w4a16_set_param("split_k", 16)
    try:
        assert lib.w4a16_gemm_static(a, a, a, 64, 131072, 8192, 128, None) == -5
    finally:
        B.w4a16_set_param("split_k", 0)
