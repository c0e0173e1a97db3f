"""GPU: bounded soak of the last-arriver reductions.

Where K (or the key range) is split across workgroups, the partial results of a column unit (or row tile) can
be summed by a second kernel or, inside the first, by whichever workgroup takes the last ticket.  Both add the
partials in split order, so the two modes must agree bit for bit on every call.  The in-kernel exchange relies
on device-scope stores, a wait for them and a relaxed ticket; this test calls it about two thousand times over
a mix of shapes, split counts, kernel families and epilogues and compares every result with the two-kernel mode
of the same call.  It stops at the first mismatch and names the call."""
import itertools

import pytest
import torch

from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

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
    B.w4a16_set_param("attn_fused_merge", 0)
    B.w4a16_set_param("attn_splits", 0)


# (M, K, N) and the knob sets that put a last-arriver sum on that call: the K-split workgroups (M <= 16 as the
# tuned plans use them, larger M too), the all-loads-up-front kernel, the column-split kernel with one, two and
# three K sets, and the library's own choice where it splits K
GEMM_CASES = [
    ((1, 8192, 1024), [dict(tiles_per_wave=8, waves_per_wg=8, prefetch_depth=1, split_k=4), dict(tiles_per_wave=2, waves_per_wg=4, prefetch_depth=2, split_k=3),
                       dict(tiles_per_wave=2, waves_per_wg=8, flat_groups=4, split_k=2)]),
    ((4, 4096, 2048), [dict(tiles_per_wave=4, waves_per_wg=8, prefetch_depth=1, split_k=4), dict(tiles_per_wave=4, waves_per_wg=4, flat_groups=4, split_k=2)]),
    ((8, 14336, 512), [dict(tiles_per_wave=4, waves_per_wg=8, prefetch_depth=1, split_k=4), dict(split_k=7)]),
    ((16, 4096, 1536), [dict(tiles_per_wave=4, waves_per_wg=8, prefetch_depth=1, split_k=2), dict(tiles_per_wave=8, waves_per_wg=8, prefetch_depth=1, split_k=4)]),
    ((24, 8192, 2048), [dict(tiles_per_wave=2, k_sets=3, prefetch_depth=1, split_k=3), dict(tiles_per_wave=2, k_sets=2, prefetch_depth=1, split_k=4),
                        dict(tiles_per_wave=8, waves_per_wg=4, prefetch_depth=1, split_k=4)]),
    ((40, 2048, 1024), [dict(tiles_per_wave=2, k_sets=3, prefetch_depth=1, split_k=2), dict(tiles_per_wave=4, k_sets=1, prefetch_depth=2, split_k=2)]),
    ((64, 4096, 1536), [dict(tiles_per_wave=4, k_sets=2, prefetch_depth=1, split_k=4), dict(tiles_per_wave=2, k_sets=2, prefetch_depth=2, split_k=3)]),
]


def test_last_arriver_gemm_matches_two_kernel_mode():
    ws = B.new_workspace(64 << 20)
    cases = []
    for (M, K, N), knob_sets in GEMM_CASES:
        inp = I.make_linear(7800 + M + K + N, M, K, N)
        res = I.make_hidden(7900 + M, M, N, 0)
        cases.append(dict(M=M, K=K, N=N, knob_sets=knob_sets, x=torch.from_numpy(inp.x).to(DEV), packed=B.pack_from_numpy(inp),
                          paired=B.pack_from_numpy(inp, gate_up=True), res=torch.from_numpy(res).to(DEV)))
    epilogues = (B.EPI_NONE, B.EPI_RESIDUAL, B.EPI_SILU_MUL)
    calls = 0
    for it, (case, epi) in zip(range(330), itertools.cycle(itertools.product(cases, epilogues))):
        M, K, N = case["M"], case["K"], case["N"]
        width = N // 2 if epi == B.EPI_SILU_MUL else N
        for knobs in case["knob_sets"]:
            outs = []
            for fused in (1, 0):
                set_knobs(**dict(knobs, fused_reduce=fused))
                y = torch.full((M + 1, width), 5.0, dtype=torch.float16, device=DEV)
                B.w4a16_gemm_fused(case["x"], case["paired"] if epi == B.EPI_SILU_MUL else case["packed"], y, M, N, K, 128, epi,
                                   case["res"] if epi == B.EPI_RESIDUAL else None, ws)
                outs.append(y)
                calls += 1
            if not torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)):
                plan = B.w4a16_plan_describe(M, N, K)
                pytest.fail(f"call {calls}: M={M} K={K} N={N} epilogue {epi} knobs {knobs}: the last-arriver sum differs from "
                            f"the second kernel's (plan {plan})")
    print(f"{calls} GEMM calls, last-arriver and two-kernel sums identical", flush=True)
    assert calls >= 1400


def test_last_arriver_attention_merge_matches_merge_kernel():
    """tree_verify_attn with the key ranges of a row tile merged by the last workgroup to finish, against the merge
    kernel: plain decoding and few-row verification, several range counts"""
    cases = []
    for M, P, Hq, Hkv, splits in ((1, 2048, 64, 8, 0), (1, 700, 16, 2, 5), (4, 1500, 32, 4, 0), (7, 2048, 64, 8, 3), (2, 300, 8, 8, 4),
                                  (16, 1000, 16, 4, 2)):
        a = I.make_attn(8800 + M + P, M=M, P=P, Hq=Hq, Hkv=Hkv, D=128, tree="chain" if M > 1 else "identity")
        cases.append((a, splits, tuple(torch.from_numpy(t).to(DEV) for t in (a.q, a.k, a.v, a.mask)),
                      B.new_workspace(B.tree_verify_attn_workspace_bytes(a.M, a.P, a.Hq, a.Hkv, a.D))))
    calls = 0
    for it in range(60):
        for a, splits, (q, k, v, mask), ws in cases:
            B.w4a16_set_param("attn_splits", splits)
            outs = []
            for mode in (2, 1):
                B.w4a16_set_param("attn_fused_merge", mode)
                out = torch.full((a.M + 1, a.Hq, a.D), 7.0, dtype=torch.float16, device=DEV)
                B.tree_verify_attn(q, k, v, mask, out, a.M, a.P, a.Hq, a.Hkv, a.D, a.scale, ws)
                outs.append(out)
                calls += 1
            if not torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)):
                pytest.fail(f"call {calls}: M={a.M} P={a.P} Hq={a.Hq} Hkv={a.Hkv} ranges {splits}: the in-kernel merge differs "
                            f"from the merge kernel")
    print(f"{calls} attention calls, in-kernel and second-kernel merges identical", flush=True)
    assert calls >= 700
