"""Launch-shape tuner for w4a16_gemm (needs a GPU).

For every (layer shape, row bucket: M <= 8, 9..16, 17..32, ...) it times each compiled kernel variant -- tiles per
wavefront, wavefronts per workgroup, prefetch depth, K splits, fused or two-kernel reduction --
through the library's ablation knobs (for M > 16 also the high-occupancy column-split variant and its K sets), on weights rotated through more than 512 MB so the
last-level cache never serves them, and writes the winners as rows of csrc/tuned_plans.inc.  The
library falls back to a generic rule for shapes that have no row.

    python -m paper_2505_22179_amd.tune --out tuned_plans.inc [--flat-out tuned_flat.inc] [--shapes 70b,8b]

Rebuild the library after copying the outputs over csrc/tuned_plans.inc and csrc/tuned_flat.inc.
"""
from __future__ import annotations

import argparse
import collections
import sys

import torch

from . import binding as B
from . import inputs as I

G = 128
KNOBS = ("tiles_per_wave", "waves_per_wg", "prefetch_depth", "split_k", "fused_reduce", "k_sets", "flat_groups")
# a plan's split_k field of 0 together with k_sets > 0 means the even split of the column-split kernel
# (not among the candidates: it lost to the plain K split on every Llama-3 shape, by 3 to 60 %)
FLAT_MAX_M = 4   # the all-loads-up-front variant stages at most this many rows


def weight_bytes(K: int, N: int) -> int:
    return K * N // 2 + (K // G) * N * 5 // 2


def make_packed(K: int, N: int, copies: int, seed: int = 1):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (K // 8, N), dtype=torch.int32, device="cuda", generator=gen)
    sc = (torch.rand((K // G, N), device="cuda", generator=gen) * 9e-3 + 1e-3).to(torch.float16)
    qz = torch.randint(-2 ** 31, 2 ** 31 - 1, (K // G, N // 8), dtype=torch.int32, device="cuda", generator=gen)
    p = torch.empty(B.w4a16_packed_bytes(N, K, G), dtype=torch.uint8, device="cuda")
    B.w4a16_pack(qw, sc, qz, p, N, K, G)
    return [p] + [p.clone() for _ in range(copies - 1)]


def time_graph(fn, copies: int, min_us: float = 1500.0) -> float:
    """Microseconds per launch: a HIP graph of `copies` launches (one per weight copy), replayed
    back to back for at least min_us after an equally long warm-up so that clocks stay up."""
    for c in range(copies):
        fn(c)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for c in range(copies):
            fn(c)
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    g.replay()
    b.record()
    torch.cuda.synchronize()
    n = max(4, int(min_us / max(a.elapsed_time(b) * 1e3, 1.0)) + 1)
    best = 1e9
    for _ in range(2):
        for _ in range(n):
            g.replay()
        a.record()
        for _ in range(n):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) / (n * copies))
    return best * 1e3


def set_knobs(values) -> None:
    for k, v in zip(KNOBS, values):
        B.w4a16_set_param(k, v)
    B.w4a16_set_param("even_split", 1 if (values[5] > 0 and values[3] == 0) else 0)


def candidates(N: int, K: int, M: int):
    if M > 16:   # high-occupancy column-split workgroups (k_sets > 0), compiled for M > 16 only
        for tw in (8, 4, 2):
            for ks in (1, 2, 3):
                for depth in (1, 2):
                    for S in (1, 2, 3, 4, 5, 6, 8, 10, 12, 16):
                        wgs = ((N // 16) // tw + 3) // 4 * S
                        if wgs < 160 or wgs > 2048 or S * ks * 2 > K // G:
                            continue
                        for fused in ((0,) if S == 1 else (0, 1)):
                            yield (tw, 0, depth, S, fused, ks, 0)
    for tw in (8, 4, 2):
        for nw in (1, 4, 8, 16):   # 1 = column-split workgroup sharing x through LDS
            for depth in (1, 2, 4):
                for S, fused in ((1, 1), (2, 1), (2, 0), (3, 0), (4, 1), (4, 0), (6, 0), (8, 0)):
                    units = (N // 16) // tw
                    waves = units * S * (nw if nw > 1 else 1)
                    if waves < 768 or waves > 16384 or S * max(nw, 2) > K // G or (nw == 1 and fused == 1 and S > 1):
                        continue
                    yield (tw, nw, depth, S, fused, 0, 0)


def flat_candidates(N: int, K: int):
    """all-loads-up-front variant (M <= FLAT_MAX_M): K / G must equal S * nw * ng exactly"""
    for tw in (2, 4, 8):
        for nw in (4, 8, 16):
            for ng in (4, 7, 8):
                for S in (1, 2, 3, 4, 6, 8):
                    if K // G != S * nw * ng:
                        continue
                    for fused in ((1,) if S == 1 else (1, 0)):
                        yield (tw, nw, 0, S, fused, 0, ng)


def tune_shape(name: str, K: int, N: int, Ms, ws, log):
    wb = weight_bytes(K, N)
    copies = max(3, int(700e6 // wb) + 1)
    packs = make_packed(K, N, copies)
    per_bucket = collections.defaultdict(list)   # row bucket (0: M <= 8, else 16-row tiles) -> list of {plan: us}
    flat_runs = []                               # M <= FLAT_MAX_M: ({flat plan: us}, best non-flat us)
    for M in Ms:
        x = torch.randn((M, K), device="cuda").to(torch.float16)
        y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        res = {}
        # the many-row kernels are bound by instruction issue and follow the clock, which sags under
        # sustained load: time them over a longer stretch than the memory-bound few-row kernels
        min_us = 1500.0 if M <= 16 else 12000.0
        for plan in candidates(N, K, M):
            set_knobs(plan)
            try:
                res[plan] = time_graph(lambda c: B.w4a16_gemm(x, packs[c], y, M, N, K, G, ws), copies, min_us)
            except B.W4A16Error:
                continue   # variant not compiled for this M
        best = min(res.values())
        if M <= FLAT_MAX_M:
            fres = {}
            for plan in flat_candidates(N, K):
                set_knobs(plan)
                try:
                    fres[plan] = time_graph(lambda c: B.w4a16_gemm(x, packs[c], y, M, N, K, G, ws), copies)
                except B.W4A16Error:
                    continue
            flat_runs.append((fres, best))
            if fres:
                fp, fus = min(fres.items(), key=lambda kv: kv[1])
                log(f"{name} K={K} N={N} M={M}: best all-loads-up-front [tw{fp[0]} nw{fp[1]} ng{fp[6]} S{fp[3]}{'f' if fp[4] else 'k'} {fus:.1f}us] vs {best:.1f}us")
        top = sorted(res.items(), key=lambda kv: kv[1])[:4]
        log(f"{name} K={K} N={N} M={M}: ideal {wb / 8e6:.1f} us | " +
            " ".join(f"[tw{p[0]} {'ks%d' % p[5] if p[5] else 'nw%d' % p[1]} d{p[2]} S{p[3]}{'f' if p[4] else 'k'} {us:.1f}us]" for p, us in top))
        per_bucket[0 if M <= 8 else (M + 15) // 16].append({p: us / best for p, us in res.items()})
    set_knobs((0, 0, 0, 0, 2, 0, 0))
    rows = []
    for mt, runs in sorted(per_bucket.items()):
        common = set(runs[0])
        for r in runs[1:]:
            common &= set(r)
        plan = min(common, key=lambda p: sum(r[p] for r in runs))
        rows.append((N, K, mt) + plan[:6])
    flat_rows = []
    if flat_runs and all(f for f, _ in flat_runs):
        common = set(flat_runs[0][0])
        for f, _ in flat_runs[1:]:
            common &= set(f)
        if common:
            plan = min(common, key=lambda p: sum(f[p] / b for f, b in flat_runs))
            if sum(f[plan] / b for f, b in flat_runs) < 0.98 * len(flat_runs):   # a clear win at every small M together
                flat_rows.append((N, K, FLAT_MAX_M, plan[0], plan[1], plan[6], plan[3], plan[4]))
    del packs
    torch.cuda.empty_cache()
    return rows, flat_rows


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    ap.add_argument("--flat-out", default=None, help="rows for csrc/tuned_flat.inc (default: <out>.flat)")
    ap.add_argument("--shapes", default="70b,8b")
    ap.add_argument("--M", default="1,4,8,12,16,32,48,64")
    args = ap.parse_args()
    Ms = [int(m) for m in args.M.split(",")]
    ws = B.new_workspace(1 << 30)

    def log(s):
        print(s, file=sys.stderr, flush=True)

    rows, flat_rows = [], []
    for which in args.shapes.split(","):
        for name, K, N in (I.LLAMA3_70B if which == "70b" else I.LLAMA3_8B):
            r, f = tune_shape(f"{which}.{name}", K, N, Ms, ws, log)
            rows += r
            flat_rows += f
    with open(args.out, "w") as f:
        f.write("// Tuned launch shapes, written by `python -m paper_2505_22179_amd.tune` on an MI355X.\n")
        f.write("// {N, K, row bucket (0: M <= 8, else 16-row tiles), tiles per wavefront, wavefronts per workgroup, prefetch depth, K splits, fused reduce, K sets}\n")
        for r in rows:
            f.write("{" + ", ".join(str(v) for v in r) + "},\n")
    flat_out = args.flat_out or args.out + ".flat"
    with open(flat_out, "w") as f:
        f.write("// Tuned launch shapes of the all-loads-up-front variant, written by `python -m paper_2505_22179_amd.tune`.\n")
        f.write("// {N, K, largest M, tiles per wavefront, wavefronts per workgroup, groups per wavefront, K splits, fused reduce}\n")
        for r in flat_rows:
            f.write("{" + ", ".join(str(v) for v in r) + "},\n")
    log(f"wrote {len(rows)} rows to {args.out} and {len(flat_rows)} rows to {flat_out}")


if __name__ == "__main__":
    main()
