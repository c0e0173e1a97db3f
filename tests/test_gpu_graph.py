"""GPU: the library's calls captured in a HIP graph and replayed.  A replay must give the bits of the eager call
every time -- also after other eager calls have used the same workspaces in between (tickets back at zero,
partial sums rewritten before they are read, nothing recorded that a replay does differently)."""
import numpy as np
import pytest
import torch

from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("M", [1, 24, 60])
def test_decoder_layer_graph_replays_equal_the_eager_call(M):
    print(f"graph replay of the decoder layer, M={M}", flush=True)
    P, Hq, Hkv, D, H, Iff = 300, 16, 4, 128, 2048, 5632
    Nqkv = (Hq + 2 * Hkv) * D
    rng = np.random.default_rng(9400 + M)
    lin = {name: I.make_linear(9410 + i, M, K, N) for i, (name, K, N) in
           enumerate((("qkv", H, Nqkv), ("o", Hq * D, H), ("gate_up", H, 2 * Iff), ("down", Iff, H)))}
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device=DEV)
    packed = [B.pack_from_numpy(lin["qkv"], head_dim=D), B.pack_from_numpy(lin["o"]),
              B.pack_from_numpy(lin["gate_up"], gate_up=True), B.pack_from_numpy(lin["down"])]
    h0 = dev(I.make_hidden(9420, M, H))
    g1, g2 = dev(I.make_gamma(9421, H)), dev(I.make_gamma(9422, H))
    if M > 1:
        parent, _, mask = I.make_tree(9423, M, 5, 3)
    else:
        parent, mask = np.array([-1]), np.ones((1, 1), dtype=np.uint8)
    pos, maskd = dev(I.tree_positions(parent, P)), dev(mask)
    cos, sin = (dev(t) for t in I.make_rope_tables(P + 16, D))
    k0 = dev(rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16))
    v0 = dev(rng.standard_normal((P + M, Hkv, D), dtype=np.float32).astype(np.float16))
    ws = B.new_workspace(max(B.w4a16_workspace_bytes(M, n, k) for n, k in ((Nqkv, H), (H, Hq * D), (2 * Iff, H), (H, Iff))))
    aws = B.new_workspace(B.tree_verify_attn_workspace_bytes(M, P, Hq, Hkv, D))
    weights = B.layer_weights(*packed, g1, g2, H, Hq, Hkv, D, Iff, 1e-5, qkv_heads_packed=True)
    bufs = [f16(M, H), None, f16(M, Hq, D), f16(M, Hq, D), f16(M, Iff)]
    scratch = B.layer_scratch(*bufs, ws, aws)
    h, k, v = h0.clone(), k0.clone(), v0.clone()

    def layer():
        B.w4a16_decoder_layer(weights, h, M, P, pos, cos, sin, P + 16, maskd, k, v, scratch)

    layer()
    torch.cuda.synchronize()
    want = (h.clone(), k.clone(), v.clone())
    graph = torch.cuda.CUDAGraph()
    h.copy_(h0); k.copy_(k0); v.copy_(v0)
    with torch.cuda.graph(graph):
        layer()
    # other work on the same workspaces between the replays: a linear of another shape and an attention call
    other = I.make_linear(9430, 40, 1024, 1056)
    other_packed, ox, oy = B.pack_from_numpy(other), dev(other.x), f16(40, 1056)
    oq, oout = f16(M, Hq, D).normal_(), f16(M, Hq, D)
    for replay in range(4):
        h.copy_(h0); k.copy_(k0); v.copy_(v0)
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((h, k, v), want, ("hidden state", "K cache", "V cache")):
            assert torch.equal(got, ref), f"replay {replay}: {name} differs from the eager call"
        B.w4a16_gemm(ox, other_packed, oy, 40, 1056, 1024, 128, ws)
        B.tree_verify_attn(oq, k0, v0, maskd, oout, M, P, Hq, Hkv, D, 0.05, aws)
        torch.cuda.synchronize()


def test_gemm_graph_with_last_arriver_sums_replays(request):
    """a K split summed by last arrivers (tickets) and one summed by a second kernel, both inside one graph"""
    M, K, N = 20, 4096, 1056
    inp = I.make_linear(9440, M, K, N)
    packed = B.pack_from_numpy(inp)
    x = torch.from_numpy(inp.x).to(DEV)
    ws = B.new_workspace(64 << 20)
    ya, yb = (torch.empty((M, N), dtype=torch.float16, device=DEV) for _ in range(2))

    def both():
        B.w4a16_set_param("split_k", 4); B.w4a16_set_param("fused_reduce", 1)
        B.w4a16_gemm(x, packed, ya, M, N, K, 128, ws)
        B.w4a16_set_param("fused_reduce", 0)
        B.w4a16_gemm(x, packed, yb, M, N, K, 128, ws)

    try:
        both()
        torch.cuda.synchronize()
        want = (ya.clone(), yb.clone())
        assert torch.equal(*want), "the two ways to sum the K splits add in the same order"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            both()
        for replay in range(4):
            ya.zero_(); yb.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(ya, want[0]) and torch.equal(yb, want[1]), replay
            B.w4a16_set_param("split_k", 3); B.w4a16_set_param("fused_reduce", 1)
            B.w4a16_gemm(x, packed, ya, M, N, K, 128, ws)   # eager, another split, same tickets
            torch.cuda.synchronize()
    finally:
        B.w4a16_set_param("split_k", 0)
        B.w4a16_set_param("fused_reduce", 2)
