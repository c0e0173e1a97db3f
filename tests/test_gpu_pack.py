"""GPU: w4a16_pack / w4a16_unpack / w4a16_dequant through the C ABI, bit-exact against the oracle."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import binding as B
from paper_2505_22179_amd import inputs as I

pytestmark = pytest.mark.gpu

SHAPES = [(128, 8), (256, 136), (384, 128), (1024, 200), (512, 1000), (4096, 4096)]


@pytest.mark.parametrize("K,N", SHAPES)
def test_pack_unpack_roundtrip_and_dequant(K, N):
    print(f"pack/unpack/dequant K={K} N={N}", flush=True)
    inp = I.make_linear(900 + K + N, 1, K, N)
    dev = "cuda"
    qw = torch.from_numpy(inp.qweight).to(dev)
    sc = torch.from_numpy(inp.scales).to(dev)
    qz = torch.from_numpy(inp.qzeros).to(dev)
    packed = torch.full((B.w4a16_packed_bytes(N, K),), 0xAB, dtype=torch.uint8, device=dev)
    B.w4a16_pack(qw, sc, qz, packed, N, K)
    qw2, sc2, qz2 = torch.empty_like(qw), torch.empty_like(sc), torch.empty_like(qz)
    B.w4a16_unpack(packed, qw2, sc2, qz2, N, K)
    W = torch.empty((K, N), dtype=torch.float32, device=dev)
    B.w4a16_dequant(packed, W, N, K)
    torch.cuda.synchronize()
    assert torch.equal(qw2, qw) and torch.equal(qz2, qz)
    assert torch.equal(sc2.view(torch.int16), sc.view(torch.int16))
    want = R.dequant(inp.qweight, inp.scales, inp.qzeros, 128)
    got = W.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_structured_codes_hit_the_right_cells():
    # code = k % 16 in column block 0, n % 16 elsewhere; zero-point = (g + n) % 16: any slip in the
    # layout's row/column bookkeeping shows up as a wrong dequantised cell
    K, N = 512, 264
    k = np.arange(K)[:, None]
    n = np.arange(N)[None, :]
    codes = np.where(n < 128, k % 16, n % 16).astype(np.uint8)
    zeros = ((np.arange(K // 128)[:, None] + n) % 16).astype(np.uint8)
    scales = (2.0 ** -(1 + (n % 5)) * np.ones((K // 128, 1))).astype(np.float16)
    qw, qz = I.pack_rows(codes), I.pack_cols(zeros)
    dev = "cuda"
    packed = torch.empty(B.w4a16_packed_bytes(N, K), dtype=torch.uint8, device=dev)
    B.w4a16_pack(torch.from_numpy(qw).to(dev), torch.from_numpy(scales).to(dev), torch.from_numpy(qz).to(dev), packed, N, K)
    W = torch.empty((K, N), dtype=torch.float32, device=dev)
    B.w4a16_dequant(packed, W, N, K)
    torch.cuda.synchronize()
    want = R.dequant(qw, scales, qz, 128)
    assert np.array_equal(W.cpu().numpy(), want)
