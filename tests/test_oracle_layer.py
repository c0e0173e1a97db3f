"""Pins of the oracle's layer glue (RMS norm, residual / SiLU-gate epilogues, rotary embedding with
K/V append): closed forms, one-hot inputs that turn the linear into a table lookup computed here with
Python floats, invariants of rotations, and the torch library routines."""
import math

import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2505_22179_amd import inputs as I


# ---- SiLU ----------------------------------------------------------------------------------------

def test_silu_closed_forms():
    assert R.silu(0.0) == 0.0
    xs = np.linspace(-12, 12, 97)
    np.testing.assert_allclose(R.silu(xs) - R.silu(-xs), xs, rtol=0, atol=1e-14)   # x s(x) + x s(-x) = x
    assert abs(R.silu(40.0) - 40.0) < 1e-15 and abs(R.silu(-40.0)) < 1e-15
    h = 1e-6
    assert abs((R.silu(h) - R.silu(-h)) / (2 * h) - 0.5) < 1e-9                    # slope 1/2 at 0
    # the minimum: d/dx = s(x)(1 + x(1 - s(x))) = 0  <=>  1 + x + exp(-x)... solved here by bisection
    lo, hi = -2.0, -1.0
    f = lambda t: 1.0 + t * (1.0 - 1.0 / (1.0 + math.exp(-t)))
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if f(mid) < 0 else (lo, mid)
    xm = 0.5 * (lo + hi)
    grid = np.linspace(-3, 0, 30001)
    assert abs(grid[np.argmin(R.silu(grid))] - xm) < 2e-4
    assert abs(R.silu(xm) - xm / (1.0 + math.exp(-xm))) < 1e-15


def test_silu_against_python_floats_and_torch():
    rng = np.random.default_rng(1)
    xs = rng.standard_normal(200) * 4
    mine = R.silu(xs)
    for x, y in zip(xs, mine):
        assert abs(y - x / (1.0 + math.exp(-x))) <= 1e-15 * max(1.0, abs(x))
    lib = torch.nn.functional.silu(torch.from_numpy(xs)).numpy()
    np.testing.assert_allclose(mine, lib, rtol=1e-14, atol=1e-15)


# ---- RMS norm ------------------------------------------------------------------------------------

def test_rms_norm_constant_row_and_unit_rms():
    K = 256
    g = np.ones(K, dtype=np.float16)
    x = np.full((1, K), 3.0, dtype=np.float16)
    y64, y16 = R.rms_norm(x, g, 0.0)
    np.testing.assert_allclose(y64, 1.0, rtol=1e-15)
    y64, _ = R.rms_norm(-x, g, 0.0)
    np.testing.assert_allclose(y64, -1.0, rtol=1e-15)
    # eps: c / sqrt(c^2 + eps)
    y64, _ = R.rms_norm(x, g, 7.0)
    np.testing.assert_allclose(y64, 3.0 / 4.0, rtol=1e-15)
    x = I.make_hidden(3, 5, K)
    y64, _ = R.rms_norm(x, g, 0.0)
    np.testing.assert_allclose(np.sqrt((y64 ** 2).mean(axis=1)), 1.0, rtol=1e-13)


def test_rms_norm_scale_invariance_and_gamma():
    K = 512
    x = I.make_hidden(4, 3, K)
    g = I.make_gamma(5, K)
    a, _ = R.rms_norm(x, g, 0.0)
    b, _ = R.rms_norm((x.astype(np.float32) * 4).astype(np.float16), g, 0.0)   # power of two: exact in fp16
    np.testing.assert_allclose(a, b, rtol=1e-14)
    ones, _ = R.rms_norm(x, np.ones(K, dtype=np.float16), 0.0)
    np.testing.assert_allclose(a, ones * g.astype(np.float64)[None, :], rtol=1e-14)
    # a single non-zero element: y_j = gamma_j v / sqrt(v^2 / K + eps)
    x1 = np.zeros((1, K), dtype=np.float16)
    x1[0, 17] = -2.5
    y, _ = R.rms_norm(x1, g, 1e-5)
    want = float(g[17]) * -2.5 / math.sqrt(2.5 * 2.5 / K + 1e-5)
    assert abs(y[0, 17] - want) < 1e-12 and np.count_nonzero(y) == 1


def test_rms_norm_against_torch():
    K = 1024
    x = I.make_hidden(6, 7, K)
    g = I.make_gamma(7, K)
    y64, y16 = R.rms_norm(x, g, 1e-5)
    lib = torch.nn.functional.rms_norm(torch.from_numpy(x.astype(np.float64)), (K,),
                                       torch.from_numpy(g.astype(np.float64)), 1e-5).numpy()
    np.testing.assert_allclose(y64, lib, rtol=1e-12)
    assert y16.dtype == np.float16 and np.array_equal(y16, lib.astype(np.float16))


# ---- epilogues of the linear ---------------------------------------------------------------------

def one_hot_x(rows, K):
    x = np.zeros((len(rows), K), dtype=np.float16)
    for m, (k, val) in enumerate(rows):
        x[m, k] = val
    return x


def test_residual_epilogue_one_hot_and_zero():
    K, N = 256, 64
    inp = I.make_linear(11, 3, K, N)
    W = R.dequant(inp.qweight, inp.scales, inp.qzeros)          # pinned elsewhere
    r = I.make_hidden(12, 3, N, 0)
    y64, y16 = R.w4a16_gemm_residual(np.zeros((3, K), dtype=np.float16), inp.qweight, inp.scales, inp.qzeros, r)
    assert np.array_equal(y16, r)
    rows = [(5, 1.0), (130, -2.0), (255, 0.5)]
    y64, _ = R.w4a16_gemm_residual(one_hot_x(rows, K), inp.qweight, inp.scales, inp.qzeros, r)
    for m, (k, val) in enumerate(rows):
        for n in range(N):
            assert y64[m, n] == float(r[m, n]) + val * float(W[k, n])


def test_silu_mul_epilogue_one_hot():
    K, N = 256, 96
    inp = I.make_linear(13, 2, K, N)
    W = R.dequant(inp.qweight, inp.scales, inp.qzeros)
    rows = [(77, 24.0), (200, -16.0)]
    y64, y16 = R.w4a16_gemm_silu_mul(one_hot_x(rows, K), inp.qweight, inp.scales, inp.qzeros)
    assert y64.shape == (2, N // 2)
    for m, (k, val) in enumerate(rows):
        for n in range(N // 2):
            g, u = val * float(W[k, n]), val * float(W[k, N // 2 + n])
            want = g / (1.0 + math.exp(-g)) * u          # gate is the FIRST half, up the second
            assert abs(y64[m, n] - want) <= 1e-14 * max(1.0, abs(want))
    assert np.array_equal(y16, y64.astype(np.float16))
    # the two halves are not interchangeable on this input
    swapped = R.silu(y64 * 0 + np.array([[val * float(W[k, N // 2 + n]) for n in range(N // 2)] for k, val in rows])) * \
        np.array([[val * float(W[k, n]) for n in range(N // 2)] for k, val in rows])
    assert np.abs(swapped - y64).max() > 1e-3


# ---- rotary embedding and append -----------------------------------------------------------------

def rope_case(seed, M=5, Hq=4, Hkv=2, D=16, P=3, n_pos=64):
    rng = np.random.default_rng(seed)
    qkv = rng.standard_normal((M, (Hq + 2 * Hkv) * D), dtype=np.float32).astype(np.float16)
    pos = rng.integers(0, n_pos, size=M).astype(np.int32)
    cos, sin = I.make_rope_tables(n_pos, D)
    kc = rng.standard_normal((P + M + 2, Hkv, D), dtype=np.float32).astype(np.float16)
    vc = rng.standard_normal((P + M + 2, Hkv, D), dtype=np.float32).astype(np.float16)
    return qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D


def test_rope_tables():
    cos, sin = I.make_rope_tables(32, 8, base=10000.0)
    assert cos.shape == (32, 4) and np.all(cos[0] == 1) and np.all(sin[0] == 0)
    for p in (1, 7, 31):
        for i in range(4):
            ang = p * 10000.0 ** (-2.0 * i / 8)
            assert abs(float(cos[p, i]) - math.cos(ang)) < 1e-7 and abs(float(sin[p, i]) - math.sin(ang)) < 1e-7


def test_rope_position_zero_is_identity_and_values_are_copied():
    qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D = rope_case(21)
    pos[:] = 0
    q64, q16, k2, v2 = R.rope_append(qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    M = qkv.shape[0]
    a = qkv.reshape(M, Hq + 2 * Hkv, D)
    assert np.array_equal(q16, a[:, :Hq]) and np.array_equal(k2[P:P + M], a[:, Hq:Hq + Hkv])
    assert np.array_equal(v2[P:P + M], a[:, Hq + Hkv:])
    assert np.array_equal(k2[:P], kc[:P]) and np.array_equal(k2[P + M:], kc[P + M:])
    assert np.array_equal(v2[:P], vc[:P]) and np.array_equal(v2[P + M:], vc[P + M:])


def test_rope_element_by_element_with_python_floats():
    qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D = rope_case(22)
    q64, _, k2, _ = R.rope_append(qkv, pos, cos, sin, kc, vc, P, Hq, Hkv, D)
    M, h = qkv.shape[0], D // 2
    for m in range(M):
        for head in range(Hq + Hkv):
            for i in range(h):
                lo, hi = float(qkv[m, head * D + i]), float(qkv[m, head * D + i + h])
                c, s = float(cos[pos[m], i]), float(sin[pos[m], i])
                w_lo, w_hi = lo * c - hi * s, hi * c + lo * s
                if head < Hq:
                    assert abs(q64[m, head, i] - w_lo) < 1e-14 and abs(q64[m, head, i + h] - w_hi) < 1e-14
                else:
                    assert k2[P + m, head - Hq, i] == np.float16(w_lo) and k2[P + m, head - Hq, i + h] == np.float16(w_hi)


def test_rope_is_a_rotation_and_dot_products_depend_on_position_difference():
    D, n_pos = 32, 128
    cos, sin = I.make_rope_tables(n_pos, D)
    rng = np.random.default_rng(23)
    a = rng.standard_normal(D).astype(np.float16)
    b = rng.standard_normal(D).astype(np.float16)
    z = np.zeros(D, dtype=np.float16)
    kc = np.zeros((2, 1, D), dtype=np.float16)

    def rotated(vec, p):
        row = np.concatenate([vec, z, z])[None, :]               # one q head, one k head, one v head
        q64, *_ = R.rope_append(row, np.array([p]), cos, sin, kc, kc, 0, 1, 1, D)
        return q64[0, 0]

    assert abs(np.linalg.norm(rotated(a, 37)) - np.linalg.norm(a.astype(np.float64))) < 1e-6
    d0 = rotated(a, 10) @ rotated(b, 4)
    d1 = rotated(a, 90) @ rotated(b, 84)
    assert abs(d0 - d1) < 1e-5 * (1 + abs(d0))                   # tables are fp32
    assert abs(d0 - rotated(a, 11) @ rotated(b, 4)) > 1e-3       # and it does depend on the difference


def test_tree_positions():
    parent = np.array([-1, 0, 0, 1, 3, 2])
    assert I.tree_positions(parent, 100).tolist() == [100, 101, 101, 102, 103, 102]
