"""Pins for the W4A16 linear-layer oracle (paper section 2.2).  None of these re-types the
oracle's own formula as the expected value: they use hand-written fixtures, exact rational
arithmetic, closed forms, library routines and structural invariants, so that a dropped term,
a wrong sign or index or a transposed operand in the oracle fails at least one of them."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import reference as R
from paper_2505_22179_amd import inputs as I

G = 128


# ---- nibble order and packing axis (hand-written fixture) -------------------------------------

def _fixture_words(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "nibble_order.txt")) if ln.startswith("word")]
    words = np.array([int(r[1], 16) for r in rows], dtype=np.uint32).view(np.int32)
    fields = np.array([[int(v) for v in r[2:10]] for r in rows], dtype=np.uint8)
    return words, fields


def test_unpack_codes_matches_hand_fixture(golden_dir):
    words, fields = _fixture_words(golden_dir)
    # one word per column: qweight [1, ncols]; the 8 fields are 8 consecutive rows k of that column
    q = R.unpack_codes(words.reshape(1, -1))
    assert q.shape == (8, len(words))
    assert np.array_equal(q, fields.T)


def test_unpack_zeros_matches_hand_fixture(golden_dir):
    words, fields = _fixture_words(golden_dir)
    # one word per group row: qzeros [nrows, 1]; the 8 fields are 8 consecutive columns n
    z = R.unpack_zeros(words.reshape(-1, 1))
    assert z.shape == (len(words), 8)
    assert np.array_equal(z, fields)


@pytest.mark.parametrize("kind", ["random", "k_mod_16", "n_mod_16", "one_hot"])
def test_pack_unpack_roundtrip(kind):
    K, N = 256, 48
    rng = np.random.default_rng(3)
    if kind == "random":
        codes = rng.integers(0, 16, (K, N), dtype=np.uint8)
    elif kind == "k_mod_16":
        codes = np.broadcast_to((np.arange(K) % 16).astype(np.uint8)[:, None], (K, N)).copy()
    elif kind == "n_mod_16":
        codes = np.broadcast_to((np.arange(N) % 16).astype(np.uint8)[None, :], (K, N)).copy()
    else:
        codes = np.zeros((K, N), dtype=np.uint8)
        codes[77, 13] = 9
    assert np.array_equal(R.unpack_codes(I.pack_rows(codes)), codes)
    zeros = codes[: K // G * 1 + 5]  # any [R, N] array of nibbles
    assert np.array_equal(R.unpack_zeros(I.pack_cols(zeros)), zeros)


# ---- dequantisation: exactness and sign ------------------------------------------------------

def test_dequant_is_exact_rational():
    inp = I.make_linear(11, 1, 256, 16)
    W = R.dequant(inp.qweight, inp.scales, inp.qzeros, G)
    for k in (0, 1, 7, 8, 127, 128, 200, 255):
        for n in range(16):
            want = (int(inp.codes[k, n]) - int(inp.zeros[k // G, n])) * Fraction(float(inp.scales[k // G, n]))
            assert Fraction(float(W[k, n])) == want


def test_dequant_hand_values():
    # one group, 8 columns; code of row k is k % 16, zero-point of column n is n, scale is 2^-n
    K, N = 128, 8
    codes = np.broadcast_to((np.arange(K) % 16).astype(np.uint8)[:, None], (K, N)).copy()
    zeros = np.arange(N, dtype=np.uint8).reshape(1, N)
    scales = (2.0 ** -np.arange(N)).astype(np.float16).reshape(1, N)
    W = R.dequant(I.pack_rows(codes), scales, I.pack_cols(zeros), G)
    assert W[5, 0] == 5.0 and W[5, 1] == 2.0 and W[5, 3] == 0.25 and W[0, 7] == -7 / 128
    assert W[15, 2] == 13 / 4 and W[16, 2] == -2 / 4


# ---- brute force in exact rational arithmetic ------------------------------------------------

@pytest.mark.parametrize("M,K,N", [(1, 128, 8), (3, 256, 16), (2, 256, 8)])
def test_bruteforce_fractions(M, K, N):
    inp = I.make_linear(100 + M + K + N, M, K, N)
    y32, y64, y16 = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    for m in range(M):
        for n in range(N):
            terms = [Fraction(float(inp.x[m, k])) * (int(inp.codes[k, n]) - int(inp.zeros[k // G, n]))
                     * Fraction(float(inp.scales[k // G, n])) for k in range(K)]
            exact = sum(terms)
            mag = float(sum(abs(t) for t in terms))
            assert abs(float(Fraction(float(y64[m, n])) - exact)) <= 1e-13 * mag + 1e-300
            assert abs(float(Fraction(float(y32[m, n])) - exact)) <= K * 2.0 ** -24 * mag
            # y16 is the correctly rounded fp16 of y32 (numpy's conversion is the library pin)
            assert y16[m, n] == np.float32(y32[m, n]).astype(np.float16)


# ---- closed form for constant codes ------------------------------------------------------------

@pytest.mark.parametrize("c,z0", [(11, 3), (2, 9), (7, 7), (0, 15), (15, 0)])
def test_constant_codes_closed_form(c, z0):
    M, K, N = 4, 512, 24
    rng = np.random.default_rng(c * 16 + z0)
    x = rng.standard_normal((M, K)).astype(np.float16)
    s0 = np.float16(0.00390625)  # 2^-8: keeps the closed form exactly representable
    qw = I.pack_rows(np.full((K, N), c, dtype=np.uint8))
    qz = I.pack_cols(np.full((K // G, N), z0, dtype=np.uint8))
    sc = np.full((K // G, N), s0, dtype=np.float16)
    y32, y64, _ = R.w4a16_gemm(x, qw, sc, qz, G)
    want = (c - z0) * float(s0) * x.astype(np.float64).sum(axis=1)
    assert np.allclose(y64, want[:, None], rtol=1e-13, atol=1e-13)
    assert np.abs(y32 - want[:, None]).max() <= 1e-4
    if c == z0:
        assert not y32.any() and not y64.any()


# ---- invariants ---------------------------------------------------------------------------------

def test_row_independence_bit_exact():
    inp = I.make_linear(21, 5, 384, 40)
    y32, y64, y16 = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    for m in range(5):
        a32, a64, a16 = R.w4a16_gemm(inp.x[m:m + 1], inp.qweight, inp.scales, inp.qzeros, G)
        assert np.array_equal(a32[0], y32[m]) and np.array_equal(a64[0], y64[m])
        assert np.array_equal(a16.view(np.uint16)[0], y16.view(np.uint16)[m])


def test_exact_arithmetic_inputs_are_order_independent():
    # x in {-2..2}, scale 2^-7: every partial sum is a multiple of 2^-7 below 2^17, so fp32
    # accumulation is exact in any order and y32 must equal the integer computation bit for bit
    inp = I.make_linear(31, 6, 1024, 32, x_kind="small_int", scale_kind="pow2")
    y32, y64, y16 = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    d = inp.codes.astype(np.int64) - np.repeat(inp.zeros.astype(np.int64), G, axis=0)
    want = (inp.x.astype(np.int64) @ d).astype(np.float64) / 128.0
    assert np.array_equal(y32.astype(np.float64), want) and np.array_equal(y64, want)


def test_numpy_matmul_special_case():
    inp = I.make_linear(41, 8, 1024, 64)
    y32, y64, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    # independent dense reconstruction (numpy broadcasting, not the oracle's dequant)
    d = inp.codes.astype(np.float64) - np.repeat(inp.zeros.astype(np.float64), G, axis=0)
    W = d * np.repeat(inp.scales.astype(np.float64), G, axis=0)
    lib64 = inp.x.astype(np.float64) @ W
    assert np.abs(y64 - lib64).max() <= 1e-11
    lib32 = inp.x.astype(np.float32) @ W.astype(np.float32)
    assert np.abs(y32 - lib32).max() <= 2e-4
    assert np.abs(y32 - lib64).max() <= 2e-4


def test_column_permutation_equivariance():
    inp = I.make_linear(51, 3, 256, 32)
    perm = np.random.default_rng(0).permutation(32)
    y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    p32, _, _ = R.w4a16_gemm(inp.x, I.pack_rows(inp.codes[:, perm]), inp.scales[:, perm].copy(),
                             I.pack_cols(inp.zeros[:, perm]), G)
    assert np.array_equal(p32, y32[:, perm])


def test_scale_locality_and_doubling():
    inp = I.make_linear(61, 2, 384, 16)
    y32, y64, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    s2 = inp.scales.copy()
    s2[1, 5] = np.float16(float(s2[1, 5]) * 2)
    a32, a64, _ = R.w4a16_gemm(inp.x, inp.qweight, s2, inp.qzeros, G)
    others = np.arange(16) != 5
    assert np.array_equal(a32[:, others], y32[:, others])
    # the change equals group 1's term of column 5 (computed independently in fp64)
    d = inp.codes[128:256, 5].astype(np.float64) - float(inp.zeros[1, 5])
    term = (inp.x[:, 128:256].astype(np.float64) @ d) * float(inp.scales[1, 5])
    assert np.allclose(a64[:, 5] - y64[:, 5], term, rtol=0, atol=1e-12)
    # doubling every scale doubles y exactly (power-of-two factor)
    b32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, (inp.scales.astype(np.float32) * 2).astype(np.float16), inp.qzeros, G)
    assert np.array_equal(b32, 2 * y32)


def test_group_locality_of_x():
    inp = I.make_linear(71, 2, 384, 16)
    _, y64, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    x0 = inp.x.copy()
    x0[:, 128:256] = 0
    _, z64, _ = R.w4a16_gemm(x0, inp.qweight, inp.scales, inp.qzeros, G)
    d = inp.codes[128:256].astype(np.float64) - inp.zeros[1].astype(np.float64)[None, :]
    term = (inp.x[:, 128:256].astype(np.float64) @ d) * inp.scales[1].astype(np.float64)[None, :]
    assert np.allclose(y64 - z64, term, rtol=0, atol=1e-12)


def test_zero_point_moves_output_the_right_way():
    # raising z[g, n] by one lowers y[m, n] by s[g, n] * sum_{k in g} x[m, k] (sign of the zero term)
    inp = I.make_linear(81, 2, 256, 8)
    zeros = inp.zeros.copy()
    zeros[0, 3] = 4
    _, a64, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, I.pack_cols(zeros), G)
    zeros[0, 3] = 5
    _, b64, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, I.pack_cols(zeros), G)
    want = -float(inp.scales[0, 3]) * inp.x[:, :128].astype(np.float64).sum(axis=1)
    assert np.allclose(b64[:, 3] - a64[:, 3], want, rtol=0, atol=1e-12)
    assert np.array_equal(np.delete(b64, 3, axis=1), np.delete(a64, 3, axis=1))


def test_generator_statistics():
    # Var(w) = Var(q - z) * E[s^2] = 42.5 * 3.7e-5 = 1.5725e-3 for the stated distributions
    for K, sigma in ((4096, 2.54), (8192, 3.59)):
        inp = I.make_linear(I.seed_for(1, 0), 8, K, 512)
        y32, _, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G, want64=False)
        assert abs(y32.std() / sigma - 1) < 0.05


def test_symmetric_weight_is_the_mid_code_special_case():
    """A symmetrically quantised weight (paper section 2.2) is the special case zero-point = 8 of the oracle's
    formula: with codes read as signed values q - 8 in -8..7 the weight is (q - 8) * s and the layer is an
    ordinary matmul with that matrix; the mid-code 8 itself is weight 0 whatever the scale."""
    M, K, N = 3, 256, 24
    inp = I.make_linear(4242, M, K, N, zero_kind="eight")
    assert (inp.zeros == 8).all() and (R.unpack_zeros(inp.qzeros) == 8).all()
    W = R.dequant(inp.qweight, inp.scales, inp.qzeros, G)
    signed = inp.codes.astype(np.int64) - 8                       # two's-complement reading of the 4-bit code
    assert signed.min() == -8 and signed.max() == 7
    s64 = np.repeat(inp.scales.astype(np.float64), G, axis=0)
    assert np.array_equal(W.astype(np.float64), signed * s64)     # exact: 4 + 11 significant bits
    assert (W[inp.codes == 8] == 0).all() and (inp.codes == 8).any()
    y32, y64, _ = R.w4a16_gemm(inp.x, inp.qweight, inp.scales, inp.qzeros, G)
    want = inp.x.astype(np.float64) @ (signed * s64)
    assert np.allclose(y64, want, rtol=0, atol=1e-12 * np.abs(want).max())
    assert np.abs(y32 - want).max() <= K * 2.0 ** -24 * (np.abs(inp.x.astype(np.float64)) @ np.abs(signed * s64)).max()
    # the same codes and scales under other zero-points give another answer: the special case is not vacuous
    other = I.make_linear(4242, M, K, N)
    assert np.array_equal(other.qweight, inp.qweight) and np.array_equal(other.scales.view(np.uint16), inp.scales.view(np.uint16))
    assert not np.array_equal(R.w4a16_gemm(other.x, other.qweight, other.scales, other.qzeros, G)[0], y32)
