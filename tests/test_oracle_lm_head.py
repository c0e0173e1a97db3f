"""Pins of the oracle's draft-side LM head (logits, log-softmax, top-k)."""
import math

import numpy as np
import torch

from oracle import reference as R
from paper_2505_22179_amd import inputs as I


def test_one_hot_hidden_state_reads_a_weight_column():
    x, W = I.make_lm_head(1, 2, 32, 50)
    x[:] = 0
    x[0, 5] = 2.0
    x[1, 31] = -1.0
    logits, idx, lp = R.lm_head_topk(x, W, 3)
    for v in range(50):
        assert logits[0, v] == 2.0 * float(W[v, 5]) and logits[1, v] == -float(W[v, 31])
    col = [2.0 * float(W[v, 5]) for v in range(50)]
    want = sorted(range(50), key=lambda v: (-col[v], v))[:3]
    assert idx[0].tolist() == want
    lse = math.log(sum(math.exp(c) for c in col))
    for j, v in enumerate(want):
        assert abs(lp[0, j] - (col[v] - lse)) < 1e-12


def test_planted_winners_and_order():
    x, W = I.make_lm_head(2, 3, 64, 400)
    W = W.astype(np.float32)
    # token 123 aligned with row 0's hidden state, token 7 a little less, token 300 opposed
    W[123] = x[0].astype(np.float32) * 0.5
    W[7] = x[0].astype(np.float32) * 0.25
    W[300] = -x[0].astype(np.float32)
    W = W.astype(np.float16)
    logits, idx, lp = R.lm_head_topk(x, W, 2)
    assert idx[0].tolist() == [123, 7]
    assert np.argmin(logits[0]) == 300
    assert lp[0, 0] > lp[0, 1] and (lp <= 0).all()


def test_probabilities_sum_to_one_and_uniform_case():
    x, W = I.make_lm_head(3, 4, 32, 97)
    logits, idx, lp = R.lm_head_topk(x, W, 97)          # all tokens
    np.testing.assert_allclose(np.exp(lp).sum(axis=1), 1.0, rtol=1e-12)
    assert all(sorted(idx[m].tolist()) == list(range(97)) for m in range(4))
    assert (np.diff(lp, axis=1) <= 0).all()
    # zero hidden state: all logits 0, uniform distribution, ties resolved by ascending token index
    x0 = np.zeros((1, 32), dtype=np.float16)
    _, idx0, lp0 = R.lm_head_topk(x0, W, 5)
    assert idx0[0].tolist() == [0, 1, 2, 3, 4]
    np.testing.assert_allclose(lp0, -math.log(97), rtol=1e-14)


def test_ties_take_the_lower_token_first():
    x, W = I.make_lm_head(4, 1, 16, 40)
    W[30] = W[9]
    W[21] = W[9]
    x[0] = W[9] * np.float16(40)         # make token 9 (and its copies) the clear winners
    _, idx, lp = R.lm_head_topk(x, W, 4)
    assert idx[0, :3].tolist() == [9, 21, 30] and lp[0, 0] == lp[0, 1] == lp[0, 2]


def test_against_torch():
    x, W = I.make_lm_head(5, 6, 128, 1000)
    logits, idx, lp = R.lm_head_topk(x, W, 10)
    tl = torch.from_numpy(x.astype(np.float64)) @ torch.from_numpy(W.astype(np.float64)).T
    np.testing.assert_allclose(logits, tl.numpy(), rtol=1e-12, atol=1e-12)
    tlp = torch.log_softmax(tl, dim=1)
    tv, ti = torch.topk(tlp, 10, dim=1)
    assert np.array_equal(idx, ti.numpy())               # no ties in these random logits
    np.testing.assert_allclose(lp, tv.numpy(), rtol=1e-12, atol=1e-12)


def test_large_logits_do_not_overflow():
    x = np.full((1, 8), 100.0, dtype=np.float16)
    W = np.zeros((3, 8), dtype=np.float16)
    W[1] = 10.0                                          # logit 8000: exp would overflow without the max shift
    logits, idx, lp = R.lm_head_topk(x, W, 2)
    assert idx[0, 0] == 1 and abs(lp[0, 0]) < 1e-12 and np.isfinite(lp).all()
