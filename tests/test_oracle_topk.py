"""Pins for the oracle's log-softmax + rank ordering (paper Section 4.3: q_i = softmax(l_i),
tokens ordered by q_i descending, sigma built from log q)."""
import numpy as np
import torch

import oracle


def _rand_logits(seed, B, V, scale=2.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, V)) * scale).astype(np.float32)


def test_matches_library_log_softmax_and_full_sort():
    x = _rand_logits(0, 5, 257)
    tok, lp = oracle.topk(x, 257)
    ref = torch.log_softmax(torch.from_numpy(x).double(), dim=-1)
    vals, idx = torch.sort(torch.from_numpy(x), dim=-1, descending=True, stable=True)
    assert np.array_equal(tok, idx.numpy().astype(np.int32))
    ref_lp = torch.gather(ref, 1, idx).numpy()
    assert np.max(np.abs(lp.astype(np.float64) - ref_lp)) < 1e-6


def test_probabilities_sum_to_one_when_K_equals_V():
    x = _rand_logits(1, 4, 1000, scale=3.0)
    _, lp = oracle.topk(x, 1000)
    s = np.exp(lp.astype(np.float64)).sum(axis=1)
    assert np.all(np.abs(s - 1.0) < 1e-6)


def test_prefix_property_in_K():
    x = _rand_logits(2, 3, 500)
    tok_full, lp_full = oracle.topk(x, 500)
    tok, lp = oracle.topk(x, 37)
    assert np.array_equal(tok, tok_full[:, :37])
    assert np.array_equal(lp, lp_full[:, :37])


def test_shift_invariance():
    x = _rand_logits(3, 4, 300)
    tok0, lp0 = oracle.topk(x, 50)
    tok1, lp1 = oracle.topk((x + np.float32(8.0)).astype(np.float32), 50)
    # adding 8.0 is exact for |x| < 2**20 up to the fp32 rounding of x + 8 itself; ranks by
    # logit can only change where two logits round together, so compare probabilities
    assert np.max(np.abs(lp0 - lp1)) < 5e-6
    same = tok0 == tok1
    assert same.mean() > 0.98


def test_uniform_row_closed_form_and_tie_order():
    V = 64
    x = np.full((2, V), 1.25, np.float32)
    tok, lp = oracle.topk(x, 10)
    assert np.array_equal(tok, np.tile(np.arange(10, dtype=np.int32), (2, 1)))
    assert np.allclose(lp, -np.log(V), atol=1e-7)


def test_duplicates_straddling_the_K_boundary():
    # five tokens share the 3rd-largest logit; K cuts through them: lower ids win
    x = np.zeros((1, 20), np.float32)
    x[0, 7] = 5.0
    x[0, 2] = 4.0
    for t in (15, 3, 11, 9, 18):
        x[0, t] = 3.0
    tok, lp = oracle.topk(x, 5)
    assert tok[0].tolist() == [7, 2, 3, 9, 11]
    assert lp[0, 2] == lp[0, 3] == lp[0, 4]
    assert np.all(np.diff(lp[0]) <= 0)


def test_lse_matches_scipy():
    from scipy.special import logsumexp
    x = _rand_logits(5, 6, 4096, scale=4.0)
    _, _, lse = oracle.topk(x, 1, return_lse=True)
    ref = logsumexp(x.astype(np.float64), axis=1)
    assert np.max(np.abs(lse - ref)) < 1e-10


def test_dominant_token_gives_zero_logprob():
    x = np.full((1, 100), -200.0, np.float32)
    x[0, 42] = 50.0
    tok, lp = oracle.topk(x, 3)
    assert tok[0, 0] == 42 and lp[0, 0] == 0.0
    assert tok[0, 1] == 0 and tok[0, 2] == 1 and lp[0, 1] == -250.0


def test_nearly_certain_token_closed_form():
    """One logit c above V - 1 zeros: log q of the top token is -log1p((V - 1) e^-c) and of the
    others -c - log1p((V - 1) e^-c); the first is far below one ulp of the row's log-sum-exp, so a
    formulation that subtracts the log-sum-exp from the logit gets it wrong by many ulps."""
    import math
    from fractions import Fraction

    for V, c in ((7, 25.0), (64, 25.0), (1000, 25.0), (1000, 12.0), (151936, 30.0)):
        x = np.zeros((1, V), np.float32)
        x[0, V // 3] = c
        tok, lp = oracle.topk(x, 2)
        # log1p(t) for tiny t by its alternating series in exact rationals (t < 1e-2: 12 terms
        # leave < 1e-26 relative), with e^-c itself from math.exp (relative error < 1e-16)
        t = Fraction(V - 1) * Fraction(math.exp(-c))
        series = sum(Fraction((-1) ** (j + 1), j) * t**j for j in range(1, 13))
        top = np.float32(-float(series))
        assert tok[0, 0] == V // 3 and tok[0, 1] == 0
        assert abs(int(lp[0, 0].view(np.int32)) - int(top.view(np.int32))) <= 1, (V, c, lp[0, 0], top)
        assert lp[0, 1] == np.float32(-c - float(series))
