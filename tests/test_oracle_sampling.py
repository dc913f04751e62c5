"""Pins of the oracle's temperature-sampling selection (paper Section 4.4, second paragraph:
verification follows the target's decoding rule, greedy or temperature-based sampling).

The selection is argmax_v(logit/tau + Gumbel noise) with noise from a counter-based generator.
Nothing here calls the HIP library."""
import numpy as np
import pytest

import oracle


def test_uniforms_lie_strictly_inside_the_unit_interval_and_look_uniform():
    u = np.array([oracle.sample_uniform(123456789, r, v) for r in range(40) for v in range(500)])
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 - 0.5 == np.round(u * 2 ** 24 - 0.5))      # 24-bit grid, centred
    hist, _ = np.histogram(u, bins=20, range=(0, 1))
    expect = len(u) / 20
    chi2 = ((hist - expect) ** 2 / expect).sum()
    assert chi2 < 60.0                                                     # 19 dof: P(chi2 > 60) ~ 4e-6
    # rows, tokens and seeds all change the draw
    assert oracle.sample_uniform(1, 0, 0) != oracle.sample_uniform(1, 1, 0)
    assert oracle.sample_uniform(1, 0, 0) != oracle.sample_uniform(1, 0, 1)
    assert oracle.sample_uniform(1, 0, 0) != oracle.sample_uniform(2, 0, 0)
    assert oracle.sample_uniform(1, 0, 0) != oracle.sample_uniform(1 + (1 << 32), 0, 0)


def test_samples_follow_softmax_of_logits_over_temperature():
    # Gumbel-max samples exactly from softmax(logits / tau): 30000 rows with the same logits
    # (the row index changes the noise) against the closed-form probabilities
    logits = np.array([1.0, 0.0, -1.0, 2.0, 0.5], np.float32)
    T = 30000
    x = np.tile(logits, (T, 1))
    for tau in (0.7, 1.0, 2.5):
        tok, run, gap = oracle.sample_tokens(x, T - 1, tau, seed=99)
        p = np.exp(logits / tau)
        p /= p.sum()
        freq = np.bincount(tok, minlength=5) / T
        sigma = np.sqrt(p * (1 - p) / T)
        assert np.all(np.abs(freq - p) < 4.5 * sigma), (tau, freq, p)
        assert np.all(gap >= 0) and np.all(run != tok)


def test_small_temperature_is_greedy_and_constant_shift_changes_nothing():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((50, 300)).astype(np.float32)
    x[7, 3] = x[7].max() + 1.0
    tok, _, _ = oracle.sample_tokens(x, 49, 1e-4, seed=3)
    srt = np.sort(x, axis=1)
    clear = srt[:, -1] - srt[:, -2] > 0.01            # gap / tau > 100 dwarfs any Gumbel difference
    assert clear.sum() > 25
    assert np.array_equal(tok[clear], x.argmax(axis=1)[clear])
    a, _, _ = oracle.sample_tokens(x, 49, 0.9, seed=8)
    b, _, _ = oracle.sample_tokens(x + np.float32(4.0), 49, 0.9, seed=8)   # exact fp32 shift for |x| < 4
    agree = np.mean(a == b)
    assert agree > 0.97                               # only rounding of x + 4 can move a near-tie
    c, _, _ = oracle.sample_tokens(x, 49, 0.9, seed=9)
    assert np.mean(a == c) < 0.5                      # a different seed is a different draw


def test_rows_past_the_tree_are_skipped_and_first_row_offsets_the_stream():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((10, 64)).astype(np.float32)
    tok, run, gap = oracle.sample_tokens(x, 5, 1.0, seed=4)
    assert np.all(tok[6:] == -1) and np.all(tok[:6] >= 0)
    # rows 3.. of one call equal rows 0.. of a call that starts its stream at row 3
    t2, _, _ = oracle.sample_tokens(x[3:], 6, 1.0, seed=4, first_row=3)
    assert np.array_equal(t2[:3], tok[3:6])


def test_walk_follows_the_selected_tokens_figure_1b():
    # the tree of Figure 1: a root with children b, c; b has d, e; c has f; d has g, h; e has i
    parent = np.array([-1, 0, 0, 1, 1, 2, 3, 3, 4], np.int32)
    tokens = np.array([10, 11, 12, 13, 14, 15, 16, 17, 18], np.int32)
    selected = np.array([11, 14, 0, 0, 99, 0, 0, 0, 0], np.int32)    # a -> b -> e -> (99: no child)
    r = oracle.walk(selected, tokens, parent, 8, 4)
    assert r["n_accepted"] == 2 and list(r["path"][:3]) == [0, 1, 4] and r["bonus"] == 99
    # nothing matches at the root: the bonus is the root's own selection
    r = oracle.walk(np.array([77] * 9, np.int32), tokens, parent, 8, 4)
    assert r["n_accepted"] == 0 and r["bonus"] == 77
    # the greedy walk is the same walk fed with row-wise argmaxes
    rng = np.random.default_rng(2)
    tl = rng.standard_normal((9, 40)).astype(np.float32)
    g = oracle.accept(tl, tokens % 40, parent, 8, 4)
    w = oracle.walk(g["posterior"], tokens % 40, parent, 8, 4)
    assert w["n_accepted"] == g["n_accepted"] and w["bonus"] == g["bonus"]
    assert np.array_equal(w["path"], g["path"])
