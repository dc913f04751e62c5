"""Pins for the oracle's greedy verifier walk and cache compaction (paper Section 4.4,
Figure 1b)."""
import numpy as np

import oracle
from tests import golden_io


def _logits_with_argmax(post, V, rng):
    x = rng.standard_normal((len(post), V)).astype(np.float32)
    for i, t in enumerate(post):
        if t >= 0:
            x[i, t] = 20.0
    return x


def test_figure_1_walk():
    g = golden_io.load(golden_io.path("fig1_walk.txt"))
    rng = np.random.default_rng(0)
    x = _logits_with_argmax(g["posterior"], 256, rng)
    r = oracle.accept(x, g["tokens"], g["parent"], 8, B=3)
    assert r["posterior"].tolist() == g["posterior"]
    assert r["n_accepted"] == g["expect_n_accepted"][0]
    assert r["path"].tolist() == g["expect_path"] + [-1]
    assert r["bonus"] == g["expect_bonus"][0]


def test_chain_fully_accepted_and_nothing_accepted():
    rng = np.random.default_rng(1)
    n, V = 5, 64
    parent = np.arange(-1, n, dtype=np.int32)
    tokens = np.array([9, 10, 11, 12, 13, 14], np.int32)
    post = [10, 11, 12, 13, 14, 33]
    r = oracle.accept(_logits_with_argmax(post, V, rng), tokens, parent, n, B=5)
    assert r["n_accepted"] == 5 and r["path"].tolist() == [0, 1, 2, 3, 4, 5] and r["bonus"] == 33
    post = [50, 11, 12, 13, 14, 33]
    r = oracle.accept(_logits_with_argmax(post, V, rng), tokens, parent, n, B=5)
    assert r["n_accepted"] == 0 and r["path"].tolist() == [0, -1, -1, -1, -1, -1]
    assert r["bonus"] == 50
    # a break in the middle
    post = [10, 11, 40, 13, 14, 33]
    r = oracle.accept(_logits_with_argmax(post, V, rng), tokens, parent, n, B=5)
    assert r["n_accepted"] == 2 and r["bonus"] == 40


def test_argmax_tie_goes_to_lower_id():
    x = np.zeros((2, 32), np.float32)
    x[0, [5, 17, 30]] = 3.0
    x[1, [31]] = 1.0
    parent = np.array([-1, 0], np.int32)
    tokens = np.array([0, 17], np.int32)
    r = oracle.accept(x, tokens, parent, 1, B=4)
    assert r["posterior"].tolist() == [5, 31]
    assert r["n_accepted"] == 0 and r["bonus"] == 5


def test_sibling_with_matching_token_under_another_parent_is_not_taken():
    # node 2 carries the right token but hangs under node 1, not under the root
    parent = np.array([-1, 0, 1, 0], np.int32)
    tokens = np.array([1, 2, 7, 3], np.int32)
    rng = np.random.default_rng(2)
    r = oracle.accept(_logits_with_argmax([7, 7, 0, 0], 16, rng), tokens, parent, 3, B=2)
    assert r["n_accepted"] == 0 and r["bonus"] == 7
    r = oracle.accept(_logits_with_argmax([2, 7, 5, 0], 16, rng), tokens, parent, 3, B=2)
    assert r["path"].tolist() == [0, 1, 2] and r["bonus"] == 5


def test_padding_rows_ignored():
    parent = np.array([-1, 0, -1, -1], np.int32)
    tokens = np.array([1, 2, -1, -1], np.int32)
    rng = np.random.default_rng(3)
    r = oracle.accept(_logits_with_argmax([2, 9, 3, 3], 16, rng), tokens, parent, 1, B=2)
    assert r["posterior"].tolist() == [2, 9, -1, -1]
    assert r["n_accepted"] == 1 and r["bonus"] == 9


def test_compact_appends_accepted_rows():
    rng = np.random.default_rng(4)
    T, Hkv, D, L = 9, 2, 4, 5
    tree_k = rng.standard_normal((T, Hkv, D)).astype(np.float32)
    cache = np.zeros((L + 4, Hkv, D), np.float32)
    cache[:L] = 1.0
    oracle.compact(tree_k, np.array([0, 1, 4, -1], np.int32), 2, cache, L)
    assert np.all(cache[:L] == 1.0)
    assert np.array_equal(cache[L:L + 3], tree_k[[0, 1, 4]])
    assert not cache[L + 3:].any()
