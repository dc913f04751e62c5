"""Pins for the oracle's Algorithm 1 (best-first heap) and ancestor mask.

Proposition 2: the result is the N highest-probability prefixes.  Proposition 1: the
surrogate objective equals the sum of prefix masses.  Proof of Proposition 3: pops are
non-increasing, every tuple has a unique predecessor, the tree is prefix-closed."""
import itertools

import numpy as np
import pytest

import oracle
from tests import golden_io


def _lp_rows(rng, B, K, dyadic=False):
    """Rank-ordered log-prob rows (non-increasing), fp32."""
    if dyadic:
        rows = -np.sort(rng.integers(0, 12, size=(B, K)), axis=1) / 8.0
        return rows.astype(np.float32)
    logits = rng.standard_normal((B, K)) * 1.5
    lp = logits - np.log(np.exp(logits).sum(axis=1, keepdims=True))
    return (-np.sort(-lp, axis=1)).astype(np.float32)


def _brute_force(lp, B, K):
    """All rank tuples of length <= B with fp32 left-fold scores, in the canonical order:
    score descending, then lexicographic rank tuple (a prefix before its extensions)."""
    items = []
    for d in range(1, B + 1):
        for rho in itertools.product(range(K), repeat=d):
            s = np.float32(0.0)
            for i, r in enumerate(rho):
                s = np.float32(s + lp[i, r])
            items.append((-float(s), rho))
    items.sort()
    return items


def _tuples_of(tree):
    """Rank tuple of every node, from the parent links."""
    tup = {0: ()}
    for i in range(1, tree["n_nodes"] + 1):
        tup[i] = tup[int(tree["parent"][i])] + (int(tree["rank"][i]),)
    return tup


@pytest.mark.parametrize("B,K,dyadic", [(1, 6, False), (2, 5, False), (3, 4, False), (4, 3, False),
                                        (4, 2, False), (3, 4, True), (4, 3, True), (2, 6, True)])
def test_brute_force_order_and_set(B, K, dyadic):
    rng = np.random.default_rng(100 * B + K + (7 if dyadic else 0))
    for trial in range(4):
        lp = _lp_rows(rng, B, K, dyadic)
        tok = np.arange(B * K, dtype=np.int32).reshape(B, K)
        order = _brute_force(lp, B, K)
        total = len(order)
        for N in sorted({1, 2, total // 3 + 1, total - 1, total}):
            if N < 1:
                continue
            tree = oracle.build_tree(tok, lp, N, root_token=999)
            assert tree["n_nodes"] == N
            tup = _tuples_of(tree)
            got = [tup[i] for i in range(1, N + 1)]
            want = [rho for _, rho in order[:N]]
            assert got == want, (B, K, dyadic, trial, N)
            for i in range(1, N + 1):
                assert tree["score"][i] == np.float32(-order[i - 1][0])
                d = len(tup[i])
                assert tree["depth"][i] == d
                assert tree["tokens"][i] == tok[d - 1, tup[i][-1]]


def test_heap_runs_dry_when_fewer_prefixes_than_budget():
    rng = np.random.default_rng(5)
    lp = _lp_rows(rng, 2, 2)
    tok = np.arange(4, dtype=np.int32).reshape(2, 2)
    tree = oracle.build_tree(tok, lp, 10)
    assert tree["n_nodes"] == 6  # 2 + 4 prefixes exist
    assert np.all(tree["parent"][7:] == -1) and np.all(tree["tokens"][7:] == -1)
    assert np.all(tree["depth"][7:] == -1)


def test_proposition_1_objective_equals_sum_of_prefix_masses():
    rng = np.random.default_rng(11)
    B, V = 3, 4
    logits = (rng.standard_normal((B, V)) * 1.5).astype(np.float32)
    tok, lp = oracle.topk(logits, V)
    q = np.exp(logits.astype(np.float64))
    q /= q.sum(axis=1, keepdims=True)
    for N in (1, 3, 7, 15, 40):
        tree = oracle.build_tree(tok, lp, N)
        nodes = set()
        toks_of = {0: ()}
        for i in range(1, tree["n_nodes"] + 1):
            toks_of[i] = toks_of[int(tree["parent"][i])] + (int(tree["tokens"][i]),)
            nodes.add(toks_of[i])
        expect = 0.0
        for y in itertools.product(range(V), repeat=B):
            Q = np.prod([q[i, y[i]] for i in range(B)])
            alpha = 0
            for d in range(1, B + 1):
                if tuple(y[:d]) in nodes:
                    alpha = d
                else:
                    break
            expect += Q * alpha
        got = np.exp(tree["score"][1:tree["n_nodes"] + 1].astype(np.float64)).sum()
        assert abs(got - expect) < 1e-5


def _check_invariants(tree, tok, lp, B, K, N):
    n = tree["n_nodes"]
    par, dep, rk, sc = tree["parent"], tree["depth"], tree["rank"], tree["score"]
    assert par[0] == -1 and dep[0] == 0
    seen = set()
    for i in range(1, n + 1):
        p = int(par[i])
        assert 0 <= p < i                       # prefix-closed, parents first
        assert dep[i] == dep[p] + 1 <= B
        assert 0 <= rk[i] < K
        assert (p, int(rk[i])) not in seen      # each tuple generated once
        seen.add((p, int(rk[i])))
        if rk[i] > 0:                           # predecessor (previous sibling) already popped
            assert (p, int(rk[i]) - 1) in seen
        assert sc[i] == np.float32(sc[p] + lp[dep[i] - 1, rk[i]])
        assert tree["tokens"][i] == tok[dep[i] - 1, rk[i]]
        if i > 1:
            assert sc[i] <= sc[i - 1]           # pops non-increasing
    assert tree["max_heap"] <= N + 1            # heap stays O(N)


def test_invariants_and_budget_nesting_on_workload_like_input():
    import ddtree_inputs as di
    logits = di.draft_logits(di.config_seed(1), 8, 1024)
    K = 64
    tok, lp = oracle.topk(logits, K)
    big = oracle.build_tree(tok, lp, 64)
    _check_invariants(big, tok, lp, 8, K, 64)
    for N in (1, 5, 16, 33):
        small = oracle.build_tree(tok, lp, N)
        _check_invariants(small, tok, lp, 8, K, N)
        for key in ("tokens", "parent", "depth", "rank", "score"):
            assert np.array_equal(small[key], big[key][:N + 1])


def test_special_shapes_chain_and_star():
    B, K = 6, 8
    tok = np.arange(B * K, dtype=np.int32).reshape(B, K) + 1000
    # sharply peaked rows, N <= B: the single trajectory of top-1 tokens (vanilla block draft)
    lp = np.full((B, K), -20.0, np.float32)
    lp[:, 0] = -0.01
    tree = oracle.build_tree(tok, lp, 5)
    assert tree["parent"].tolist() == [-1, 0, 1, 2, 3, 4]
    assert tree["tokens"][1:].tolist() == [1000 + K * d for d in range(5)]
    # N = 1: the single node is the top-1 token of the first position
    one = oracle.build_tree(tok, lp, 1)
    assert one["tokens"].tolist() == [0, 1000] and one["parent"].tolist() == [-1, 0]
    # flat first row whose last rank still beats any depth-2 prefix: a star
    lp2 = np.full((B, K), -3.0, np.float32)
    lp2[0] = -np.linspace(1.0, 1.7, K).astype(np.float32)
    star = oracle.build_tree(tok, lp2, K)
    assert star["parent"][1:].tolist() == [0] * K
    assert star["rank"][1:].tolist() == list(range(K))


def test_hand_worked_tree():
    g = golden_io.load(golden_io.path("w1_tree.txt"))
    lp = np.array(g["lp"], np.float32)
    tok = np.array(g["tok"], np.int32)
    tree = oracle.build_tree(tok, lp, 9, root_token=7)
    for key in ("parent", "depth", "rank", "tokens"):
        assert tree[key].tolist() == g[key], key
    assert tree["score"].tolist() == g["score"]
    six = oracle.build_tree(tok, lp, 6, root_token=7)
    mask = oracle.ancestor_mask(six["parent"], six["n_nodes"])
    assert mask[:, 0].tolist() == g["mask6"]
    obj = np.exp(six["score"][1:].astype(np.float64)).sum()
    assert abs(obj - g["objective6"][0]) < 2e-6
    tie = oracle.build_tree(tok, np.array(g["tie_lp"], np.float32), 6, root_token=7)
    for key in ("parent", "depth", "rank"):
        assert tie[key].tolist() == g["tie_" + key], key
    assert tie["score"].tolist() == g["tie_score"]


def test_mask_closed_forms():
    n = 70  # spans two 64-bit words
    chain = np.arange(-1, n, dtype=np.int32)
    m = oracle.ancestor_mask(chain, n)
    assert m.shape == (n + 1, 2)
    for i in range(n + 1):
        bits = [(int(m[i, j >> 6]) >> (j & 63)) & 1 for j in range(n + 1)]
        assert bits == [1] * (i + 1) + [0] * (n - i)       # lower triangular
    star = np.zeros(n + 1, np.int32)
    star[0] = -1
    m = oracle.ancestor_mask(star, n)
    for i in range(1, n + 1):
        want = [0, 0]
        want[0] |= 1
        want[i >> 6] |= 1 << (i & 63)
        assert [int(m[i, 0]), int(m[i, 1])] == want
    # padding rows are zero, popcount = depth + 1, child row contains parent row
    rng = np.random.default_rng(3)
    par = np.full(100, -1, np.int32)
    dep = np.zeros(100, np.int64)
    for i in range(1, 80):
        par[i] = rng.integers(0, i)
        dep[i] = dep[par[i]] + 1
    m = oracle.ancestor_mask(par, 79, T=100)
    assert not m[80:].any()
    for i in range(80):
        assert sum(bin(int(w)).count("1") for w in m[i]) == dep[i] + 1
        if i:
            assert all(int(m[par[i], w]) & ~int(m[i, w]) == 0 for w in range(2))
