"""Pins for the oracle's tree attention (paper Section 4.4: a node attends to the cached
context and, inside the tree, only to the root, its ancestors and itself)."""
import numpy as np
import torch

import oracle


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def _random_tree(rng, T):
    par = np.full(T, -1, np.int32)
    for i in range(1, T):
        par[i] = rng.integers(0, i)
    return par


def _dense_visibility(par, L):
    """Boolean [T, L+T] built by an independent ancestor walk (not via the oracle's mask)."""
    T = len(par)
    vis = np.zeros((T, L + T), bool)
    vis[:, :L] = True
    for i in range(T):
        j = i
        while j >= 0:
            vis[i, L + j] = True
            j = par[j]
    return vis


def _sdpa(q, k_cache, v_cache, k_tree, v_tree, vis, scale=None):
    """Library attention in fp64 with an explicit boolean mask (what the paper's target used)."""
    T, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    G = Hq // Hkv
    k = np.concatenate([k_cache, k_tree], axis=0)
    v = np.concatenate([v_cache, v_tree], axis=0)
    qt = torch.from_numpy(q).double().permute(1, 0, 2)                     # [Hq,T,D]
    kt = torch.from_numpy(k).double().permute(1, 0, 2).repeat_interleave(G, dim=0)
    vt = torch.from_numpy(v).double().permute(1, 0, 2).repeat_interleave(G, dim=0)
    m = torch.from_numpy(vis)[None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=m, scale=scale)
    return o.permute(1, 0, 2).numpy()


def test_chain_tree_is_causal_attention():
    rng = np.random.default_rng(0)
    T, L, Hq, Hkv, D = 70, 37, 4, 2, 32
    q, kc, vc, kt, vt = (_rand(rng, T, Hq, D), _rand(rng, L, Hkv, D), _rand(rng, L, Hkv, D),
                         _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D))
    chain = np.arange(-1, T - 1, dtype=np.int32)
    mask = oracle.ancestor_mask(chain, T - 1)
    got = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    # textbook causal attention over the concatenated sequence: the T queries are its last
    # T positions, so query i sees keys 0 .. L+i
    G = Hq // Hkv
    k = np.concatenate([kc, kt]); v = np.concatenate([vc, vt])
    qf = np.concatenate([np.zeros((L, Hq, D), np.float32), q])
    qt_ = torch.from_numpy(qf).double().permute(1, 0, 2)
    kt_ = torch.from_numpy(k).double().permute(1, 0, 2).repeat_interleave(G, dim=0)
    vt_ = torch.from_numpy(v).double().permute(1, 0, 2).repeat_interleave(G, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(qt_, kt_, vt_, is_causal=True)
    ref = ref.permute(1, 0, 2).numpy()[L:]
    assert np.max(np.abs(got - ref)) < 1e-12


def test_random_tree_matches_dense_mask_sdpa():
    rng = np.random.default_rng(1)
    for (T, L, Hq, Hkv, D) in [(17, 128, 2, 1, 64), (130, 5, 8, 2, 16), (66, 0, 3, 3, 8)]:
        par = _random_tree(rng, T)
        q, kc, vc, kt, vt = (_rand(rng, T, Hq, D), _rand(rng, L, Hkv, D), _rand(rng, L, Hkv, D),
                             _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D))
        mask = oracle.ancestor_mask(par, T - 1)
        got = oracle.verify_attn(q, kc, vc, kt, vt, mask)
        ref = _sdpa(q, kc, vc, kt, vt, _dense_visibility(par, L))
        assert np.max(np.abs(got - ref)) < 1e-12
        # the (node, head) pair interface returns the same rows
        pairs = np.array([[T - 1, Hq - 1], [0, 0], [T // 2, 1 % Hq]], np.int32)
        sub = oracle.verify_attn(q, kc, vc, kt, vt, mask, pairs=pairs)
        for r, (i, h) in enumerate(pairs):
            assert np.array_equal(sub[r], got[i, h])


def test_custom_scale_is_applied():
    rng = np.random.default_rng(2)
    T, L, Hq, Hkv, D = 9, 11, 2, 2, 8
    par = _random_tree(rng, T)
    q, kc, vc, kt, vt = (_rand(rng, T, Hq, D), _rand(rng, L, Hkv, D), _rand(rng, L, Hkv, D),
                         _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D))
    mask = oracle.ancestor_mask(par, T - 1)
    got = oracle.verify_attn(q, kc, vc, kt, vt, mask, scale=0.7)
    ref = _sdpa(q, kc, vc, kt, vt, _dense_visibility(par, L), scale=0.7)
    assert np.max(np.abs(got - ref)) < 1e-12


def test_closed_forms():
    rng = np.random.default_rng(3)
    T, L, Hq, Hkv, D = 12, 20, 4, 2, 16
    par = _random_tree(rng, T)
    mask = oracle.ancestor_mask(par, T - 1)
    kc, vc, kt, vt = (_rand(rng, L, Hkv, D), _rand(rng, L, Hkv, D), _rand(rng, T, Hkv, D),
                      _rand(rng, T, Hkv, D))
    # q = 0: uniform weights, output = mean of the visible value rows
    got = oracle.verify_attn(np.zeros((T, Hq, D), np.float32), kc, vc, kt, vt, mask)
    vis = _dense_visibility(par, L)
    v_all = np.concatenate([vc, vt]).astype(np.float64)
    for i in range(T):
        for h in range(Hq):
            want = v_all[vis[i], h // 2].mean(axis=0)
            assert np.max(np.abs(got[i, h] - want)) < 1e-13
    # no cache: the root sees only itself, so its output is exactly its own value row
    q = _rand(rng, T, Hq, D)
    e = np.zeros((0, Hkv, D), np.float32)
    got = oracle.verify_attn(q, e, e, kt, vt, mask)
    for h in range(Hq):
        assert np.array_equal(got[0, h], vt[0, h // 2].astype(np.float64))


def test_a_non_ancestor_key_has_no_influence_and_an_ancestor_has():
    rng = np.random.default_rng(4)
    T, L, Hq, Hkv, D = 8, 6, 2, 1, 8
    par = np.array([-1, 0, 0, 1, 1, 2, 3, 3], np.int32)    # the Figure 1 shape, 8 of 9 nodes
    mask = oracle.ancestor_mask(par, T - 1)
    q, kc, vc, kt, vt = (_rand(rng, T, Hq, D), _rand(rng, L, Hkv, D), _rand(rng, L, Hkv, D),
                         _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D))
    base = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    vt2 = vt.copy(); vt2[2] += 100.0                        # node 2 = 'c': ancestor of 5 only
    got = oracle.verify_attn(q, kc, vc, kt, vt2, mask)
    changed = [i for i in range(T) if not np.array_equal(got[i], base[i])]
    assert changed == [2, 5]


def test_padding_rows_give_zero():
    rng = np.random.default_rng(5)
    T, L, Hq, Hkv, D = 6, 0, 1, 1, 4
    par = np.array([-1, 0, 1, -1, -1, -1], np.int32)
    mask = oracle.ancestor_mask(par, 2, T=T)
    q, kt, vt = _rand(rng, T, Hq, D), _rand(rng, T, Hkv, D), _rand(rng, T, Hkv, D)
    e = np.zeros((0, Hkv, D), np.float32)
    got = oracle.verify_attn(q, e, e, kt, vt, mask)
    assert not got[3:].any() and got[:3].any()
