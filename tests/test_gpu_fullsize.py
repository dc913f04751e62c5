"""GPU parity at the full workload sizes, in the launch configuration bench.py times (batch,
shapes, workspace from ddtree_workspace_bytes).  Every stage is compared in full: top-K, tree,
mask, walk, and every (node, head) row of the attention output against the fp64 oracle, with the
error also reported on the scale of the outputs (max-abs / rms of the reference)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import ddtree_inputs as di  # noqa: E402
import oracle  # noqa: E402

if torch.cuda.is_available():
    import paper_2604_12989_amd as dd  # noqa: E402
    from tests import gpu_util as gu  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests selected but no GPU is visible")


# at these context lengths the outputs are averages of thousands of unit-variance rows (rms
# 0.01 .. 0.03), so the absolute bound alone would be loose: the error is also held to a fraction
# of that rms (bf16 rounding of such an output is 2**-9 of its own size, a few per cent of the rms
# for the largest elements; measured 0.017 .. 0.029 on these workloads)
RMS_FRACTION = 0.05


@pytest.mark.parametrize("config,spike", [(3, 0.0), (3, 20.0), (4, 0.0), (2, 25.0)])
def test_single_sequence_configs_full_size(config, spike):
    c = di.CONFIGS[config]
    seed = di.config_seed(config)
    B, V, N, Hq, Hkv, D, L = c["B"], c["V"], c["N"], c["Hq"], c["Hkv"], c["D"], c["L"]
    K, T = N, N + 1
    x = di.draft_logits(seed, B, V)
    if spike:  # a peaked drafter: deep tree instead of the recipe's shallow one
        x[np.arange(B), (np.arange(B) * 9973 + 17) % V] += spike
    print(f"config {config} spike {spike}: oracle top-K", flush=True)
    tok_o, lp_o = oracle.topk(x, K)
    tree_o = oracle.build_tree(tok_o, lp_o, N, root_token=42)
    mask_o = oracle.ancestor_mask(tree_o["parent"], tree_o["n_nodes"], T=T)

    ws = dd.Workspace(1, B, V, N, Hq, Hkv, D, L)
    tok_g, lp_g = dd.topk(gu.to_dev(x[None]), K, ws)
    tree_g = dd.build(tok_g, lp_g, N, gu.to_dev(np.array([42], np.int32)), ws)
    torch.cuda.synchronize()
    assert np.array_equal(tok_g.cpu().numpy()[0], tok_o)
    lp_same = np.array_equal(lp_g.cpu().numpy()[0], lp_o)
    assert gu_ulp(lp_g.cpu().numpy()[0], lp_o) <= 2
    print(f"  lp bit-exact: {lp_same}; max depth {tree_o['depth'].max()}", flush=True)
    tg = {k: v.cpu().numpy()[0] for k, v in tree_g.items()}
    if not lp_same:  # compare against the oracle tree built from the GPU's own log-probs
        tree_o = oracle.build_tree(tok_o, lp_g.cpu().numpy()[0], N, root_token=42)
        mask_o = oracle.ancestor_mask(tree_o["parent"], tree_o["n_nodes"], T=T)
    for key in ("tokens", "parent", "depth", "rank"):
        assert np.array_equal(tg[key], tree_o[key]), key
    assert np.array_equal(tg["node_score"].view(np.uint32), tree_o["score"].view(np.uint32))
    assert np.array_equal(tg["ancestor_mask"].view(np.uint64), mask_o)
    assert int(tg["n_nodes"]) == tree_o["n_nodes"] == N

    # attention, every (node, head) row
    q, kc, vc, kt, vt = di.attn_tensors(seed, T, L, Hq, Hkv, D, "bf16")
    out = dd.verify_attn(gu.bf16_dev(q), gu.bf16_dev(kc), gu.bf16_dev(vc), gu.bf16_dev(kt),
                         gu.bf16_dev(vt), tree_g["ancestor_mask"], [0, L], 1, T, Hq, Hkv, D,
                         1.0 / np.sqrt(D), dd.DTYPE_BF16, ws)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().reshape(T, Hq, D)
    assert np.isfinite(got).all()
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask_o)
    err = gu.attn_err(got, ref)
    frac, rms = gu.attn_err_over_rms(got, ref)
    print(f"  attention: all {T * Hq} rows, max-abs err {err:.2e}, rms(ref) {rms:.4f}, "
          f"max-abs / rms {frac:.3f}", flush=True)
    assert err < 1e-2
    assert frac < RMS_FRACTION

    # accept, full
    plant = di.planted_tokens(seed, tree_o["depth"], tok_o[:, 0], B, p=0.9 if spike else 0.8)
    tl = di.target_logits(seed, T, V, plant)
    acc_o = oracle.accept(tl, tree_o["tokens"], tree_o["parent"], tree_o["n_nodes"], B)
    acc_g = dd.accept(gu.to_dev(tl[None]), tree_g["tokens"], tree_g["parent"], tree_g["depth"],
                      tree_g["n_nodes"], B, ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc_g["posterior"].cpu().numpy()[0], acc_o["posterior"])
    assert np.array_equal(acc_g["path"].cpu().numpy()[0], acc_o["path"])
    assert int(acc_g["n_accepted"][0]) == acc_o["n_accepted"]
    assert int(acc_g["bonus_token"][0]) == acc_o["bonus"]
    print(f"  accepted {acc_o['n_accepted']}", flush=True)


def gu_ulp(a, b):
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7FFFFFFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFFFFFF), ib)
    return int(np.abs(ia - ib).max())


def test_batched_ragged_config_full_size():
    """Config 5: 16 sequences, N = 128, Hq = 64, ragged caches of 1024..8192 rows.  To keep host
    generation short, sequence s's draft / target logits are one seeded block rolled by a
    per-sequence shift along the vocabulary (plus its own spikes / plants): every element is
    still compared against the oracle run on exactly the same bytes."""
    c = di.CONFIGS[5]
    seed = di.config_seed(5)
    batch, B, V, N, Hq, Hkv, D = c["batch"], c["B"], c["V"], c["N"], c["Hq"], c["Hkv"], c["D"]
    K, T = N, N + 1
    Ls = di.ragged_lengths(seed, batch, *c["L"])
    off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
    base = di.draft_logits(seed, B, V)
    xs = np.stack([np.roll(base, 7919 * s, axis=1) for s in range(batch)])
    for s in range(batch):
        xs[s, np.arange(B), (np.arange(B) * 31 + 1000 * s) % V] += 4.0 + s  # flat ... peaked
    ws = dd.Workspace(batch, B, V, N, Hq, Hkv, D, int(off[-1]))
    tok_g, lp_g = dd.topk(gu.to_dev(xs), K, ws)
    roots = np.arange(batch, dtype=np.int32) + 100
    tree_g = dd.build(tok_g, lp_g, N, gu.to_dev(roots), ws)
    torch.cuda.synchronize()
    tok_h, lp_h = tok_g.cpu().numpy(), lp_g.cpu().numpy()
    trees, masks = [], []
    for s in range(batch):
        tok_o, lp_o = oracle.topk(xs[s], K)
        assert np.array_equal(tok_h[s], tok_o), s
        assert gu_ulp(lp_h[s], lp_o) <= 2
        t = oracle.build_tree(tok_o, lp_h[s], N, root_token=int(roots[s]))
        m = oracle.ancestor_mask(t["parent"], t["n_nodes"], T=T)
        for key in ("tokens", "parent", "depth", "rank"):
            assert np.array_equal(tree_g[key][s].cpu().numpy(), t[key]), (s, key)
        assert np.array_equal(tree_g["ancestor_mask"][s].cpu().numpy().view(np.uint64), m), s
        trees.append(t); masks.append(m)
    print("config 5: top-K and trees match; depths", [int(t["depth"].max()) for t in trees], flush=True)

    # ragged attention: K/V cache generated once for the longest total and shared bytes per sequence
    q, _, _, kt, vt = di.attn_tensors(seed, batch * T, 0, Hq, Hkv, D, "bf16")
    _, kc, vc, _, _ = di.attn_tensors(seed + 1, 1, int(off[-1]), Hq, Hkv, D, "bf16")
    out = dd.verify_attn(gu.bf16_dev(q), gu.bf16_dev(kc), gu.bf16_dev(vc), gu.bf16_dev(kt),
                         gu.bf16_dev(vt), tree_g["ancestor_mask"], off, batch, T, Hq, Hkv, D,
                         1.0 / np.sqrt(D), dd.DTYPE_BF16, ws)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().reshape(batch, T, Hq, D)
    assert np.isfinite(got).all()
    worst, worst_frac = 0.0, 0.0
    for s in range(batch):
        ref = oracle.verify_attn(q[s * T:(s + 1) * T], kc[off[s]:off[s + 1]], vc[off[s]:off[s + 1]],
                                 kt[s * T:(s + 1) * T], vt[s * T:(s + 1) * T], masks[s])
        worst = max(worst, gu.attn_err(got[s], ref))
        worst_frac = max(worst_frac, gu.attn_err_over_rms(got[s], ref)[0])
    print(f"  ragged attention: all {batch * T * Hq} rows, max-abs err {worst:.2e}, "
          f"max-abs / rms {worst_frac:.3f}", flush=True)
    assert worst < 1e-2
    assert worst_frac < RMS_FRACTION

    # accept on [16*129, V]
    tbase = di.target_logits(seed, T, V, np.full(T, -1))
    tl = np.stack([np.roll(tbase, 104729 * s, axis=1) for s in range(batch)])
    for s in range(batch):
        plant = di.planted_tokens(seed + s, trees[s]["depth"], tok_h[s][:, 0], B, p=0.9, batch_index=s)
        rows = np.nonzero(plant >= 0)[0]
        tl[s, rows, plant[rows]] = 10.0
    acc_g = dd.accept(gu.to_dev(tl), tree_g["tokens"], tree_g["parent"], tree_g["depth"],
                      tree_g["n_nodes"], B, ws)
    torch.cuda.synchronize()
    for s in range(batch):
        a = oracle.accept(tl[s], trees[s]["tokens"], trees[s]["parent"], trees[s]["n_nodes"], B)
        assert np.array_equal(acc_g["posterior"][s].cpu().numpy(), a["posterior"]), s
        assert np.array_equal(acc_g["path"][s].cpu().numpy(), a["path"]), s
        assert int(acc_g["bonus_token"][s]) == a["bonus"]
    print("  accept matches; accepted", acc_g["n_accepted"].cpu().numpy().tolist(), flush=True)


def test_attention_retry_when_scores_outgrow_the_reference():
    """Keys late in the range score > 2^64 above the row's first keys: the workgroup must redo its
    range with the true maxima and still match the oracle."""
    T, L, Hq, Hkv, D = 40, 700, 8, 2, 128
    rng = np.random.default_rng(77)
    par = np.arange(-1, T - 1, dtype=np.int32)
    par[5:] = rng.integers(0, 5, T - 5)
    mask = oracle.ancestor_mask(par, T - 1)
    q, kc, vc, kt, vt = di.attn_tensors(77, T, L, Hq, Hkv, D, "bf16")
    # cache keys 600.. are 7x the query of node (j % T), head 0 of the kv group: score ~ 7*|q|^2/sqrt(D) ~ 80
    for j in range(600, L):
        for hk in range(Hkv):
            kc[j, hk] = di.round_to_bf16(7.0 * q[j % T, hk * (Hq // Hkv)])
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, "bf16")[0]
    assert np.isfinite(got).all()
    err = gu.attn_err(got, ref)
    print(f"retry case: max err {err:.2e}")
    assert err < 1e-2


def test_sampled_walk_full_size_config3():
    """Temperature sampling at the headline shape (257 rows x 151936 tokens, the launch shape of
    the greedy scan): every selection against the oracle's fp64 Gumbel-max, the walk exactly."""
    c = di.CONFIGS[3]
    seed = di.config_seed(3, 2)
    B, V, N = c["B"], c["V"], c["N"]
    T = N + 1
    x = di.draft_logits(seed, B, V)
    tok_o, lp_o = oracle.topk(x, N)
    tr = oracle.build_tree(tok_o, lp_o, N, 11)
    plant = di.planted_tokens(seed, tr["depth"], tok_o[:, 0], B)
    tl = di.target_logits(seed, T, V, plant)
    for tau, s in ((1.0, 2026), (0.25, 7)):
        got = gu.gpu_accept(tl, tr["tokens"], tr["parent"], tr["depth"], tr["n_nodes"], B,
                            temperature=tau, seed=s)
        sel, run, gap = oracle.sample_tokens(tl, tr["n_nodes"], tau, s)
        post = got["posterior"][0]
        clear = gap > 2e-4
        assert clear.sum() >= T - 3
        assert np.array_equal(post[clear], sel[clear])
        assert np.all((post[~clear] == sel[~clear]) | (post[~clear] == run[~clear]))
        w = oracle.walk(post, tr["tokens"], tr["parent"], tr["n_nodes"], B)
        assert int(got["n_accepted"][0]) == w["n_accepted"]
        assert int(got["bonus_token"][0]) == w["bonus"]
        assert np.array_equal(got["path"][0], w["path"])
        print(f"tau={tau}: accepted {w['n_accepted']}, {int((~clear).sum())} close selections")
