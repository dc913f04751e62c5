"""GPU parity: every stage of the HIP library against the CPU oracle, element by element, on
the same seeded inputs.  Bit-exact for tokens / tree / mask / walk; log-probabilities within
2 ulp (fp64 log-sum-exp on both sides, different summation order); attention within 1e-2
(bf16) or 1e-5 (fp32) max-abs on unit-variance inputs."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import ddtree_inputs as di  # noqa: E402
import oracle  # noqa: E402

if torch.cuda.is_available():
    from tests import gpu_util as gu  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests selected but no GPU is visible")


def attn_err(got, ref):
    """The attention bound as the tolerance states it: max-abs error, 1e-2 (bf16) / 1e-5 (fp32),
    on every element whose reference magnitude is below 4 (everything unit-variance inputs give);
    an element of magnitude 4 or more is compared relative to its own size (a bf16 value in [4, 8)
    is spaced 2**-5 apart, so half a step alone exceeds 1e-2)."""
    return gu.attn_err(got, ref)


def ulp_diff(a, b):
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7FFFFFFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFFFFFF), ib)
    return np.abs(ia - ib)


# ------------------------------------------------------------------------------- top-K
TOPK_CASES = [
    ("tiny_config1", dict(B=8, V=1024, K=16, seed=di.config_seed(1))),
    ("odd_V_unaligned_rows", dict(B=5, V=50001, K=64, seed=7)),
    ("K_equals_V", dict(B=3, V=300, K=300, seed=8)),
    ("one_chunk_short_tail", dict(B=2, V=12290, K=100, seed=9)),
    ("wide_K", dict(B=2, V=40000, K=1024, seed=10)),
]


@pytest.mark.parametrize("name,c", TOPK_CASES, ids=[n for n, _ in TOPK_CASES])
def test_topk_matches_oracle(name, c):
    x = di.draft_logits(c["seed"], c["B"], c["V"])
    tok_o, lp_o = oracle.topk(x, c["K"])
    tok_g, lp_g = gu.gpu_topk(x, c["K"])
    assert np.array_equal(tok_g[0], tok_o)
    assert ulp_diff(lp_g[0], lp_o).max() <= 2
    print(f"{name}: lp bit-exact rate {np.mean(lp_g[0] == lp_o):.6f}")


def test_topk_duplicates_and_flat_rows():
    rng = np.random.default_rng(3)
    V = 30000
    x = np.round(rng.standard_normal((6, V)) * 4).astype(np.float32) / 4  # heavy duplication
    x[1] = 2.5                                                          # one value everywhere
    x[2, :] = -1.0
    x[2, [29999, 17, 4000]] = 0.0                                       # ties at the top
    x[3] = np.where(np.arange(V) % 2 == 0, 1.0, -1.0)                   # half the row ties at K
    x[4] = -np.arange(V, dtype=np.float32)                              # strictly decreasing
    x[5] = np.arange(V, dtype=np.float32) * 1e-3                        # strictly increasing
    for K in (1, 7, 256):
        tok_o, lp_o = oracle.topk(x, K)
        tok_g, lp_g = gu.gpu_topk(x, K)
        assert np.array_equal(tok_g[0], tok_o), K
        assert ulp_diff(lp_g[0], lp_o).max() <= 2


def test_topk_masked_vocabulary():
    """Rows where most of the vocabulary is masked with -inf, some with fewer finite entries
    than K: the -inf entries then fill the tail in token order, with log-probability -inf."""
    V, K = 30000, 64
    x = di.draft_logits(21, 4, V)
    x[0, 100:] = -np.inf                     # 100 finite entries >= K
    x[1, 40:] = -np.inf                      # 40 finite entries < K
    x[2, ::2] = -np.inf                      # every other entry masked
    x[3, :29000] = -np.inf                   # whole chunks masked
    tok_o, lp_o = oracle.topk(x, K)
    tok_g, lp_g = gu.gpu_topk(x, K)
    assert np.array_equal(tok_g[0], tok_o)
    fin = np.isfinite(lp_o)
    assert np.array_equal(np.isfinite(lp_g[0]), fin)
    assert np.all(lp_g[0][~fin] == -np.inf)
    assert ulp_diff(lp_g[0][fin], lp_o[fin]).max() <= 2


def test_topk_masked_rows_with_a_last_chunk_shorter_than_K():
    """V = 12289 at K = 1024 is cut into 12 chunks of 1028 with a last chunk of 981 < K entries;
    with masked (-inf) entries in it every one of its elements is a candidate."""
    rng = np.random.default_rng(323)
    for V, K in ((12289, 1024), (4100, 1024), (2049, 1024), (1030, 1024)):
        x = rng.standard_normal((3, V)).astype(np.float32)
        x[:, rng.random(V) < 0.7] = -np.inf
        x[:, 0] = 0.0
        x[2, V - 500:] = -np.inf                 # a last chunk that is masked altogether
        tok_o, lp_o = oracle.topk(x, K)
        tok_g, lp_g = gu.gpu_topk(x, K)
        assert np.array_equal(tok_g[0], tok_o), (V, K)
        fin = np.isfinite(lp_o)
        assert np.array_equal(np.isfinite(lp_g[0]), fin)
        assert ulp_diff(lp_g[0][fin], lp_o[fin]).max() <= 2


def test_topk_batched():
    xs = np.stack([di.draft_logits(11, 4, 20000, batch_index=b) for b in range(3)])
    tok_g, lp_g = gu.gpu_topk(xs, 32)
    for b in range(3):
        tok_o, lp_o = oracle.topk(xs[b], 32)
        assert np.array_equal(tok_g[b], tok_o)
        assert ulp_diff(lp_g[b], lp_o).max() <= 2


def test_topk_many_rows():
    """128 rows or more take the one-workgroup-per-row kernel: vocabulary sizes from one element
    to several passes per thread with ragged heads and tails, K up to 1024, row kinds that overflow
    its candidate list (flat rows, heavy ties, masked rows) and rows with one dominant token."""
    rng = np.random.default_rng(4242)
    worst = 0
    for case, (V, K) in enumerate(((1, 1), (7, 7), (1000, 16), (4097, 256), (8191, 1024), (8193, 64),
                                   (20000, 1024), (50001, 256), (151936, 128), (151936, 1024))):
        batch, B = (8, 16) if V < 100000 else (16, 16)
        x = rng.standard_normal((batch, B, V)).astype(np.float32) * np.float32(3.0)
        x[0, 0] = 1.25                                        # flat row: every entry ties
        x[0, 1] = np.round(x[0, 1])                           # heavy ties
        x[0, 2, rng.random(V) < 0.7] = -np.inf                # masked row
        x[0, 2, 0] = 0.0
        x[0, 3, rng.integers(0, V)] += np.float32(40.0)       # nearly certain token
        x[0, 4] = -np.arange(V, dtype=np.float32) * np.float32(1e-3)   # strictly decreasing
        x[0, 5] = np.arange(V, dtype=np.float32) * np.float32(1e-3)    # strictly increasing
        tok_g, lp_g = gu.gpu_topk(x, K)
        for b in range(batch):
            tok_o, lp_o = oracle.topk(x[b], K)
            assert np.array_equal(tok_g[b], tok_o), (V, K, b)
            fin = np.isfinite(lp_o)
            assert np.array_equal(np.isfinite(lp_g[b]), fin), (V, K, b)
            if fin.any():
                u = int(ulp_diff(lp_g[b][fin], lp_o[fin]).max())
                worst = max(worst, u)
                assert u <= 2, (V, K, b, u)
    print(f"worst log-probability difference {worst} ulp")


def test_topk_nearly_certain_rows():
    """One token holds all but 1e-5 .. 1e-11 of the probability: its log-probability is a tiny
    negative number that only survives when the log-sum-exp is formed as max + log1p(rest)."""
    for V, K in ((7, 7), (64, 16), (1000, 16), (50001, 64)):
        rng = np.random.default_rng(V)
        x = rng.standard_normal((6, V)).astype(np.float32)
        x[np.arange(6), rng.integers(0, V, 6)] += np.float32(25.0)
        x[5, :] = x[5, :].min()                 # ... and a row whose maximum is repeated V times
        tok_o, lp_o = oracle.topk(x, K)
        tok_g, lp_g = gu.gpu_topk(x, K)
        assert np.array_equal(tok_g[0], tok_o), V
        assert np.all(lp_o[:5, 0] < 0) and np.all(lp_o[:5, 0] > -1e-3)
        assert ulp_diff(lp_g[0], lp_o).max() <= 2, V


def test_topk_randomized_shapes():
    """Seeded sweep over vocabulary sizes (one element to several chunks with a ragged tail), K,
    batch and row kinds; token ids bit-exact, log-probabilities within 2 ulp."""
    rng = np.random.default_rng(2024)
    worst = 0
    for c in range(60):
        V = int(rng.choice([1, 2, 7, 64, 1000, 4096, 12288, 12289, 20000, 50001, 151936, 200003]))
        B = int(rng.integers(1, 17))
        K = int(min(V, rng.choice([1, 2, 16, 64, 255, 256, 257, 512, 1024])))
        kind = ["normal", "wide", "ints", "const", "spiky", "masked"][c % 6]
        if kind == "normal":
            x = rng.standard_normal((B, V))
        elif kind == "wide":
            x = rng.standard_normal((B, V)) * rng.uniform(0.1, 30, size=(B, 1))
        elif kind == "ints":
            x = rng.integers(-3, 4, size=(B, V)).astype(np.float64)
        elif kind == "const":
            x = np.full((B, V), float(rng.normal()))
        elif kind == "spiky":
            x = rng.standard_normal((B, V))
            x[np.arange(B), rng.integers(0, V, B)] += 25.0
        else:
            x = rng.standard_normal((B, V))
            x[:, rng.random(V) < 0.7] = -np.inf
            x[:, 0] = 0.0
        x = x.astype(np.float32)
        tok_o, lp_o = oracle.topk(x, K)
        tok_g, lp_g = gu.gpu_topk(x, K)
        fin = np.isfinite(lp_o)
        assert np.array_equal(tok_g[0], tok_o), (c, kind, B, V, K)
        assert np.array_equal(np.isfinite(lp_g[0]), fin), (c, kind, B, V, K)
        if fin.any():
            u = int(ulp_diff(lp_g[0][fin], lp_o[fin]).max())
            worst = max(worst, u)
            assert u <= 2, (c, kind, B, V, K, u)
    print(f"worst log-probability difference {worst} ulp")


# ------------------------------------------------------------------------------- build
@pytest.fixture(params=["auto", "pops", "levels"])
def build_algo(request):
    """Every build test runs under each construction: the choice may change speed, never the tree."""
    import paper_2604_12989_amd as dd
    dd.set_build_algorithm({"auto": dd.BUILD_AUTO, "pops": dd.BUILD_POPS, "levels": dd.BUILD_LEVELS}[request.param])
    yield request.param
    dd.set_build_algorithm(dd.BUILD_AUTO)


def _peaked_logits(seed, B, V, spike):
    x = di.draft_logits(seed, B, V)
    rng = np.random.default_rng(seed)
    x[np.arange(B), rng.integers(0, V, B)] += spike
    return x


def _check_build(tok, lp, N, root=5):
    o = oracle.build_tree(tok, lp, N, root)
    g = gu.gpu_build(tok, lp, N, root)
    assert int(g["n_nodes"][0]) == o["n_nodes"]
    for key, okey in (("tokens", "tokens"), ("parent", "parent"), ("depth", "depth"),
                      ("rank", "rank")):
        assert np.array_equal(g[key][0], o[okey]), key
    assert np.array_equal(g["node_score"][0].view(np.uint32), o["score"].view(np.uint32))
    m = oracle.ancestor_mask(o["parent"], o["n_nodes"], T=N + 1)
    assert np.array_equal(g["ancestor_mask"][0], m)
    return o


@pytest.mark.parametrize("N", [1, 2, 16, 63, 64, 65, 128, 256, 512, 1024])
def test_build_matches_oracle_on_workload_logits(N, build_algo):
    x = di.draft_logits(di.config_seed(2), 16, 20000)
    K = min(N, 20000)
    tok, lp = oracle.topk(x, K)
    _check_build(tok, lp, N)


@pytest.mark.parametrize("spike,N", [(6.0, 64), (9.0, 256), (12.0, 256), (14.0, 512), (20.0, 100)])
def test_build_deep_trees(spike, N, build_algo):
    import paper_2604_12989_amd as dd
    x = _peaked_logits(21, 16, 8192, spike)
    tok, lp = oracle.topk(x, min(N, 8192))
    before = dd.build_giveups()
    o = _check_build(tok, lp, N)
    # tie-free logits: the level construction must carry these through on its own
    assert dd.build_giveups() == before
    print(f"spike {spike}: max depth {o['depth'].max()}")


@pytest.mark.parametrize("spike,N", [(16.0, 1024), (24.0, 1024), (18.0, 768)])
def test_build_large_budget_on_peaked_rows(spike, N, build_algo):
    # deep trees at large budgets: the level construction has to squeeze dead members out
    import paper_2604_12989_amd as dd
    x = _peaked_logits(23, 16, 8192, spike)
    tok, lp = oracle.topk(x, N)
    before = dd.build_giveups()
    o = _check_build(tok, lp, N)
    assert o["depth"].max() == 16
    assert dd.build_giveups() == before


@pytest.mark.parametrize("B,spike,N,K", [(24, 13.0, 256, 256), (32, 12.0, 300, 200), (32, 14.0, 512, 512), (17, 13.0, 128, 64)])
def test_build_more_than_sixteen_positions(B, spike, N, K, build_algo):
    # block sizes beyond 16: deep chains that run past row 16 (the level construction enters the
    # low ranks off the top-1 chain two rows per thread there) and fewer ranks than budget
    x = _peaked_logits(29, B, 4096, spike)
    tok, lp = oracle.topk(x, K)
    o = _check_build(tok, lp, N)
    assert o["depth"].max() > 16


@pytest.mark.parametrize("p_top,N", [(0.3, 256), (0.6, 256), (0.6, 512), (0.9, 256), (0.9, 512), (0.9, 1024), (0.97, 128)])
def test_build_rows_peaked_at_a_given_probability(p_top, N, build_algo):
    # every draft row with one token at probability p_top: at 0.9 the whole tree comes from the
    # prefixes entered up front and is enumerated by generations; at 0.6 and N = 512 that attempt
    # lets in too many members and the levels take over; at 0.3 no cut is known up front
    import paper_2604_12989_amd as dd
    x = di.peaked_draft_logits(31, 16, 30000, p_top)
    tok, lp = oracle.topk(x, min(N, 30000))
    before = dd.build_giveups()
    _check_build(tok, lp, N)
    assert dd.build_giveups() == before


def test_build_rows_with_minus_infinity(build_algo):
    # masked vocabulary: rows end in -inf log-probabilities, which never become nodes
    rng = np.random.default_rng(9)
    for K_live, N in ((5, 40), (12, 64), (3, 30)):
        x = rng.normal(size=(6, 64)).astype(np.float32) * 2.0
        x[:, K_live:] = -np.inf
        tok, lp = oracle.topk(x, 32)
        _check_build(tok, lp, N)


def test_build_finite_prefixes_run_out(build_algo):
    """Fewer prefixes of finite score than the budget: the tree ends where they do.  Algorithm 1 as
    written would go on popping candidates of score -inf (tokens of probability zero, which the
    paper's assumption q in (0,1) excludes); the library stops there.  The expected tree is the
    unmodified oracle's, cut at its first -inf score; the rows behind it are padding."""
    rng = np.random.default_rng(19)
    for K_live, B, N in ((2, 3, 40), (1, 4, 10), (3, 2, 64), (2, 5, 100), (1, 1, 7), (4, 3, 300)):
        x = rng.normal(size=(B, 64)).astype(np.float32) * 2.0
        x[:, K_live:] = -np.inf
        K = min(N, 32)
        tok, lp = oracle.topk(x, K)
        o = oracle.build_tree(tok, lp, N, 5)
        live = min(K_live, K)
        n_fin = sum(live ** d for d in range(1, B + 1))
        assert n_fin < N
        sc = o["score"][1:o["n_nodes"] + 1]
        assert np.isfinite(sc[:n_fin]).all() and not np.isfinite(sc[n_fin:]).any()
        g = gu.gpu_build(tok, lp, N, 5)
        assert int(g["n_nodes"][0]) == n_fin, (K_live, B, N)
        for key in ("tokens", "parent", "depth", "rank"):
            assert np.array_equal(g[key][0][:n_fin + 1], o[key][:n_fin + 1]), key
            assert np.all(g[key][0][n_fin + 1:] == -1), key
        assert np.array_equal(g["node_score"][0][:n_fin + 1].view(np.uint32),
                              o["score"][:n_fin + 1].view(np.uint32))
        assert not g["node_score"][0][n_fin + 1:].any()
        assert np.array_equal(g["ancestor_mask"][0], oracle.ancestor_mask(o["parent"], n_fin, T=N + 1))


def test_build_randomized_shapes(build_algo):
    # a seeded sweep over depths, rank counts (also fewer ranks than budget), budgets and kinds of
    # rows: smooth, peaked, mixed sharpness per row, and rows with many exactly equal values
    rng = np.random.default_rng(77)

    def rows(B, K, kind):
        if kind == "dyadic":
            return (-np.sort(rng.integers(0, 8, size=(B, K)), axis=1) / 4.0).astype(np.float32)
        if kind == "few":
            x = rng.integers(0, 4, size=(B, K)).astype(np.float64) * 1.5
        elif kind == "peaked":
            x = rng.normal(size=(B, K)); x[:, 0] += rng.uniform(2, 12, size=B)
        elif kind == "mixed":
            x = rng.normal(size=(B, K)) * rng.uniform(0.2, 4, size=(B, 1)); x[:, 0] += rng.uniform(0, 10, size=B)
        else:
            x = rng.normal(size=(B, K))
        x = -np.sort(-x, axis=1)
        m = x.max(1, keepdims=True)
        return (x - (np.log(np.exp(x - m).sum(1, keepdims=True)) + m)).astype(np.float32)

    import paper_2604_12989_amd as dd
    for case in range(300):
        kind = ["flat", "peaked", "mixed", "dyadic", "few"][case % 5]
        B = int(rng.integers(1, 33))
        N = int(rng.choice([1, 2, 5, 17, 40, 64, 65, 100, 129, 200, 256, 300, 512, 777, 1024]))
        K = int(min(N, rng.choice([1, 2, 3, 8, 50, 200, 1024])))
        if 4 * B * (K + 3) + 8 * (N + 1) > 153600:
            continue
        lp = rows(B, K, kind)
        tok = rng.permutation(B * K).astype(np.int32).reshape(B, K)
        before = dd.build_giveups()
        _check_build(tok, lp, N, root=3)
        # rows without exact ties: the level construction carries them through on its own
        # (candidate arrays that overflow are counted first and searched again)
        if kind in ("flat", "peaked", "mixed"):
            assert dd.build_giveups() == before, (kind, B, K, N)


def test_build_exact_ties_and_dry_heap(build_algo):
    rng = np.random.default_rng(5)
    for trial in range(20):
        B, K = int(rng.integers(1, 6)), int(rng.integers(1, 7))
        lp = (-np.sort(rng.integers(0, 6, size=(B, K)), axis=1) / 4.0).astype(np.float32)
        tok = rng.permutation(B * K).astype(np.int32).reshape(B, K)
        total = sum(K ** d for d in range(1, B + 1))
        for N in {1, min(total, 40), min(total + 3, 70)}:
            _check_build(tok, lp, N)


def test_build_batched(build_algo):
    toks, lps = [], []
    for b in range(4):
        x = _peaked_logits(30 + b, 8, 4096, 5.0 + 3 * b)
        t, l = oracle.topk(x, 96)
        toks.append(t); lps.append(l)
    g = gu.gpu_build(np.stack(toks), np.stack(lps), 96, [1, 2, 3, 4])
    for b in range(4):
        o = oracle.build_tree(toks[b], lps[b], 96, b + 1)
        assert np.array_equal(g["tokens"][b], o["tokens"])
        assert np.array_equal(g["parent"][b], o["parent"])
        assert np.array_equal(g["ancestor_mask"][b],
                              oracle.ancestor_mask(o["parent"], o["n_nodes"], T=97))


# ------------------------------------------------------------------------------- attention
def _random_tree(rng, T, n_nodes=None, chainy=0.5):
    n = T - 1 if n_nodes is None else n_nodes
    par = np.full(T, -1, np.int32)
    for i in range(1, n + 1):
        par[i] = i - 1 if rng.random() < chainy else rng.integers(0, i)
    return par, n


def _attn_case(seed, T, L, Hq, Hkv, D, dtype, n_nodes=None):
    rng = np.random.default_rng(seed)
    par, n = _random_tree(rng, T, n_nodes)
    mask = oracle.ancestor_mask(par, n, T=T)
    q, kc, vc, kt, vt = di.attn_tensors(seed, T, L, Hq, Hkv, D, dtype)
    return q, kc, vc, kt, vt, mask


ATTN_BF16 = [(17, 128, 4, 1, 1), (65, 100, 8, 2, 2), (257, 333, 8, 2, 3), (129, 1000, 16, 2, 4),
             (257, 0, 4, 4, 5), (64, 64, 32, 8, 6), (513, 2048, 8, 2, 7), (40, 4100, 32, 8, 8),
             # row counts a few blocks past whole tiles of 8 (uneven tiling: 2, 3 and 4 spare blocks)
             (75, 3000, 16, 4, 9), (273, 5000, 32, 8, 10), (90, 700, 8, 2, 11),
             # query heads per KV head that are not powers of two (3, 5, 12)
             (65, 500, 6, 2, 12), (129, 300, 10, 2, 13), (40, 1000, 12, 1, 14)]


@pytest.mark.parametrize("T,L,Hq,Hkv,seed", ATTN_BF16)
def test_attn_bf16_mfma_matches_oracle(T, L, Hq, Hkv, seed):
    D = 128
    q, kc, vc, kt, vt, mask = _attn_case(seed, T, L, Hq, Hkv, D, "bf16")
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, "bf16")[0]
    err = attn_err(got, ref)
    print(f"T={T} L={L}: max err {err:.2e} (abs {np.abs(got - ref).max():.2e}), "
          f"rms(ref) {np.sqrt((ref ** 2).mean()):.3f}")
    assert err < 1e-2


def test_attn_largest_tree():
    """T = DDTREE_MAX_N + 1 = 1025 rows (17 mask words per row), checked on sampled (node, head)
    pairs that include the last node and rows of every mask word."""
    T, L, Hq, Hkv, D = 1025, 1500, 8, 2, 128
    q, kc, vc, kt, vt, mask = _attn_case(77, T, L, Hq, Hkv, D, "bf16")
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, "bf16")[0]
    rng = np.random.default_rng(77)
    nodes = np.concatenate([[0, 1, 63, 64, 65, 1023, 1024], rng.integers(0, T, 57)])
    pairs = np.stack([nodes, rng.integers(0, Hq, nodes.size)], axis=1).astype(np.int32)
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask, pairs=pairs)
    assert attn_err(got[pairs[:, 0], pairs[:, 1]], ref) < 1e-2


def test_largest_batch_through_every_stage():
    """DDTREE_MAX_BATCH = 64 sequences in one call of each stage (ragged caches, the last empty)."""
    batch, B, V, N, Hq, Hkv, D = 64, 4, 3000, 20, 4, 2, 128
    K, T = N, N + 1
    rng = np.random.default_rng(64)
    xs = np.stack([_peaked_logits(640 + s, B, V, 6.0) for s in range(batch)])
    tok_g, lp_g = gu.gpu_topk(xs, K)
    roots = np.arange(batch, dtype=np.int32)
    tree_g = gu.gpu_build(tok_g, lp_g, N, roots)
    Ls = rng.integers(0, 300, batch)
    Ls[-1] = 0
    off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
    q, _, _, kt, vt = di.attn_tensors(64, batch * T, 0, Hq, Hkv, D, "bf16")
    _, kc, vc, _, _ = di.attn_tensors(65, 1, int(off[-1]), Hq, Hkv, D, "bf16")
    trees, tls = [], []
    for s in range(batch):
        tok_o, lp_o = oracle.topk(xs[s], K)
        assert np.array_equal(tok_g[s], tok_o), s
        assert ulp_diff(lp_g[s], lp_o).max() <= 2
        t = oracle.build_tree(tok_o, lp_g[s], N, root_token=int(roots[s]))
        for key in ("tokens", "parent", "depth"):
            assert np.array_equal(tree_g[key][s], t[key]), (s, key)
        assert np.array_equal(tree_g["ancestor_mask"][s], oracle.ancestor_mask(t["parent"], t["n_nodes"], T=T)), s
        trees.append(t)
        plant = di.planted_tokens(700 + s, t["depth"], tok_o[:, 0], B, p=0.9, batch_index=s)
        tls.append(di.target_logits(700 + s, T, V, plant, batch_index=s))
    got = gu.gpu_attn(q, kc, vc, kt, vt, tree_g["ancestor_mask"], off, batch, T, "bf16")
    for s in (0, 1, 31, 62, 63):
        ref = oracle.verify_attn(q[s * T:(s + 1) * T], kc[off[s]:off[s + 1]], vc[off[s]:off[s + 1]],
                                 kt[s * T:(s + 1) * T], vt[s * T:(s + 1) * T], tree_g["ancestor_mask"][s])
        assert attn_err(got[s], ref) < 1e-2, s
    acc = gu.gpu_accept(np.stack(tls), tree_g["tokens"], tree_g["parent"], tree_g["depth"],
                        tree_g["n_nodes"], B)
    for s in range(batch):
        o = oracle.accept(tls[s], trees[s]["tokens"], trees[s]["parent"], trees[s]["n_nodes"], B)
        assert np.array_equal(acc["path"][s], o["path"]), s
        assert int(acc["n_accepted"][s]) == o["n_accepted"] and int(acc["bonus_token"][s]) == o["bonus"], s


def test_attn_fp32_config1():
    c = di.CONFIGS[1]
    T = c["N"] + 1
    q, kc, vc, kt, vt, mask = _attn_case(di.config_seed(1), T, c["L"], c["Hq"], c["Hkv"], c["D"],
                                         "fp32")
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, c["L"]], 1, T, "fp32")[0]
    assert attn_err(got, ref) < 1e-5


@pytest.mark.parametrize("dtype,D,tol", [("fp32", 64, 1e-5), ("fp32", 128, 1e-5), ("bf16", 64, 1e-2),
                                         ("fp32", 40, 1e-5)])
def test_attn_generic_path(dtype, D, tol):
    T, L, Hq, Hkv = 70, 300, 6, 3
    q, kc, vc, kt, vt, mask = _attn_case(12, T, L, Hq, Hkv, D, dtype)
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, dtype)[0]
    assert attn_err(got, ref) < tol


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_attn_mask_leak_adversarial(dtype):
    """A wrongly visible non-ancestor (or a wrongly hidden ancestor) must move the output by
    O(10..100): keys aligned with the query carry large values."""
    T, L, Hq, Hkv, D = 200, 70, 4, 2, 128
    rng = np.random.default_rng(99)
    par, n = _random_tree(rng, T, chainy=0.3)
    mask = oracle.ancestor_mask(par, n, T=T)
    q, kc, vc, kt, vt = di.attn_tensors(99, T, L, Hq, Hkv, D, dtype)
    rnd = di.round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    # every tree key is strongly aligned with the queries of head 0 of its KV group for a
    # different node: the key of node j points along q[(j * 7 + 3) % T]
    for j in range(T):
        tgt = (j * 7 + 3) % T
        for hk in range(Hkv):
            kt[j, hk] = rnd(3.0 * q[tgt, hk * (Hq // Hkv)])
    vt[:] = rnd((100.0 * np.sign(vt) + vt).astype(np.float32))
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, dtype)[0]
    # values are +-100: bf16 probabilities (8 mantissa bits) leave ~0.5 absolute; a leak is O(100)
    atol = 1.0 if dtype == "bf16" else 1e-2
    assert np.abs(got - ref).max() <= atol
    # the construction is sensitive: one wrongly visible key in the oracle moves the row by O(100)
    for j in range(1, T):
        i = (j * 7 + 3) % T
        if i != j and not (int(mask[i, j >> 6]) >> (j & 63)) & 1:
            break
    mask2 = mask.copy()
    mask2[i, j >> 6] |= np.uint64(1) << np.uint64(j & 63)
    moved = oracle.verify_attn(q, kc, vc, kt, vt, mask2, pairs=[[i, 0]])
    assert np.abs(moved[0] - ref[i, 0]).max() > 50.0


def test_attn_large_values_through_split_partials():
    """Value rows of magnitude 1e5 (beyond the fp16 range of 65504) on a shape whose key range is
    split: the partial results are stored relative to their row's magnitude, so nothing overflows."""
    import paper_2604_12989_amd as dd
    T, L, Hq, Hkv, D = 257, 4100, 8, 2, 128
    assert dd.verify_attn_workspace_bytes(1, T, Hq, Hkv, D, dd.DTYPE_BF16, L) > 0   # split: partials in scratch
    q, kc, vc, kt, vt, mask = _attn_case(31, T, L, Hq, Hkv, D, "bf16")
    vc = di.round_to_bf16((1.0e5 * (1.0 + 0.1 * vc)).astype(np.float32))
    vt = di.round_to_bf16((1.0e5 * (1.0 + 0.1 * vt)).astype(np.float32))
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, "bf16")[0]
    assert np.isfinite(got).all()
    assert np.abs(ref).min() > 5.0e4          # every element is compared relative to its size
    err = attn_err(got, ref)
    print(f"values of 1e5: max relative err {err:.2e}")
    assert err < 1e-2


def test_attn_chain_tree_and_no_cache():
    T, Hq, Hkv, D = 130, 4, 2, 128
    q, kc, vc, kt, vt = di.attn_tensors(5, T, 0, Hq, Hkv, D, "bf16")
    mask = oracle.ancestor_mask(np.arange(-1, T - 1, dtype=np.int32), T - 1)
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, 0], 1, T, "bf16")[0]
    assert attn_err(got, ref) < 1e-2
    # the root sees only itself: its output is its own value row, exactly
    for h in range(Hq):
        assert np.array_equal(got[0, h], vt[0, h // 2])


def test_attn_generic_randomized_shapes():
    """Seeded sweep of the generic kernel (fp32 at any head size, bf16 at head sizes other than 128):
    head sizes from 8 to 256, head layouts, ragged batches, short and empty caches, padded trees."""
    rng = np.random.default_rng(808)
    worst = {"fp32": 0.0, "bf16": 0.0}
    for case in range(40):
        dtype = "fp32" if case % 2 == 0 else "bf16"
        D = int(rng.choice([8, 16, 40, 64, 72, 96, 128, 200, 256] if dtype == "fp32" else [8, 16, 40, 64, 72, 200, 256]))
        Hkv = int(rng.choice([1, 2, 3])); Hq = Hkv * int(rng.choice([1, 2, 4]))
        T = int(rng.choice([1, 2, 9, 33, 70, 130])); batch = int(rng.choice([1, 2, 3]))
        Ls = [int(rng.choice([0, 1, 7, 100, 255, 256, 257, 600])) for _ in range(batch)]
        off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
        qs, kcs, vcs, kts, vts, ms = [], [], [], [], [], []
        for b in range(batch):
            q, kc, vc, kt, vt = di.attn_tensors(9000 + 10 * case + b, T, Ls[b], Hq, Hkv, D, dtype)
            par, n = _random_tree(rng, T, int(rng.integers(0, T)) if rng.random() < 0.3 else None)
            qs.append(q); kcs.append(kc); vcs.append(vc); kts.append(kt); vts.append(vt)
            ms.append(oracle.ancestor_mask(par, n, T=T))
        got = gu.gpu_attn(np.concatenate(qs), np.concatenate(kcs), np.concatenate(vcs), np.concatenate(kts),
                          np.concatenate(vts), np.stack(ms), off, batch, T, dtype)
        for b in range(batch):
            ref = oracle.verify_attn(qs[b], kcs[b], vcs[b], kts[b], vts[b], ms[b])
            err = attn_err(got[b], ref)
            assert err < (1e-5 if dtype == "fp32" else 1e-2), (case, dtype, D, Hq, Hkv, T, Ls, b, err)
            worst[dtype] = max(worst[dtype], err)
    print(f"worst error fp32 {worst['fp32']:.2e}, bf16 {worst['bf16']:.2e}")


def test_attn_padding_rows_are_zero():
    T, L, Hq, Hkv, D = 80, 50, 4, 2, 128
    q, kc, vc, kt, vt, mask = _attn_case(6, T, L, Hq, Hkv, D, "bf16", n_nodes=40)
    ref = oracle.verify_attn(q, kc, vc, kt, vt, mask)
    got = gu.gpu_attn(q, kc, vc, kt, vt, mask[None], [0, L], 1, T, "bf16")[0]
    assert not got[41:].any() and not ref[41:].any()
    assert attn_err(got, ref) < 1e-2


def test_attn_batched_ragged():
    batch, T, Hq, Hkv, D = 3, 33, 16, 2, 128
    Ls = [130, 0, 517]
    off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
    qs, kcs, vcs, kts, vts, ms, refs = [], [], [], [], [], [], []
    for b in range(batch):
        q, kc, vc, kt, vt, mask = _attn_case(40 + b, T, Ls[b], Hq, Hkv, D, "bf16")
        refs.append(oracle.verify_attn(q, kc, vc, kt, vt, mask))
        qs.append(q); kcs.append(kc); vcs.append(vc); kts.append(kt); vts.append(vt); ms.append(mask)
    got = gu.gpu_attn(np.concatenate(qs), np.concatenate(kcs), np.concatenate(vcs),
                      np.concatenate(kts), np.concatenate(vts), np.stack(ms), off, batch, T, "bf16")
    for b in range(batch):
        assert attn_err(got[b], refs[b]) < 1e-2


def test_attn_key_range_with_many_tree_tiles():
    """Eight sequences of 1024 rows on eight KV heads: 256 workgroups with the key range unsplit, so
    each walks all 16 tree tiles (more than the kernel keeps mask words for on chip: the later ones
    are fetched as it goes), behind short, empty and ragged caches."""
    batch, T, Hq, Hkv, D = 8, 1024, 8, 8, 128
    Ls = [100, 0, 64, 7, 129, 1, 63, 200]
    off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
    rng = np.random.default_rng(1025)
    qs, kcs, vcs, kts, vts, ms = [], [], [], [], [], []
    for b in range(batch):
        q, kc, vc, kt, vt, mask = _attn_case(170 + b, T, Ls[b], Hq, Hkv, D, "bf16")
        qs.append(q); kcs.append(kc); vcs.append(vc); kts.append(kt); vts.append(vt); ms.append(mask)
    got = gu.gpu_attn(np.concatenate(qs), np.concatenate(kcs), np.concatenate(vcs),
                      np.concatenate(kts), np.concatenate(vts), np.stack(ms), off, batch, T, "bf16")
    for b in range(batch):
        nodes = np.concatenate([[0, 1, 63, 64, 511, 512, 513, 575, 576, 577, 960, 1022, 1023], rng.integers(0, T, 30)])
        pairs = np.stack([nodes, rng.integers(0, Hq, nodes.size)], axis=1).astype(np.int32)
        ref = oracle.verify_attn(qs[b], kcs[b], vcs[b], kts[b], vts[b], ms[b], pairs=pairs)
        assert attn_err(got[b][pairs[:, 0], pairs[:, 1]], ref) < 1e-2, b


def test_attn_randomized_shapes():
    # seeded sweep over head layouts, row counts, ragged batches and cache lengths (every tiling
    # and key split the planner can choose), checked on sampled (node, head) pairs
    rng = np.random.default_rng(123)
    worst = 0.0
    for case in range(30):
        Hkv = int(rng.choice([1, 2, 4, 8])); G = int(rng.choice([1, 2, 4, 8])); Hq = Hkv * G
        T = int(rng.choice([2, 9, 17, 33, 40, 65, 66, 100, 129, 200, 257, 258, 300, 513]))
        batch = int(rng.choice([1, 1, 1, 2, 3]))
        Ls = [int(rng.choice([0, 1, 63, 64, 65, 200, 1000, 2048, 4100])) for _ in range(batch)]
        off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
        qs, kcs, vcs, kts, vts, ms = [], [], [], [], [], []
        for b in range(batch):
            q, kc, vc, kt, vt = di.attn_tensors(5000 + 10 * case + b, T, Ls[b], Hq, Hkv, 128, "bf16")
            par, n = _random_tree(rng, T, int(rng.integers(1, T)) if rng.random() < 0.3 else None)
            qs.append(q); kcs.append(kc); vcs.append(vc); kts.append(kt); vts.append(vt)
            ms.append(oracle.ancestor_mask(par, n, T=T))
        got = gu.gpu_attn(np.concatenate(qs), np.concatenate(kcs), np.concatenate(vcs), np.concatenate(kts),
                          np.concatenate(vts), np.stack(ms), off, batch, T, "bf16")
        for b in range(batch):
            pairs = np.stack([rng.integers(0, T, 32), rng.integers(0, Hq, 32)], axis=1).astype(np.int32)
            pairs[0] = (T - 1, Hq - 1)
            pairs[1] = (0, 0)
            ref = oracle.verify_attn(qs[b], kcs[b], vcs[b], kts[b], vts[b], ms[b], pairs=pairs)
            err = attn_err(got[b][pairs[:, 0], pairs[:, 1]], ref)
            assert err < 1e-2, (case, b, T, Hq, Hkv, Ls, err)
            worst = max(worst, err)
    print(f"worst error over the sweep {worst:.2e}")


# ------------------------------------------------------------------------------- accept
def _tree_for_accept(seed, B, V, N, spike):
    x = _peaked_logits(seed, B, V, spike)
    tok, lp = oracle.topk(x, min(N, V))
    return tok, oracle.build_tree(tok, lp, N, root_token=3)


@pytest.mark.parametrize("V,N,spike,p", [(1024, 16, 6.0, 0.8), (151936, 64, 12.0, 0.9),
                                         (50001, 200, 10.0, 1.0), (30000, 40, 8.0, 0.0)])
def test_accept_matches_oracle(V, N, spike, p):
    B = 8
    tok, tree = _tree_for_accept(50, B, V, N, spike)
    plant = di.planted_tokens(51, tree["depth"], tok[:, 0], B, p=p)
    x = di.target_logits(51, N + 1, V, plant)
    o = oracle.accept(x, tree["tokens"], tree["parent"], tree["n_nodes"], B)
    g = gu.gpu_accept(x, tree["tokens"], tree["parent"], tree["depth"], [tree["n_nodes"]], B)
    assert np.array_equal(g["posterior"][0], o["posterior"])
    assert int(g["n_accepted"][0]) == o["n_accepted"]
    assert np.array_equal(g["path"][0], o["path"])
    assert int(g["bonus_token"][0]) == o["bonus"]
    print(f"V={V} N={N}: accepted {o['n_accepted']}")


def test_accept_branches_with_rank_above_zero_and_ties():
    B, V, N = 8, 5000, 60
    tok, tree = _tree_for_accept(60, B, V, N, 9.0)
    rng = np.random.default_rng(61)
    n = tree["n_nodes"]
    # walk target: the deepest node whose last rank is above zero (a branch off the top-1 chain)
    cands = [i for i in range(1, n + 1) if tree["rank"][i] > 0]
    leaf = max(cands, key=lambda i: tree["depth"][i])
    on_path = {}
    j = leaf
    while j > 0:
        on_path[int(tree["parent"][j])] = j
        j = int(tree["parent"][j])
    # every node's target token is one of its children's tokens: the path child on the path,
    # a random child elsewhere
    plant = np.full(N + 1, -1, np.int64)
    for i in range(n + 1):
        kids = [c for c in range(1, n + 1) if tree["parent"][c] == i]
        if i in on_path:
            plant[i] = tree["tokens"][on_path[i]]
        elif kids:
            plant[i] = tree["tokens"][rng.choice(kids)]
    x = di.target_logits(61, N + 1, V, plant)
    off = next(i for i in range(1, n + 1) if i not in on_path and i != leaf)
    x[off, :] = 0.0
    x[off, [4000, 77, 900]] = 3.0                     # tie: lowest id wins
    o = oracle.accept(x, tree["tokens"], tree["parent"], n, B)
    g = gu.gpu_accept(x, tree["tokens"], tree["parent"], tree["depth"], [n], B)
    assert o["posterior"][off] == 77
    assert o["n_accepted"] >= tree["depth"][leaf] >= 1
    assert np.array_equal(g["posterior"][0], o["posterior"])
    assert np.array_equal(g["path"][0], o["path"]) and int(g["bonus_token"][0]) == o["bonus"]
    assert int(g["n_accepted"][0]) == o["n_accepted"]


def test_accept_batched_with_padding_rows():
    B, V, N = 4, 3000, 30
    toks, trees, xs = [], [], []
    rng = np.random.default_rng(7)
    for b in range(3):
        K = 2 if b == 1 else 30            # b == 1: only 2+4+8+16 = 30 prefixes... use N=30 anyway
        xl = _peaked_logits(70 + b, B, V, 7.0)
        tok, lp = oracle.topk(xl, K)
        tree = oracle.build_tree(tok, lp, N, root_token=b)
        if b == 2:
            tree = oracle.build_tree(tok[:, :1], lp[:, :1], N, root_token=b)  # chain of 4, rest padding
        plant = di.planted_tokens(80 + b, tree["depth"], tok[:, 0], B, p=0.9)
        xs.append(di.target_logits(80 + b, N + 1, V, plant, batch_index=b))
        trees.append(tree)
    g = gu.gpu_accept(np.stack(xs), np.stack([t["tokens"] for t in trees]),
                      np.stack([t["parent"] for t in trees]), np.stack([t["depth"] for t in trees]),
                      [t["n_nodes"] for t in trees], B)
    for b in range(3):
        o = oracle.accept(xs[b], trees[b]["tokens"], trees[b]["parent"], trees[b]["n_nodes"], B)
        assert np.array_equal(g["posterior"][b], o["posterior"])
        assert np.array_equal(g["path"][b], o["path"])
        assert int(g["n_accepted"][b]) == o["n_accepted"] and int(g["bonus_token"][b]) == o["bonus"]


def test_compact_matches_oracle():
    import paper_2604_12989_amd as dd
    batch, T, B, Hkv, D = 2, 20, 6, 2, 128
    rng = np.random.default_rng(9)
    kt = di.round_to_bf16(rng.standard_normal((batch * T, Hkv, D)).astype(np.float32))
    vt = di.round_to_bf16(rng.standard_normal((batch * T, Hkv, D)).astype(np.float32))
    rows = 64
    kc = np.zeros((rows, Hkv, D), np.float32); vc = np.zeros((rows, Hkv, D), np.float32)
    path = np.array([[0, 3, 7, 12, -1, -1, -1], [0, -1, -1, -1, -1, -1, -1]], np.int32)
    nacc = np.array([3, 0], np.int32)
    dst = [10, 40]
    kcd, vcd = gu.bf16_dev(kc), gu.bf16_dev(vc)
    dd.compact(gu.bf16_dev(kt), gu.bf16_dev(vt), gu.to_dev(path), gu.to_dev(nacc), dst, batch, T, B,
               Hkv, D, kcd, vcd)
    torch.cuda.synchronize()
    for b in range(batch):
        oracle.compact(kt[b * T:(b + 1) * T], path[b], int(nacc[b]), kc, dst[b])
        oracle.compact(vt[b * T:(b + 1) * T], path[b], int(nacc[b]), vc, dst[b])
    assert np.array_equal(kcd.float().cpu().numpy(), kc)
    assert np.array_equal(vcd.float().cpu().numpy(), vc)


# ------------------------------------------------------------------------------- end to end
@pytest.mark.parametrize("config", [1, 2])
def test_end_to_end_chain(config):
    """topk -> build -> attention -> accept on the GPU, each stage fed by the GPU's own previous
    stage, against the oracle chain from the same logits."""
    c = di.CONFIGS[config]
    seed = di.config_seed(config)
    B, V, N = c["B"], c["V"], c["N"]
    K, T = min(N, V), N + 1
    x = di.draft_logits(seed, B, V)
    tok_o, lp_o = oracle.topk(x, K)
    tree = oracle.build_tree(tok_o, lp_o, N, root_token=11)
    mask_o = oracle.ancestor_mask(tree["parent"], tree["n_nodes"], T=T)
    plant = di.planted_tokens(seed, tree["depth"], tok_o[:, 0], B)
    tl = di.target_logits(seed, T, V, plant)
    acc_o = oracle.accept(tl, tree["tokens"], tree["parent"], tree["n_nodes"], B)

    tok_g, lp_g = gu.gpu_topk(x, K)
    assert np.array_equal(tok_g[0], tok_o)
    g = gu.gpu_build(tok_g[0], lp_g[0], N, 11)
    # the tree from the GPU's own log-probabilities must equal the oracle tree built from them
    o2 = oracle.build_tree(tok_g[0], lp_g[0], N, root_token=11)
    for key in ("tokens", "parent", "depth"):
        assert np.array_equal(g[key][0], o2[key])
    same_lp = np.array_equal(lp_g[0], lp_o)
    print(f"config {config}: lp bit-exact {same_lp}")
    if same_lp:
        assert np.array_equal(g["tokens"][0], tree["tokens"])
        assert np.array_equal(g["ancestor_mask"][0], mask_o)
    q, kc, vc, kt, vt = di.attn_tensors(seed, T, c["L"], c["Hq"], c["Hkv"], c["D"], c["dtype"])
    ref = oracle.verify_attn(q, kc, vc, kt, vt, g["ancestor_mask"][0])
    got = gu.gpu_attn(q, kc, vc, kt, vt, g["ancestor_mask"], [0, c["L"]], 1, T, c["dtype"])[0]
    assert attn_err(got, ref) < (1e-5 if c["dtype"] == "fp32" else 1e-2)
    ga = gu.gpu_accept(tl, g["tokens"][0], g["parent"][0], g["depth"][0], g["n_nodes"], B)
    if same_lp:
        assert np.array_equal(ga["path"][0], acc_o["path"])
        assert int(ga["n_accepted"][0]) == acc_o["n_accepted"]
        assert int(ga["bonus_token"][0]) == acc_o["bonus"]


def test_decoding_rounds_with_a_growing_cache():
    """Five consecutive rounds on one sequence: top-K, build, attention over the cache as it stands,
    accept, and compaction of the accepted path into the cache, whose new length the host reads back
    as a serving loop would.  Every round is compared with the oracle's round on the oracle's own
    cache; after the last round both caches hold the same rows."""
    import paper_2604_12989_amd as dd
    B, V, N, Hq, Hkv, D, L0, rounds = 8, 5000, 40, 8, 2, 128, 100, 5
    K, T = N, N + 1
    cap = L0 + rounds * (B + 1)
    _, kc0, vc0, _, _ = di.attn_tensors(900, 1, L0, Hq, Hkv, D, "bf16")
    cache_k_o = np.zeros((cap, Hkv, D), np.float32); cache_k_o[:L0] = kc0
    cache_v_o = np.zeros((cap, Hkv, D), np.float32); cache_v_o[:L0] = vc0
    cache_k_g = gu.bf16_dev(cache_k_o); cache_v_g = gu.bf16_dev(cache_v_o)
    ws = dd.Workspace(1, B, V, N, Hq, Hkv, D, cap)
    L, root, lengths = L0, 7, []
    for r in range(rounds):
        x = _peaked_logits(910 + r, B, V, 7.0)
        tok_o, lp_o = oracle.topk(x, K)
        tree = oracle.build_tree(tok_o, lp_o, N, root_token=root)
        mask_o = oracle.ancestor_mask(tree["parent"], tree["n_nodes"], T=T)
        q, _, _, kt, vt = di.attn_tensors(920 + r, T, 0, Hq, Hkv, D, "bf16")
        plant = di.planted_tokens(930 + r, tree["depth"], tok_o[:, 0], B, p=0.85)
        tl = di.target_logits(930 + r, T, V, plant)
        ref = oracle.verify_attn(q, cache_k_o[:L], cache_v_o[:L], kt, vt, mask_o)
        acc_o = oracle.accept(tl, tree["tokens"], tree["parent"], tree["n_nodes"], B)
        # the same round on the GPU, each stage fed by the stage before it
        tok_g, lp_g = dd.topk(gu.to_dev(x[None]), K, ws)
        tree_g = dd.build(tok_g, lp_g, N, gu.to_dev(np.array([root], np.int32)), ws)
        out = dd.verify_attn(gu.bf16_dev(q), cache_k_g, cache_v_g, gu.bf16_dev(kt), gu.bf16_dev(vt),
                             tree_g["ancestor_mask"], [0, L], 1, T, Hq, Hkv, D, 1.0 / np.sqrt(D), dd.DTYPE_BF16, ws)
        acc_g = dd.accept(gu.to_dev(tl[None]), tree_g["tokens"], tree_g["parent"], tree_g["depth"],
                          tree_g["n_nodes"], B, ws)
        kt_g, vt_g = gu.bf16_dev(kt), gu.bf16_dev(vt)
        dd.compact(kt_g, vt_g, acc_g["path"], acc_g["n_accepted"], [L], 1, T, B, Hkv, D, cache_k_g, cache_v_g)
        torch.cuda.synchronize()
        assert np.array_equal(tree_g["parent"].cpu().numpy()[0], tree["parent"]), r
        assert np.array_equal(tree_g["tokens"].cpu().numpy()[0], tree["tokens"]), r
        assert attn_err(out.float().cpu().numpy().reshape(T, Hq, D), ref) < 1e-2, r
        n_acc = int(acc_g["n_accepted"][0])            # the host learns the new length here
        assert n_acc == acc_o["n_accepted"], r
        assert np.array_equal(acc_g["path"].cpu().numpy()[0], acc_o["path"]), r
        assert int(acc_g["bonus_token"][0]) == acc_o["bonus"], r
        oracle.compact(kt, acc_o["path"], n_acc, cache_k_o, L)
        oracle.compact(vt, acc_o["path"], n_acc, cache_v_o, L)
        L += n_acc + 1
        root = acc_o["bonus"]
        lengths.append(n_acc)
    assert max(lengths) >= 2, lengths
    assert np.array_equal(cache_k_g.float().cpu().numpy()[:L], cache_k_o[:L])
    assert np.array_equal(cache_v_g.float().cpu().numpy()[:L], cache_v_o[:L])
    print(f"accepted per round {lengths}, cache grew from {L0} to {L} rows")


def test_batched_decoding_rounds_with_cache_spans():
    """Three sequences, each with its own region of the cache and room behind it; four rounds of
    attention (ddtree_verify_attn_spans), accept and in-place compaction, the regions listed out of
    order and with gaps.  Compared per sequence and round with the oracle on its own cache copy."""
    import paper_2604_12989_amd as dd
    batch, B, V, N, Hq, Hkv, D, rounds = 3, 6, 4000, 30, 8, 2, 128, 4
    K, T = N, N + 1
    room = rounds * (B + 1)
    L = [150, 0, 75]
    start = [500, 20, 900]                       # regions out of order, gaps between them
    rows = 900 + 75 + room + 10
    cache_k_o = np.zeros((rows, Hkv, D), np.float32); cache_v_o = np.zeros_like(cache_k_o)
    for s in range(batch):
        _, kc, vc, _, _ = di.attn_tensors(1200 + s, 1, L[s], Hq, Hkv, D, "bf16")
        cache_k_o[start[s]:start[s] + L[s]] = kc
        cache_v_o[start[s]:start[s] + L[s]] = vc
    cache_k_g = gu.bf16_dev(cache_k_o); cache_v_g = gu.bf16_dev(cache_v_o)
    ws = dd.Workspace(batch, B, V, N, Hq, Hkv, D, sum(L) + batch * room)
    roots = np.array([3, 4, 5], np.int32)
    total_accepted = 0
    for r in range(rounds):
        xs = np.stack([_peaked_logits(1300 + 10 * r + s, B, V, 7.0) for s in range(batch)])
        q, _, _, kt, vt = di.attn_tensors(1400 + r, batch * T, 0, Hq, Hkv, D, "bf16")
        trees, tls, refs, accs = [], [], [], []
        for s in range(batch):
            tok_o, lp_o = oracle.topk(xs[s], K)
            t = oracle.build_tree(tok_o, lp_o, N, root_token=int(roots[s]))
            m = oracle.ancestor_mask(t["parent"], t["n_nodes"], T=T)
            plant = di.planted_tokens(1500 + 10 * r + s, t["depth"], tok_o[:, 0], B, p=0.85, batch_index=s)
            tl = di.target_logits(1500 + 10 * r + s, T, V, plant, batch_index=s)
            sl = slice(start[s], start[s] + L[s])
            refs.append(oracle.verify_attn(q[s * T:(s + 1) * T], cache_k_o[sl], cache_v_o[sl],
                                           kt[s * T:(s + 1) * T], vt[s * T:(s + 1) * T], m))
            accs.append(oracle.accept(tl, t["tokens"], t["parent"], t["n_nodes"], B))
            trees.append(t); tls.append(tl)
        tok_g, lp_g = dd.topk(gu.to_dev(xs), K, ws)
        tree_g = dd.build(tok_g, lp_g, N, gu.to_dev(roots), ws)
        kt_g, vt_g = gu.bf16_dev(kt), gu.bf16_dev(vt)
        out = dd.verify_attn_spans(gu.bf16_dev(q), cache_k_g, cache_v_g, kt_g, vt_g, tree_g["ancestor_mask"],
                                   start, L, batch, T, Hq, Hkv, D, 1.0 / np.sqrt(D), dd.DTYPE_BF16, ws)
        acc_g = dd.accept(gu.to_dev(np.stack(tls)), tree_g["tokens"], tree_g["parent"], tree_g["depth"],
                          tree_g["n_nodes"], B, ws)
        dd.compact(kt_g, vt_g, acc_g["path"], acc_g["n_accepted"], [start[s] + L[s] for s in range(batch)],
                   batch, T, B, Hkv, D, cache_k_g, cache_v_g)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy().reshape(batch, T, Hq, D)
        n_acc = acc_g["n_accepted"].cpu().numpy()
        for s in range(batch):
            assert np.array_equal(tree_g["parent"][s].cpu().numpy(), trees[s]["parent"]), (r, s)
            assert attn_err(got[s], refs[s]) < 1e-2, (r, s)
            assert int(n_acc[s]) == accs[s]["n_accepted"], (r, s)
            assert np.array_equal(acc_g["path"][s].cpu().numpy(), accs[s]["path"]), (r, s)
            oracle.compact(kt[s * T:(s + 1) * T], accs[s]["path"], int(n_acc[s]), cache_k_o[start[s]:], L[s])
            oracle.compact(vt[s * T:(s + 1) * T], accs[s]["path"], int(n_acc[s]), cache_v_o[start[s]:], L[s])
            L[s] += int(n_acc[s]) + 1
            roots[s] = accs[s]["bonus"]
            total_accepted += int(n_acc[s])
    assert total_accepted >= rounds
    assert np.array_equal(cache_k_g.float().cpu().numpy(), cache_k_o)
    assert np.array_equal(cache_v_g.float().cpu().numpy(), cache_v_o)


# ------------------------------------------------------------------------------- sampled walk
# fp32 keys on the GPU against fp64 keys in the oracle: a selection is compared where the oracle's
# gap between winner and runner-up exceeds what fp32 can blur (logit/tau up to ~50 in magnitude:
# 2^-24 * 50 * a few operations, plus the hardware log2 at 1 ulp), and must be one of the two
# candidates where it does not.
SAMPLE_GAP_TOL = 2e-4


def _check_sampled(tl, tokens, parent, depth, n_nodes, B, tau, seed, batch_rows=None):
    got = gu.gpu_accept(tl, tokens, parent, depth, n_nodes, B, temperature=tau, seed=seed)
    x = tl if tl.ndim == 3 else tl[None]
    tok2 = np.asarray(tokens).reshape(x.shape[0], -1)
    par2 = np.asarray(parent).reshape(x.shape[0], -1)
    nn = np.asarray(n_nodes).reshape(-1)
    close = 0
    for b in range(x.shape[0]):
        T = x.shape[1]
        sel, run, gap = oracle.sample_tokens(x[b], int(nn[b]), tau, seed, first_row=b * T)
        post = got["posterior"][b]
        clear = gap > SAMPLE_GAP_TOL
        assert np.array_equal(post[clear], sel[clear])
        assert np.all((post[~clear] == sel[~clear]) | (post[~clear] == run[~clear]))
        close += int((~clear).sum())
        # the walk is exact given the GPU's own selection
        w = oracle.walk(post, tok2[b], par2[b], int(nn[b]), B)
        assert int(got["n_accepted"][b]) == w["n_accepted"]
        assert int(got["bonus_token"][b]) == w["bonus"]
        assert np.array_equal(got["path"][b], w["path"])
    return got, close


@pytest.mark.parametrize("tau", [0.05, 0.3, 1.0, 2.0, 25.0])
def test_accept_sampled_matches_oracle(tau):
    rng = np.random.default_rng(31)
    T, V, B = 65, 50001, 8
    n = T - 1
    par = np.full(T, -1, np.int32)
    depth = np.zeros(T, np.int32)
    for i in range(1, T):                       # a random tree no deeper than B
        ok = np.flatnonzero(depth[:i] < B)
        par[i] = i - 1 if (depth[i - 1] < B and rng.random() < 0.5) else rng.choice(ok)
        depth[i] = depth[par[i]] + 1
    tokens = rng.integers(0, V, T).astype(np.int32)
    tl = (rng.standard_normal((T, V)) * 2.0).astype(np.float32)
    got, close = _check_sampled(tl, tokens, par, depth, n, B, tau, seed=0xC0FFEE12345)
    print(f"tau={tau}: {close} of {n + 1} selections closer than the fp32 tolerance")
    # a different seed draws different tokens; the same seed repeats them
    again = gu.gpu_accept(tl, tokens, par, depth, n, B, temperature=tau, seed=0xC0FFEE12345)
    other = gu.gpu_accept(tl, tokens, par, depth, n, B, temperature=tau, seed=7)
    assert np.array_equal(again["posterior"], got["posterior"])
    if tau >= 0.3:   # (close to greedy, the largest logit wins whatever the seed)
        assert np.mean(other["posterior"][0][: n + 1] == got["posterior"][0][: n + 1]) < 0.5


@pytest.mark.parametrize("V", [5, 70, 300, 1000, 1027, 2500])
def test_accept_sampled_small_vocabularies(V):
    """Rows shorter than one round of a scan workgroup (fewer than 256 groups of four logits): some
    waves of the workgroup are only partly filled, or idle, from the first round on."""
    rng = np.random.default_rng(V)
    T, B = 40, 8
    n = T - 1
    par = np.full(T, -1, np.int32)
    depth = np.zeros(T, np.int32)
    for i in range(1, T):
        ok = np.flatnonzero(depth[:i] < B)
        par[i] = rng.choice(ok)
        depth[i] = depth[par[i]] + 1
    tokens = rng.integers(0, V, T).astype(np.int32)
    for rep in range(3):
        tl = (rng.standard_normal((T, V)) * 2.0).astype(np.float32)
        _check_sampled(tl, tokens, par, depth, n, B, float(rng.choice([0.3, 1.0, 2.0])),
                       seed=int(rng.integers(1, 2**62)))


def test_accept_sampled_walks_down_a_planted_chain_and_batches():
    # two sequences; in the first a chain of tokens dominates its rows (logit + 60: sampled with
    # probability ~1 at tau = 1), so the walk must descend it; the second has nothing planted
    rng = np.random.default_rng(32)
    T, V, B = 7, 20000, 6
    par = np.stack([np.arange(-1, T - 1), np.arange(-1, T - 1)]).astype(np.int32)   # chains
    depth = np.stack([np.arange(T), np.arange(T)]).astype(np.int32)
    tokens = rng.integers(0, V, (2, T)).astype(np.int32)
    tl = rng.standard_normal((2, T, V)).astype(np.float32)
    for i in range(4):
        tl[0, i, tokens[0, i + 1]] += 60.0
    got, _ = _check_sampled(tl, tokens, par, depth, np.array([T - 1, T - 1]), B, 1.0, seed=5)
    assert int(got["n_accepted"][0]) >= 4
    assert list(got["path"][0][:5]) == [0, 1, 2, 3, 4]


def test_accept_randomized_shapes():
    """Seeded sweep of the acceptance step over vocabulary sizes (one segment to many, ragged
    tails), budgets, batch sizes with different node counts per sequence, tree shapes (bushy to
    chains), how often the target agrees with the tree, and ties in the target's logits; greedy
    rule bit-exact, sampled rule checked as in the tests above."""
    rng = np.random.default_rng(777)
    accepted = []
    for case in range(36):
        V = int(rng.choice([2, 7, 1000, 4096, 12289, 50001, 151936]))
        B = int(rng.integers(1, 17))
        N = int(rng.choice([1, 2, 15, 64, 100, 256]))
        batch = int(rng.integers(1, 4)) if V * (N + 1) < 3e7 else 1
        spike = float(rng.uniform(0.0, 14.0))
        p = float(rng.choice([0.0, 0.5, 0.9, 1.0]))
        xs, trees = [], []
        for b in range(batch):
            xl = _peaked_logits(1000 + 10 * case + b, B, V, spike)
            K = int(min(V, N, rng.choice([1, 2, 4, N])))
            tok, lp = oracle.topk(xl, K)
            tree = oracle.build_tree(tok, lp, N, root_token=int(rng.integers(0, V)))
            plant = di.planted_tokens(2000 + case, tree["depth"], tok[:, 0], B, p=p)
            x = di.target_logits(2000 + case, N + 1, V, plant, batch_index=b)
            if case % 4 == 3:                    # exact ties: the first maximum has to win
                x = np.round(x * 2) / 2
            xs.append(x.astype(np.float32))
            trees.append(tree)
        stack = lambda k: np.stack([t[k] for t in trees])
        nn = [t["n_nodes"] for t in trees]
        g = gu.gpu_accept(np.stack(xs), stack("tokens"), stack("parent"), stack("depth"), nn, B)
        for b in range(batch):
            o = oracle.accept(xs[b], trees[b]["tokens"], trees[b]["parent"], trees[b]["n_nodes"], B)
            n = trees[b]["n_nodes"]
            what = (case, b, V, B, N, batch, n)
            assert np.array_equal(g["posterior"][b][:n], o["posterior"][:n]), what
            assert np.array_equal(g["path"][b], o["path"]), what
            assert int(g["n_accepted"][b]) == o["n_accepted"] and int(g["bonus_token"][b]) == o["bonus"], what
            accepted.append(o["n_accepted"])
        if case % 3 == 0 and V >= 1000:
            tau = float(rng.choice([0.3, 1.0, 2.0]))
            _check_sampled(np.stack(xs), stack("tokens"), stack("parent"), stack("depth"), nn, B, tau,
                           seed=int(rng.integers(1, 2**62)))
    print(f"accepted lengths seen: min {min(accepted)} max {max(accepted)}")


def test_accept_sampled_rejects_bad_temperature():
    import paper_2604_12989_amd as dd
    x = np.zeros((1, 3, 8), np.float32)
    z = np.zeros((1, 3), np.int32)
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(dd.DDTreeError):
            gu.gpu_accept(x, z, z, z, np.array([2]), 2, temperature=bad, seed=1)

