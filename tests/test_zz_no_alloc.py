"""ddtree_accept_noalloc (scratch in the library's static device array) against ddtree_accept
(scratch in the caller's workspace): same outputs, bit for bit, on two calls in a row, the second
with a smaller input -- the array still holds the first call's partials then."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import ddtree_inputs as di  # noqa: E402
import oracle  # noqa: E402

if torch.cuda.is_available():
    import paper_2604_12989_amd as dd  # noqa: E402
    from tests import gpu_util as gu  # noqa: E402


def _case(seed, B, V, N, spike):
    x = di.draft_logits(seed, B, V)
    x[np.arange(B), (np.arange(B) * 131 + 7) % V] += spike
    tok, lp = oracle.topk(x, min(N, V))
    tr = oracle.build_tree(tok, lp, N, 3)
    plant = di.planted_tokens(seed, tr["depth"], tok[:, 0], B, p=0.95)
    tl = di.target_logits(seed, N + 1, V, plant)
    return tr, tl


def _run_both(tr, tl, B):
    T, V = tl.shape
    f = lambda a: gu.to_dev(np.asarray(a, np.int32).reshape(1, -1))
    tokens, parent, depth = f(tr["tokens"]), f(tr["parent"]), f(tr["depth"])
    n_nodes = gu.to_dev(np.array([tr["n_nodes"]], np.int32))
    logits = gu.to_dev(tl[None])
    ws = gu.ws_for(1, B, V, T - 1)
    ref = dd.accept(logits, tokens, parent, depth, n_nodes, B, ws)
    out = {k: torch.full_like(v, -7) for k, v in ref.items()}
    dd.accept_noalloc(logits, tokens, parent, depth, n_nodes, B, out)
    torch.cuda.synchronize()
    for k in ref:
        assert np.array_equal(out[k].cpu().numpy(), ref[k].cpu().numpy()), k
    return {k: v.cpu().numpy()[0] for k, v in out.items()}


def test_noalloc_accept_matches_the_workspace_entry_point_twice():
    assert torch.cuda.is_available(), "GPU tests selected but no GPU is visible"
    B = 8
    # first call: 130 rows of 50001 logits (several segments per row)
    tr1, tl1 = _case(901, B, 50001, 129, 9.0)
    got1 = _run_both(tr1, tl1, B)
    o1 = oracle.accept(tl1, tr1["tokens"], tr1["parent"], tr1["n_nodes"], B)
    assert np.array_equal(got1["posterior"], o1["posterior"])
    assert np.array_equal(got1["path"], o1["path"]) and int(got1["n_accepted"]) == o1["n_accepted"]
    assert int(got1["bonus_token"]) == o1["bonus"]
    # second call, smaller in rows and in vocabulary: the array keeps the first call's partials
    tr2, tl2 = _case(902, B, 9000, 20, 7.0)
    got2 = _run_both(tr2, tl2, B)
    o2 = oracle.accept(tl2, tr2["tokens"], tr2["parent"], tr2["n_nodes"], B)
    assert np.array_equal(got2["posterior"], o2["posterior"])
    assert np.array_equal(got2["path"], o2["path"]) and int(got2["n_accepted"]) == o2["n_accepted"]
    assert int(got2["bonus_token"]) == o2["bonus"]
    print(f"accepted {o1['n_accepted']} then {o2['n_accepted']}")
