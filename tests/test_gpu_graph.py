"""The whole step recorded into a HIP graph and replayed: the entry points only launch kernels on the
caller's stream (no allocation, no synchronisation, no memset or copy nodes), so a serving loop may
capture topk -> build -> verify-attention -> accept -> compact once and replay it.  Every replay, with
eager work and synchronisations between them and new contents in the same input buffers, has to give
what the eager calls give on those inputs (which the parity tests hold to the oracle)."""
import numpy as np
import pytest
import torch

import ddtree_inputs as di
import oracle

pytestmark = pytest.mark.gpu


def _inputs(seed, B, V, T, L, Hq, Hkv, D):
    from tests import gpu_util as gu
    x = di.draft_logits(seed, B, V)
    x[np.arange(B), (np.arange(B) * 31 + seed) % V] += 6.0
    q, kc, vc, kt, vt = di.attn_tensors(seed, T, L, Hq, Hkv, D, "bf16")
    tok_o, lp_o = oracle.topk(x, T - 1)
    tree_o = oracle.build_tree(tok_o, lp_o, T - 1, 5)
    plant = di.planted_tokens(seed, tree_o["depth"], tok_o[:, 0], B, p=0.9)   # the walk accepts a few nodes
    tl = di.target_logits(seed, T, V, plant)
    return dict(x=gu.to_dev(x[None]), q=gu.bf16_dev(q), kc=gu.bf16_dev(kc), vc=gu.bf16_dev(vc),
                kt=gu.bf16_dev(kt), vt=gu.bf16_dev(vt), tl=gu.to_dev(tl[None]))


def test_step_replays_from_a_captured_graph():
    import paper_2604_12989_amd as dd
    B, V, N, Hq, Hkv, D, L = 8, 20000, 96, 8, 2, 128, 700
    K, T = N, N + 1
    dev = "cuda:0"
    sets = [_inputs(100 + i, B, V, T, L, Hq, Hkv, D) for i in range(3)]
    ws = dd.Workspace(1, B, V, N, Hq, Hkv, D, L)
    root = torch.tensor([5], dtype=torch.int32, device=dev)
    scale = 1.0 / np.sqrt(D)

    # static buffers the graph reads and writes; the caches have room for the appended rows
    cur = {k: torch.empty_like(v) for k, v in sets[0].items()}
    cache_k = torch.zeros((L + B + 1, Hkv, D), dtype=torch.bfloat16, device=dev)
    cache_v = torch.zeros_like(cache_k)
    tok = torch.empty((1, B, K), dtype=torch.int32, device=dev)
    lp = torch.empty((1, B, K), dtype=torch.float32, device=dev)
    tree = dd.build(*dd.topk(sets[0]["x"], K, ws), N, root)       # allocates the output dict once
    att = torch.empty_like(sets[0]["q"])
    acc = dd.accept(sets[0]["tl"], tree["tokens"], tree["parent"], tree["depth"], tree["n_nodes"], B, ws)

    def load(i):
        for k in cur:
            cur[k].copy_(sets[i][k])
        cache_k.zero_()
        cache_v.zero_()
        cache_k[:L].copy_(cur["kc"])
        cache_v[:L].copy_(cur["vc"])

    def step():
        dd.topk(cur["x"], K, ws, tok, lp)
        dd.build(tok, lp, N, root, out=tree)
        dd.verify_attn(cur["q"], cache_k, cache_v, cur["kt"], cur["vt"], tree["ancestor_mask"], [0, L], 1,
                       T, Hq, Hkv, D, scale, dd.DTYPE_BF16, ws, out=att)
        dd.accept(cur["tl"], tree["tokens"], tree["parent"], tree["depth"], tree["n_nodes"], B, ws, out=acc)
        dd.compact(cur["kt"], cur["vt"], acc["path"], acc["n_accepted"], [L], 1, T, B, Hkv, D, cache_k, cache_v)

    def snapshot():
        torch.cuda.synchronize()
        got = dict(tok=tok, lp=lp, att=att, cache_k=cache_k, cache_v=cache_v)
        got.update({f"tree_{k}": v for k, v in tree.items()})
        got.update({f"acc_{k}": v for k, v in acc.items() if v is not None})
        return {k: v.clone() for k, v in got.items()}

    eager = []
    for i in range(3):
        load(i)
        step()
        eager.append(snapshot())
    assert int(eager[0]["acc_n_accepted"][0]) >= 1
    assert not torch.equal(eager[0]["tree_tokens"], eager[1]["tree_tokens"])

    load(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for n_replay, i in enumerate((1, 2, 0, 1)):
        load(i)                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for k, ref in eager[i].items():
            if k in ("tree_depth", "tree_rank", "tree_tokens", "tree_parent", "tree_node_score",
                     "tree_ancestor_mask", "acc_posterior"):
                n = int(eager[i]["tree_n_nodes"][0])
                assert torch.equal(got[k][:, :n], ref[:, :n]), (n_replay, i, k)
            elif k in ("att", "lp"):
                assert torch.equal(got[k].view(torch.int16 if k == "att" else torch.int32),
                                   ref.view(torch.int16 if k == "att" else torch.int32)), (n_replay, i, k)
            else:
                assert torch.equal(got[k], ref), (n_replay, i, k)
