"""Stand-ins for a race detector on the GPU path, at the headline shapes: every stage is run 20
times on identical inputs and must give bit-identical outputs each time, and every output buffer
and the workspace sit between 4 KiB guard zones that must come back untouched.  A lost update, an
uninitialised read, a reduction whose order depends on timing or a store past the end of a buffer
shows up here even when a single run happens to match the oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import ddtree_inputs as di  # noqa: E402
import oracle  # noqa: E402

if torch.cuda.is_available():
    import paper_2604_12989_amd as dd  # noqa: E402
    from tests import gpu_util as gu  # noqa: E402

GUARD = 4096
PATTERN = 0xA5
REPEATS = 20


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests selected but no GPU is visible")


class Guarded:
    """A device buffer with a guard zone of GUARD bytes on either side of the payload."""

    def __init__(self, shape, dtype):
        self.shape, self.dtype = tuple(shape), dtype
        self.nbytes = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        pad = (-self.nbytes) % 256
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), PATTERN, dtype=torch.uint8, device=gu.DEV)
        assert self.raw.data_ptr() % 256 == 0
        self.tensor = self.raw[GUARD:GUARD + self.nbytes].view(dtype).view(self.shape)
        self.tail = GUARD + self.nbytes

    def check(self, what):
        raw = self.raw.cpu().numpy()
        assert (raw[:GUARD] == PATTERN).all(), f"{what}: bytes before the buffer were written"
        assert (raw[self.tail:] == PATTERN).all(), f"{what}: bytes behind the buffer were written"

    def bits(self):
        return self.raw[GUARD:self.tail].cpu().numpy().copy()


class GuardedWorkspace:
    """Scratch of exactly ddtree_workspace_bytes between two guard zones (duck-types dd.Workspace)."""

    def __init__(self, *shape_args):
        n = dd.workspace_bytes(*shape_args)
        assert n > 0
        self.g = Guarded((n,), torch.uint8)
        self.nbytes = n
        self.ptr = self.g.tensor.data_ptr()
        assert self.ptr % 256 == 0

    def check(self):
        self.g.check("workspace")


def _repeat(run, outputs, ws, what):
    """run() REPEATS times; outputs: dict name -> Guarded.  Returns the (common) result bits."""
    first = None
    for r in range(REPEATS):
        for g in outputs.values():           # every run starts from outputs full of the pattern
            g.raw[GUARD:g.tail] = PATTERN
        run()
        torch.cuda.synchronize()
        bits = {k: g.bits() for k, g in outputs.items()}
        if first is None:
            first = bits
        else:
            for k in bits:
                assert np.array_equal(bits[k], first[k]), f"{what}: output {k} of run {r} differs from run 0"
    for k, g in outputs.items():
        g.check(f"{what}.{k}")
    ws.check()
    return first


def test_repeat_runs_and_guard_zones_at_the_headline_shapes():
    c = di.CONFIGS[3]
    seed = di.config_seed(3, 1)
    B, V, N, Hq, Hkv, D, L = c["B"], c["V"], c["N"], c["Hq"], c["Hkv"], c["D"], c["L"]
    K, T, W = N, N + 1, (N + 1 + 63) // 64
    i32, f32 = torch.int32, torch.float32
    ws = GuardedWorkspace(1, B, V, N, Hq, Hkv, D, L)

    # a peaked drafter, so that the tree has depth and the level construction, masks and walk do work
    x = di.peaked_draft_logits(seed, B, V, 0.8)
    logits = gu.to_dev(x[None])
    tok, lp = Guarded((1, B, K), i32), Guarded((1, B, K), f32)
    _repeat(lambda: dd.topk(logits, K, ws, tok.tensor, lp.tensor), dict(tok=tok, lp=lp), ws, "topk")
    tok_o, lp_o = oracle.topk(x, K)
    assert np.array_equal(tok.tensor.cpu().numpy()[0], tok_o)

    tree = dict(tokens=Guarded((1, T), i32), parent=Guarded((1, T), i32), depth=Guarded((1, T), i32),
                rank=Guarded((1, T), i32), node_score=Guarded((1, T), f32),
                ancestor_mask=Guarded((1, T, W), torch.int64), n_nodes=Guarded((1,), i32))
    root = gu.to_dev(np.array([7], np.int32))
    views = {k: g.tensor for k, g in tree.items()}
    for algo in (dd.BUILD_AUTO, dd.BUILD_POPS, dd.BUILD_LEVELS):
        dd.set_build_algorithm(algo)
        try:
            _repeat(lambda: dd.build(tok.tensor, lp.tensor, N, root, ws, views), tree, ws, f"build[{algo}]")
        finally:
            dd.set_build_algorithm(dd.BUILD_AUTO)
    tr = oracle.build_tree(tok_o, lp.tensor.cpu().numpy()[0], N, 7)
    assert np.array_equal(views["parent"].cpu().numpy()[0], tr["parent"])
    assert tr["depth"].max() >= 8

    q, kc, vc, kt, vt = di.attn_tensors(seed, T, L, Hq, Hkv, D, "bf16")
    dq, dkc, dvc, dkt, dvt = (gu.bf16_dev(a) for a in (q, kc, vc, kt, vt))
    out = Guarded((T, Hq, D), torch.bfloat16)
    _repeat(lambda: dd.verify_attn(dq, dkc, dvc, dkt, dvt, views["ancestor_mask"], [0, L], 1, T, Hq, Hkv, D,
                                   1.0 / np.sqrt(D), dd.DTYPE_BF16, ws, out.tensor),
            dict(out=out), ws, "verify_attn")

    plant = di.planted_tokens(seed, tr["depth"], tok_o[:, 0], B, p=0.9)
    tl = gu.to_dev(di.target_logits(seed, T, V, plant)[None])
    acc = dict(path=Guarded((1, B + 1), i32), n_accepted=Guarded((1,), i32), bonus_token=Guarded((1,), i32),
               posterior=Guarded((1, T), i32))
    av = {k: g.tensor for k, g in acc.items()}
    _repeat(lambda: dd.accept(tl, views["tokens"], views["parent"], views["depth"], views["n_nodes"], B, ws, av),
            acc, ws, "accept")
    _repeat(lambda: dd.accept(tl, views["tokens"], views["parent"], views["depth"], views["n_nodes"], B, ws, av,
                              temperature=0.7, seed=99), acc, ws, "accept_sampled")
    _repeat(lambda: dd.accept_noalloc(tl, views["tokens"], views["parent"], views["depth"], views["n_nodes"], B, av),
            acc, ws, "accept_noalloc")


def test_repeat_runs_batched_ragged():
    """The batched path (one-workgroup-per-row top-K, several trees per launch, ragged attention with
    its XCD-balanced work list): 20 identical runs, guard zones intact."""
    batch, B, V, N, Hq, Hkv, D = 8, 16, 20000, 64, 16, 4, 128
    K, T, W = N, N + 1, (N + 1 + 63) // 64
    i32, f32 = torch.int32, torch.float32
    Ls = [700, 64, 2100, 0, 1500, 333, 1024, 65]
    off = np.concatenate([[0], np.cumsum(Ls)]).astype(np.int32)
    ws = GuardedWorkspace(batch, B, V, N, Hq, Hkv, D, int(off[-1]))
    xs = np.stack([di.peaked_draft_logits(500 + s, B, V, 0.5 + 0.05 * s) for s in range(batch)])
    logits = gu.to_dev(xs)
    tok, lp = Guarded((batch, B, K), i32), Guarded((batch, B, K), f32)
    _repeat(lambda: dd.topk(logits, K, ws, tok.tensor, lp.tensor), dict(tok=tok, lp=lp), ws, "topk")
    tree = dict(tokens=Guarded((batch, T), i32), parent=Guarded((batch, T), i32), depth=Guarded((batch, T), i32),
                rank=Guarded((batch, T), i32), node_score=Guarded((batch, T), f32),
                ancestor_mask=Guarded((batch, T, W), torch.int64), n_nodes=Guarded((batch,), i32))
    views = {k: g.tensor for k, g in tree.items()}
    roots = gu.to_dev(np.arange(batch, dtype=np.int32))
    _repeat(lambda: dd.build(tok.tensor, lp.tensor, N, roots, ws, views), tree, ws, "build")
    q, _, _, kt, vt = di.attn_tensors(77, batch * T, 0, Hq, Hkv, D, "bf16")
    _, kc, vc, _, _ = di.attn_tensors(78, 1, int(off[-1]), Hq, Hkv, D, "bf16")
    dq, dkc, dvc, dkt, dvt = (gu.bf16_dev(a) for a in (q, kc, vc, kt, vt))
    out = Guarded((batch * T, Hq, D), torch.bfloat16)
    _repeat(lambda: dd.verify_attn(dq, dkc, dvc, dkt, dvt, views["ancestor_mask"], off, batch, T, Hq, Hkv, D,
                                   1.0 / np.sqrt(D), dd.DTYPE_BF16, ws, out.tensor),
            dict(out=out), ws, "verify_attn")
    tl = gu.to_dev(np.stack([di.target_logits(600 + s, T, V, np.full(T, -1)) for s in range(batch)]))
    acc = dict(path=Guarded((batch, B + 1), i32), n_accepted=Guarded((batch,), i32),
               bonus_token=Guarded((batch,), i32), posterior=Guarded((batch, T), i32))
    av = {k: g.tensor for k, g in acc.items()}
    _repeat(lambda: dd.accept(tl, views["tokens"], views["parent"], views["depth"], views["n_nodes"], B, ws, av),
            acc, ws, "accept")
