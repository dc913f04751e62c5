"""The seeded generators: determinism, distribution shape, bf16 rounding."""
import numpy as np
import torch

import ddtree_inputs as di


def test_streams_are_reproducible_and_chunk_independent():
    a = di.normal(42, 7, 10)
    b = di.normal(42, 7, (1 << 22) + 10)
    assert np.array_equal(a, b[:10])
    assert not np.array_equal(a, di.normal(42, 8, 10))
    assert abs(b.mean()) < 3e-3 and abs(b.std() - 1) < 3e-3


def test_bf16_rounding_matches_torch():
    x = di.normal(1, 1, 10000).astype(np.float32)
    ours = di.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(di.f32_to_bf16_bits(di.round_to_bf16(x)), ours)


def test_draft_logits_law():
    x = di.draft_logits(di.config_seed(3), 16, 4096)
    sd = x.std(axis=1)
    want = 3.0 * 0.85 ** np.arange(16)
    assert np.all(np.abs(sd / want - 1) < 0.08)
    assert x.dtype == np.float32 and np.isfinite(x).all()


def test_planting():
    depth = np.array([0, 1, 1, 2, 16, -1])
    top1 = np.arange(100, 116)
    tok = di.planted_tokens(5, depth, top1, B=16, p=1.0)
    assert tok.tolist() == [100, 101, 101, 102, -1, -1]
    x = di.target_logits(5, 6, 512, tok)
    assert x.argmax(axis=1)[:4].tolist() == [100, 101, 101, 102]
