"""Seeded synthetic inputs for the DDTree draft-tree step.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no softmax, no top-k, no tree, no attention), so both the
CPU oracle's tests and the GPU library's tests can feed from it without sharing
anything else.  Numbers come from a counter-based generator (splitmix64 of
seed/stream/counter, Box-Muller in fp64), so a given (seed, stream) always
yields the same bytes whatever the numpy version.

Workload recipe (stands in for the drafter / target model of the paper's
experiments, which need trained checkpoints):
  draft logits   row d (0-based): 3.0 * 0.85**d * z, z ~ N(0,1), then +4 on one
                 seeded token per row -- confident early positions, flatter late ones
  q, k, v        N(0,1), rounded to bf16 (round-to-nearest-even) in bf16 configs
  target logits  N(0,1); the caller names, per row, the token on which a value
                 of 10 is planted (so that row's argmax is known by construction)
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)

# The five workload shapes (B draft rows, V vocabulary, N node budget, ...).
CONFIGS = {
    1: dict(name="tiny", batch=1, B=8, V=1024, N=16, Hq=2, Hkv=1, D=64, L=128, dtype="fp32"),
    2: dict(name="n64_l2k", batch=1, B=16, V=151936, N=64, Hq=32, Hkv=8, D=128, L=2048,
            dtype="bf16"),
    3: dict(name="n256_l8k", batch=1, B=16, V=151936, N=256, Hq=32, Hkv=8, D=128, L=8192,
            dtype="bf16"),
    4: dict(name="n512_l32k", batch=1, B=16, V=151936, N=512, Hq=32, Hkv=8, D=128, L=32768,
            dtype="bf16"),
    5: dict(name="batch16_ragged", batch=16, B=16, V=151936, N=128, Hq=64, Hkv=8, D=128,
            L=(1024, 8192), dtype="bf16"),
}


def config_seed(config: int, trial: int = 0) -> int:
    return 12989000 + 100 * int(config) + int(trial)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _key(seed: int, stream: int) -> np.uint64:
    k = _splitmix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64))
    k = _splitmix64(k ^ np.uint64(stream & 0xFFFFFFFFFFFFFFFF))
    return k[0]


def bits64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words: word i = mix(mix(key + i))."""
    ctr = np.arange(offset, offset + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _splitmix64(_splitmix64((ctr + _key(seed, stream)) & _M64))


def uniform(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n doubles in (0, 1)."""
    return ((bits64(seed, stream, n, offset) >> np.uint64(11)).astype(np.float64) + 0.5) * (
        1.0 / 9007199254740992.0)


def randint(seed: int, stream: int, n: int, hi: int) -> np.ndarray:
    """n integers in [0, hi)."""
    return np.minimum((uniform(seed, stream, n) * hi).astype(np.int64), hi - 1)


def normal(seed: int, stream: int, n: int) -> np.ndarray:
    """n standard normals (fp64), Box-Muller on pairs of uniforms, generated in chunks."""
    out = np.empty(n, np.float64)
    chunk = 1 << 22
    for start in range(0, n, chunk):
        m = min(chunk, n - start)
        half = (m + 1) // 2
        # pair p of this chunk uses uniforms 2*(start/2 + p) and +1; start is even
        u = uniform(seed, stream, 2 * half, offset=start)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        th = (2.0 * np.pi) * u[1::2]
        z = np.empty(2 * half, np.float64)
        z[0::2] = r * np.cos(th)
        z[1::2] = r * np.sin(th)
        out[start:start + m] = z[:m]
    return out


# ---------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


# ---------------------------------------------------------------- workload tensors
def draft_logits(seed: int, B: int, V: int, batch_index: int = 0) -> np.ndarray:
    """fp32 [B, V] drafter logits with a depth-decaying scale and one +4 spike per row."""
    stream = 1000 + 10 * batch_index
    z = normal(seed, stream, B * V).reshape(B, V)
    scale = 3.0 * 0.85 ** np.arange(B, dtype=np.float64)
    x = z * scale[:, None]
    spike = randint(seed, stream + 1, B, V)
    x[np.arange(B), spike] += 4.0
    return x.astype(np.float32)


def peaked_draft_logits(seed: int, B: int, V: int, p: float, batch_index: int = 0) -> np.ndarray:
    """draft_logits() with the spiked token of every row raised until it holds probability p of
    that row (a confident drafter: trees then reach the last position).  The height comes from
    the log-sum-exp of the row's other entries; that calibrates the input distribution and is
    not a step of the method."""
    x = draft_logits(seed, B, V, batch_index).astype(np.float64)
    spike = randint(seed, 1000 + 10 * batch_index + 1, B, V)
    for d in range(B):
        others = np.delete(x[d], spike[d])
        m = others.max()
        x[d, spike[d]] = m + np.log(np.exp(others - m).sum()) + np.log(p / (1.0 - p))
    return x.astype(np.float32)


def attn_tensors(seed: int, T: int, L: int, Hq: int, Hkv: int, D: int, dtype: str,
                 batch_index: int = 0):
    """q [T,Hq,D], k_cache/v_cache [L,Hkv,D], k_tree/v_tree [T,Hkv,D] as fp32 arrays.

    With dtype == "bf16" every value is rounded to bf16 first (still stored as fp32);
    use f32_to_bf16_bits() to get the 16-bit patterns for the device."""
    stream = 2000 + 10 * batch_index
    shapes = [(T, Hq, D), (L, Hkv, D), (L, Hkv, D), (T, Hkv, D), (T, Hkv, D)]
    out = []
    for s, shp in enumerate(shapes):
        x = normal(seed, stream + s, int(np.prod(shp))).astype(np.float32).reshape(shp)
        if dtype == "bf16":
            x = round_to_bf16(x)
        out.append(x)
    return tuple(out)


def plant_draws(seed: int, T: int, batch_index: int = 0) -> np.ndarray:
    """One uniform per verifier row; the caller plants when draw < p**depth."""
    return uniform(seed, 3000 + 10 * batch_index, T)


def target_logits(seed: int, T: int, V: int, plant_tok, batch_index: int = 0,
                  plant_value: float = 10.0) -> np.ndarray:
    """fp32 [T, V] ~ N(0,1); row i gets plant_value at column plant_tok[i] when plant_tok[i] >= 0."""
    x = normal(seed, 3001 + 10 * batch_index, T * V).astype(np.float32).reshape(T, V)
    plant_tok = np.asarray(plant_tok)
    rows = np.nonzero(plant_tok >= 0)[0]
    x[rows, plant_tok[rows]] = np.float32(plant_value)
    return x


def planted_tokens(seed: int, depth, top1_tok, B: int, p: float = 0.8,
                   batch_index: int = 0) -> np.ndarray:
    """Which token to plant in each verifier row: the drafter's most likely token for the
    next position (top1_tok[depth]) with probability p**depth, else none (-1).  depth < 0
    marks a padding row.  Pure selection; the tree's depth array is supplied by the caller."""
    depth = np.asarray(depth, np.int64)
    T = depth.shape[0]
    u = plant_draws(seed, T, batch_index)
    ok = (depth >= 0) & (depth < B) & (u < np.power(p, np.maximum(depth, 0)))
    tok = np.full(T, -1, np.int64)
    tok[ok] = np.asarray(top1_tok)[depth[ok]]
    return tok


def ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Per-sequence context lengths, uniform on [lo, hi]."""
    return lo + randint(seed, 4000, batch, hi - lo + 1)
