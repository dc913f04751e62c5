"""CPU oracle for the DDTree draft-tree step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``ddtree_oracle.c`` (plain C, fp64 where floating
point matters).  Only tests, the smoke check and the benchmark's CPU-baseline
leg may import this package; the GPU library never does, and the two share no
code.  Every function cites the passage of the paper it follows in the C file.

Pins (what each function is checked against, see tests/test_oracle_*.py):
  topk          full sort + library log-softmax, sum-to-one, shift invariance,
                engineered duplicate logits
  build         brute-force enumeration of all prefixes (Proposition 2),
                Proposition 1 by enumeration of all sequences, hand-worked tree,
                structural invariants from the proof of Proposition 3
  ancestor_mask chain / star closed forms, popcount = depth + 1
  verify_attn   chain tree == causal attention (library SDPA), dense-mask SDPA,
                closed forms (q = 0, single visible key)
  accept        the walk drawn in Figure 1b, chain closed forms
  compact       gather identity
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ddtree_oracle.c")
_LIB = os.path.join(_HERE, "libddtree_oracle.so")

_lib = None

# how the oracle is compiled (reported next to its timings by the benchmark)
CFLAGS = ["-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host only).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", *CFLAGS, "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB + ".tmp", "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("oracle_topk", "oracle_build", "oracle_ancestor_mask", "oracle_verify_attn",
                     "oracle_accept", "oracle_compact", "oracle_num_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def topk(logits, K, return_lse=False):
    """logits fp32 [B,V] -> (tok int32 [B,K], lp fp32 [B,K])."""
    logits = _c(logits, np.float32)
    B, V = logits.shape
    tok = np.empty((B, K), np.int32)
    lp = np.empty((B, K), np.float32)
    lse = np.empty((B,), np.float64)
    rc = _load().oracle_topk(_p(logits, ctypes.c_float), B, V, int(K), _p(tok, ctypes.c_int32),
                             _p(lp, ctypes.c_float), _p(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_topk failed: {rc}")
    return (tok, lp, lse) if return_lse else (tok, lp)


def build_tree(tok, lp, N, root_token=0):
    """Algorithm 1.  Returns dict(tokens, parent, depth, rank, score, n_nodes, max_heap)."""
    tok = _c(tok, np.int32)
    lp = _c(lp, np.float32)
    B, K = tok.shape
    assert lp.shape == (B, K)
    T = N + 1
    out = dict(tokens=np.empty(T, np.int32), parent=np.empty(T, np.int32),
               depth=np.empty(T, np.int32), rank=np.empty(T, np.int32),
               score=np.empty(T, np.float32))
    n_nodes = ctypes.c_int32(0)
    max_heap = ctypes.c_int32(0)
    rc = _load().oracle_build(_p(tok, ctypes.c_int32), _p(lp, ctypes.c_float), B, K, int(N),
                              ctypes.c_int32(int(root_token)),
                              _p(out["tokens"], ctypes.c_int32), _p(out["parent"], ctypes.c_int32),
                              _p(out["depth"], ctypes.c_int32), _p(out["rank"], ctypes.c_int32),
                              _p(out["score"], ctypes.c_float), ctypes.byref(n_nodes),
                              ctypes.byref(max_heap))
    if rc != 0:
        raise ValueError(f"oracle_build failed: {rc}")
    out["n_nodes"] = int(n_nodes.value)
    out["max_heap"] = int(max_heap.value)
    return out


def ancestor_mask(parent, n_nodes, T=None):
    """parent int32 [>=n_nodes+1] -> uint64 [T, ceil(T/64)]."""
    parent = _c(parent, np.int32)
    T = int(T if T is not None else parent.shape[0])
    W = (T + 63) // 64
    mask = np.empty((T, W), np.uint64)
    rc = _load().oracle_ancestor_mask(_p(parent, ctypes.c_int32), int(n_nodes), T,
                                      _p(mask, ctypes.c_uint64))
    if rc != 0:
        raise ValueError(f"oracle_ancestor_mask failed: {rc}")
    return mask


def verify_attn(q, k_cache, v_cache, k_tree, v_tree, mask, scale=None, pairs=None):
    """Tree attention in fp64.  q [T,Hq,D], k/v_cache [L,Hkv,D], k/v_tree [T,Hkv,D]
    (fp32 arrays; bf16 inputs are passed already rounded and up-cast).
    Returns float64 [T,Hq,D], or [n_pairs,D] when pairs (int32 [n,2] of (node, head)) is given."""
    q = _c(q, np.float32)
    T, Hq, D = q.shape
    k_tree = _c(k_tree, np.float32)
    v_tree = _c(v_tree, np.float32)
    Hkv = k_tree.shape[1]
    k_cache = _c(k_cache, np.float32).reshape(-1, Hkv, D)
    v_cache = _c(v_cache, np.float32).reshape(-1, Hkv, D)
    L = k_cache.shape[0]
    assert v_cache.shape == (L, Hkv, D) and k_tree.shape == (T, Hkv, D) == v_tree.shape
    mask = _c(mask, np.uint64)
    assert mask.shape == (T, (T + 63) // 64)
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    if pairs is not None:
        pairs = _c(pairs, np.int32).reshape(-1, 2)
        n_pairs = pairs.shape[0]
        out = np.empty((n_pairs, D), np.float64)
    else:
        n_pairs = 0
        out = np.empty((T, Hq, D), np.float64)
    rc = _load().oracle_verify_attn(_p(q, ctypes.c_float), _p(k_cache, ctypes.c_float),
                                    _p(v_cache, ctypes.c_float), _p(k_tree, ctypes.c_float),
                                    _p(v_tree, ctypes.c_float), _p(mask, ctypes.c_uint64), L, T,
                                    Hq, Hkv, D, ctypes.c_double(float(scale)),
                                    _p(pairs, ctypes.c_int32), n_pairs, _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_verify_attn failed: {rc}")
    return out


def accept(target_logits, tokens, parent, n_nodes, B):
    """Greedy walk.  Returns dict(path int32 [B+1], n_accepted, bonus, posterior int32 [T])."""
    target_logits = _c(target_logits, np.float32)
    T, V = target_logits.shape
    tokens = _c(tokens, np.int32)
    parent = _c(parent, np.int32)
    path = np.empty(B + 1, np.int32)
    post = np.empty(T, np.int32)
    n_acc = ctypes.c_int32(0)
    bonus = ctypes.c_int32(0)
    rc = _load().oracle_accept(_p(target_logits, ctypes.c_float), T, V, _p(tokens, ctypes.c_int32),
                               _p(parent, ctypes.c_int32), int(n_nodes), int(B),
                               _p(path, ctypes.c_int32), ctypes.byref(n_acc), ctypes.byref(bonus),
                               _p(post, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_accept failed: {rc}")
    return dict(path=path, n_accepted=int(n_acc.value), bonus=int(bonus.value), posterior=post)


def sample_uniform(seed, row, v):
    """The uniform in (0,1) that the sampled walk draws for (seed, row, v)."""
    f = _load().oracle_sample_uniform
    f.restype = ctypes.c_double
    f.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32]
    return float(f(int(seed), int(row), int(v)))


def sample_tokens(target_logits, n_nodes, temperature, seed, first_row=0):
    """Token the target selects at every node when sampling at `temperature` (Gumbel-max, fp64).
    Returns (token int32 [T], runner_up int32 [T], gap float64 [T]); rows past n_nodes get -1."""
    target_logits = _c(target_logits, np.float32)
    T, V = target_logits.shape
    tok = np.empty(T, np.int32)
    run = np.empty(T, np.int32)
    gap = np.empty(T, np.float64)
    f = _load().oracle_sample_tokens
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int, ctypes.c_int, ctypes.c_int,
                  ctypes.c_double, ctypes.c_uint64, ctypes.c_int, ctypes.POINTER(ctypes.c_int32),
                  ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
    rc = f(_p(target_logits, ctypes.c_float), T, V, int(n_nodes), float(temperature), int(seed),
           int(first_row), _p(tok, ctypes.c_int32), _p(run, ctypes.c_int32), _p(gap, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_sample_tokens failed: {rc}")
    return tok, run, gap


def walk(selected, tokens, parent, n_nodes, B):
    """The verifier walk given the token selected at every node.  Returns dict(path, n_accepted, bonus)."""
    selected = _c(selected, np.int32)
    tokens = _c(tokens, np.int32)
    parent = _c(parent, np.int32)
    path = np.empty(B + 1, np.int32)
    n_acc = ctypes.c_int32(0)
    bonus = ctypes.c_int32(0)
    rc = _load().oracle_walk(_p(selected, ctypes.c_int32), _p(tokens, ctypes.c_int32),
                             _p(parent, ctypes.c_int32), int(n_nodes), int(B), _p(path, ctypes.c_int32),
                             ctypes.byref(n_acc), ctypes.byref(bonus))
    if rc != 0:
        raise ValueError(f"oracle_walk failed: {rc}")
    return dict(path=path, n_accepted=int(n_acc.value), bonus=int(bonus.value))


def compact(tree_rows, path, n_accepted, cache, L):
    """Append tree rows path[0..n_accepted] to cache (fp32 [>=L+n_accepted+1, ...]) in place."""
    tree_rows = _c(tree_rows, np.float32)
    path = _c(path, np.int32)
    assert cache.dtype == np.float32 and cache.flags["C_CONTIGUOUS"]
    row_elems = int(np.prod(tree_rows.shape[1:]))
    assert cache.shape[0] >= L + n_accepted + 1
    rc = _load().oracle_compact(_p(tree_rows, ctypes.c_float), _p(path, ctypes.c_int32),
                                int(n_accepted), row_elems, int(L), _p(cache, ctypes.c_float))
    if rc != 0:
        raise ValueError(f"oracle_compact failed: {rc}")
    return cache
