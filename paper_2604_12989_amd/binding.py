"""ctypes binding with the same names as the C ABI in include/ddtree.h (argument marshalling
only).  Tensors are torch tensors on the GPU; the calls enqueue on torch's current stream."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

DTYPE_BF16 = 0
DTYPE_FP32 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("DDTREE_LIB", os.path.join(_HERE, "libddtree.so"))
_lib = None

_vp, _sz, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_SIGNATURES = {
    "ddtree_version": (ctypes.c_int, []),
    "ddtree_error_string": (ctypes.c_char_p, [_i]),
    "ddtree_workspace_bytes": (_sz, [_i] * 8),
    "ddtree_verify_attn_workspace_bytes": (_sz, [_i] * 6 + [ctypes.c_longlong]),
    "ddtree_topk": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "ddtree_build": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                          _sz, _vp]),
    "ddtree_verify_attn": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i,
                                ctypes.c_float, _i, _vp, _vp, _sz, _vp]),
    "ddtree_accept": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _sz,
                           _vp]),
    "ddtree_accept_noalloc": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp]),
    "ddtree_accept_sampled": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, ctypes.c_float,
                                   ctypes.c_uint64, _vp, _vp, _vp, _vp, _i, _vp, _sz, _vp]),
    "ddtree_compact": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp]),
    "ddtree_verify_attn_spans": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i,
                                      ctypes.c_float, _i, _vp, _vp, _sz, _vp]),
    "ddtree_set_build_algorithm": (_i, [_i]),
    "ddtree_selftest_host": (_i, []),
    "ddtree_build_giveups": (_i, [ctypes.POINTER(ctypes.c_uint)]),
    "ddtree_profile_enable": (_i, [ctypes.c_uint, _i]),
    "ddtree_profile_enable_every": (_i, [ctypes.c_uint, _i, _i]),
    "ddtree_profile_reset": (_i, []),
    "ddtree_profile_read": (_i, [_i, _vp, _i]),
}

KERNELS = {"topk_chunk": 0, "topk_merge": 1, "build": 2, "attn": 3, "attn_merge": 4,
           "accept_argmax": 5, "accept_walk": 6, "attn_generic": 7}


class DDTreeError(RuntimeError):
    pass


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load libddtree.so; raises if it has not been built (no CPU or eager fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise DDTreeError(f"{_LIB_PATH} is missing: build it with "
                              "`python -m paper_2604_12989_amd.build` first")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def version() -> int:
    return int(load().ddtree_version())


def error_string(code: int) -> str:
    return load().ddtree_error_string(int(code)).decode()


def _check(code: int, what: str):
    if code != 0:
        raise DDTreeError(f"{what} failed: {error_string(code)} ({code})")


def _call(name, args, result, defer):
    """Run the C entry point now, or (defer=True) return a zero-argument callable that runs it
    with the arguments marshalled once: tight loops then pay one ctypes call per stage."""
    fn = getattr(load(), name)
    if not defer:
        _check(fn(*args), name)
        return result

    # the callable holds raw pointers: the caller keeps the tensors alive while it is in use
    keep = (args, result)

    def run():
        rc = fn(*keep[0])
        if rc != 0:
            _check(rc, name)
        return keep[1]

    return run


def _keepalive(fn, *objs):
    def run():
        return fn()
    run.keep = objs
    return run


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise DDTreeError(f"{what}: expected a contiguous CUDA tensor of dtype {dtype}")
    return t


def workspace_bytes(batch, B, V, N, Hq, Hkv, D, max_sum_L) -> int:
    return int(load().ddtree_workspace_bytes(batch, B, V, N, Hq, Hkv, D, max_sum_L))


def verify_attn_workspace_bytes(batch, T, Hq, Hkv, D, dtype, sum_L):
    """Scratch that one verify_attn call uses for this shape and total cache length."""
    return int(load().ddtree_verify_attn_workspace_bytes(batch, T, Hq, Hkv, D, dtype, int(sum_L)))


class Workspace:
    """Device scratch sized by ddtree_workspace_bytes (plain torch allocation)."""

    def __init__(self, batch, B, V, N, Hq, Hkv, D, max_sum_L, device="cuda"):
        n = workspace_bytes(batch, B, V, N, Hq, Hkv, D, max_sum_L)
        if n == 0:
            raise DDTreeError("unsupported shape for ddtree_workspace_bytes")
        self.nbytes = n
        self.buf = torch.empty(n + 256, dtype=torch.uint8, device=device)
        off = (-self.buf.data_ptr()) % 256
        self.ptr = self.buf.data_ptr() + off


def _ws(ws):
    if ws is None:
        return None, 0
    return ctypes.c_void_p(ws.ptr), ws.nbytes


def topk(logits, K, ws, topk_tok=None, topk_lp=None, defer=False):
    """logits fp32 [batch,B,V] (or [B,V]) -> (topk_tok int32, topk_lp fp32) [batch,B,K]."""
    _dev(logits, torch.float32, "logits")
    x = logits if logits.dim() == 3 else logits.unsqueeze(0)
    batch, B, V = x.shape
    if topk_tok is None:
        topk_tok = torch.empty((batch, B, K), dtype=torch.int32, device=x.device)
    if topk_lp is None:
        topk_lp = torch.empty((batch, B, K), dtype=torch.float32, device=x.device)
    p, n = _ws(ws)
    args = (_ptr(x), batch, B, V, K, _ptr(topk_tok), _ptr(topk_lp), p, n, _stream())
    return _call("ddtree_topk", args, (topk_tok, topk_lp), defer)


def build(topk_tok, topk_lp, N, root_token, ws=None, out=None, defer=False):
    """Returns dict(tokens, parent, depth, rank, node_score, ancestor_mask, n_nodes)."""
    _dev(topk_tok, torch.int32, "topk_tok")
    _dev(topk_lp, torch.float32, "topk_lp")
    _dev(root_token, torch.int32, "root_token")
    batch, B, K = topk_tok.shape
    T, W = N + 1, (N + 1 + 63) // 64
    dev = topk_tok.device
    if out is None:
        out = dict(tokens=torch.empty((batch, T), dtype=torch.int32, device=dev),
                   parent=torch.empty((batch, T), dtype=torch.int32, device=dev),
                   depth=torch.empty((batch, T), dtype=torch.int32, device=dev),
                   rank=torch.empty((batch, T), dtype=torch.int32, device=dev),
                   node_score=torch.empty((batch, T), dtype=torch.float32, device=dev),
                   ancestor_mask=torch.empty((batch, T, W), dtype=torch.int64, device=dev),
                   n_nodes=torch.empty((batch,), dtype=torch.int32, device=dev))
    p, n = _ws(ws)
    args = (_ptr(topk_tok), _ptr(topk_lp), batch, B, K, N, _ptr(root_token), _ptr(out["tokens"]),
            _ptr(out["parent"]), _ptr(out["depth"]), _ptr(out.get("rank")),
            _ptr(out.get("node_score")), _ptr(out["ancestor_mask"]), _ptr(out["n_nodes"]), p, n,
            _stream())
    return _call("ddtree_build", args, out, defer)


def verify_attn(q, k_cache, v_cache, k_tree, v_tree, ancestor_mask, kv_offset, batch, T, Hq, Hkv,
                D, softmax_scale, dtype, ws, out=None, defer=False):
    """q [batch*T,Hq,D]; k/v_cache [sum_L,Hkv,D]; k/v_tree [batch*T,Hkv,D]; mask int64 [batch,T,W];
    kv_offset: host int32 sequence of batch+1 entries."""
    tdt = torch.bfloat16 if dtype == DTYPE_BF16 else torch.float32
    for name, t in (("q", q), ("k_tree", k_tree), ("v_tree", v_tree)):
        _dev(t, tdt, name)
    if k_cache is not None:
        _dev(k_cache, tdt, "k_cache")
        _dev(v_cache, tdt, "v_cache")
    _dev(ancestor_mask, torch.int64, "ancestor_mask")
    off = np.ascontiguousarray(np.asarray(kv_offset, dtype=np.int32))
    if off.shape != (batch + 1,):
        raise DDTreeError("kv_offset must have batch+1 entries")
    if out is None:
        out = torch.empty_like(q)
    p, n = _ws(ws)
    args = (_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree), _ptr(v_tree), _ptr(ancestor_mask),
            off.ctypes.data_as(ctypes.c_void_p), batch, T, Hq, Hkv, D, ctypes.c_float(softmax_scale),
            dtype, _ptr(out), p, n, _stream())
    run = _call("ddtree_verify_attn", args, out, defer)
    return _keepalive(run, off) if defer else run


def verify_attn_spans(q, k_cache, v_cache, k_tree, v_tree, ancestor_mask, kv_start, kv_len, batch, T, Hq,
                      Hkv, D, softmax_scale, dtype, ws, out=None, defer=False):
    """verify_attn with sequence s owning cache rows kv_start[s] .. kv_start[s] + kv_len[s] - 1
    (host int32 sequences of batch entries each; the spans need not touch)."""
    tdt = torch.bfloat16 if dtype == DTYPE_BF16 else torch.float32
    for name, t in (("q", q), ("k_tree", k_tree), ("v_tree", v_tree)):
        _dev(t, tdt, name)
    if k_cache is not None:
        _dev(k_cache, tdt, "k_cache")
        _dev(v_cache, tdt, "v_cache")
    _dev(ancestor_mask, torch.int64, "ancestor_mask")
    start = np.ascontiguousarray(np.asarray(kv_start, dtype=np.int32))
    length = np.ascontiguousarray(np.asarray(kv_len, dtype=np.int32))
    if start.shape != (batch,) or length.shape != (batch,):
        raise DDTreeError("kv_start and kv_len must have batch entries each")
    if out is None:
        out = torch.empty_like(q)
    p, n = _ws(ws)
    args = (_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree), _ptr(v_tree), _ptr(ancestor_mask),
            start.ctypes.data_as(ctypes.c_void_p), length.ctypes.data_as(ctypes.c_void_p), batch, T, Hq,
            Hkv, D, ctypes.c_float(softmax_scale), dtype, _ptr(out), p, n, _stream())
    run = _call("ddtree_verify_attn_spans", args, out, defer)
    return _keepalive(run, start, length) if defer else run


def accept(target_logits, tokens, parent, depth, n_nodes, B, ws, out=None, want_posterior=True,
           defer=False, temperature=None, seed=0):
    """target_logits fp32 [batch,T,V] -> dict(path [batch,B+1], n_accepted, bonus_token, posterior).
    temperature=None: greedy rule (ddtree_accept); a positive temperature: sampled selection
    (ddtree_accept_sampled) with the given 64-bit seed."""
    _dev(target_logits, torch.float32, "target_logits")
    batch, T, V = target_logits.shape
    dev = target_logits.device
    if out is None:
        out = dict(path=torch.empty((batch, B + 1), dtype=torch.int32, device=dev),
                   n_accepted=torch.empty((batch,), dtype=torch.int32, device=dev),
                   bonus_token=torch.empty((batch,), dtype=torch.int32, device=dev),
                   posterior=(torch.empty((batch, T), dtype=torch.int32, device=dev)
                              if want_posterior else None))
    p, n = _ws(ws)
    if temperature is not None:
        args = (_ptr(target_logits), batch, T, V, _ptr(tokens), _ptr(parent), _ptr(depth),
                _ptr(n_nodes), ctypes.c_float(float(temperature)), ctypes.c_uint64(int(seed)),
                _ptr(out["path"]), _ptr(out["n_accepted"]), _ptr(out["bonus_token"]),
                _ptr(out.get("posterior")), B, p, n, _stream())
        return _call("ddtree_accept_sampled", args, out, defer)
    args = (_ptr(target_logits), batch, T, V, _ptr(tokens), _ptr(parent), _ptr(depth),
            _ptr(n_nodes), _ptr(out["path"]), _ptr(out["n_accepted"]), _ptr(out["bonus_token"]),
            _ptr(out.get("posterior")), B, p, n, _stream())
    return _call("ddtree_accept", args, out, defer)


def accept_noalloc(target_logits, tokens, parent, depth, n_nodes, B, out, defer=False):
    """ddtree_accept_noalloc: the greedy walk with its scratch in the library's static device
    array.  `out` (dict of path, n_accepted, bonus_token, posterior-or-None) is supplied by the
    caller: this path allocates nothing, here or in the library."""
    _dev(target_logits, torch.float32, "target_logits")
    batch, T, V = target_logits.shape
    args = (_ptr(target_logits), batch, T, V, _ptr(tokens), _ptr(parent), _ptr(depth),
            _ptr(n_nodes), _ptr(out["path"]), _ptr(out["n_accepted"]), _ptr(out["bonus_token"]),
            _ptr(out.get("posterior")), B, _stream())
    return _call("ddtree_accept_noalloc", args, out, defer)


def compact(k_tree, v_tree, path, n_accepted, dst_row, batch, T, B, Hkv, D, k_cache, v_cache):
    """Append the accepted tree rows of K and V to the caches in place."""
    dst = np.ascontiguousarray(np.asarray(dst_row, dtype=np.int32))
    if dst.shape != (batch,):
        raise DDTreeError("dst_row must have batch entries")
    _check(load().ddtree_compact(_ptr(k_tree), _ptr(v_tree), _ptr(path), _ptr(n_accepted),
                                 dst.ctypes.data_as(ctypes.c_void_p), batch, T, B, Hkv, D,
                                 k_tree.element_size(), _ptr(k_cache), _ptr(v_cache), _stream()),
           "ddtree_compact")


BUILD_AUTO, BUILD_POPS, BUILD_LEVELS = 0, 1, 2


def set_build_algorithm(algo):
    """Force one construction in ddtree_build (BUILD_POPS / BUILD_LEVELS) or let it choose (BUILD_AUTO)."""
    _check(load().ddtree_set_build_algorithm(int(algo)), "ddtree_set_build_algorithm")


def selftest_host():
    """Host-side self-check of the attention kernel's launch arithmetic (no GPU): 0 if it holds."""
    return int(load().ddtree_selftest_host())


def build_giveups():
    """Sequences (since load) that the level-synchronous construction handed back to the pops."""
    n = ctypes.c_uint(0)
    _check(load().ddtree_build_giveups(ctypes.byref(n)), "ddtree_build_giveups")
    return int(n.value)


def profile_enable(kernels, capacity, every=1):
    """Time one launch in `every` of the named kernels (see KERNELS) with HIP events; [] switches it off."""
    mask = 0
    for k in kernels:
        mask |= 1 << KERNELS[k]
    _check(load().ddtree_profile_enable_every(mask, int(capacity), int(every)), "ddtree_profile_enable_every")


def profile_reset():
    _check(load().ddtree_profile_reset(), "ddtree_profile_reset")


def profile_read(kernel, max_records=1 << 16):
    """Elapsed milliseconds of the recorded launches of one kernel (synchronise first)."""
    buf = np.empty(max_records, np.float32)
    n = load().ddtree_profile_read(KERNELS[kernel], buf.ctypes.data_as(ctypes.c_void_p), max_records)
    if n < 0:
        _check(n, "ddtree_profile_read")
    return buf[:n].copy()
