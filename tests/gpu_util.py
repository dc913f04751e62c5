"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run one stage of
the HIP library through the Python binding, bring results back as numpy."""
import numpy as np
import torch

import ddtree_inputs as di
import paper_2604_12989_amd as dd

DEV = "cuda:0"


def attn_err(got, ref):
    """Worst attention error in the units of the tolerance: |got - ref| where |ref| < 4 (the
    literal max-abs bound), |got - ref| / |ref| for elements of magnitude 4 or more."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    d = np.abs(got - ref)
    a = np.abs(ref)
    big = a >= 4.0
    err = float(d[~big].max()) if (~big).any() else 0.0
    if big.any():
        err = max(err, float((d[big] / a[big]).max()))
    return err


def attn_err_over_rms(got, ref):
    """max-abs error divided by rms(ref): how large the error is on the scale of the outputs
    themselves (long contexts average unit-variance values down to rms ~ 1/sqrt(L))."""
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt((ref ** 2).mean()))
    return float(np.abs(np.asarray(got, np.float64) - ref).max()) / max(rms, 1e-30), rms


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def bf16_dev(a_f32):
    """fp32 numpy array of bf16-representable values -> torch.bfloat16 tensor on the device."""
    bits = di.f32_to_bf16_bits(np.ascontiguousarray(a_f32, np.float32)).reshape(np.shape(a_f32))
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def ws_for(batch, B, V, N, Hq=1, Hkv=1, D=8, sum_L=0):
    return dd.Workspace(batch, B, V, N, Hq, Hkv, D, sum_L)


def gpu_topk(logits, K):
    x = logits if logits.ndim == 3 else logits[None]
    batch, B, V = x.shape
    ws = ws_for(batch, B, V, max(K, 1))
    tok, lp = dd.topk(to_dev(x), K, ws)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), lp.cpu().numpy()


def gpu_build(tok, lp, N, root):
    tok = tok if tok.ndim == 3 else tok[None]
    lp = lp if lp.ndim == 3 else lp[None]
    batch = tok.shape[0]
    root = np.full(batch, root, np.int32) if np.isscalar(root) else np.asarray(root, np.int32)
    out = dd.build(to_dev(tok.astype(np.int32)), to_dev(lp.astype(np.float32)), N, to_dev(root))
    torch.cuda.synchronize()
    res = {k: v.cpu().numpy() for k, v in out.items()}
    res["ancestor_mask"] = res["ancestor_mask"].view(np.uint64)
    return res


def gpu_attn(q, kc, vc, kt, vt, mask, kv_offset, batch, T, dtype, scale=None):
    """All arrays fp32 numpy (bf16-representable when dtype == 'bf16'); mask uint64 [batch,T,W]."""
    Hq, D = q.shape[-2], q.shape[-1]
    Hkv = kt.shape[-2]
    sum_L = int(kv_offset[-1])
    conv = bf16_dev if dtype == "bf16" else (lambda a: to_dev(np.asarray(a, np.float32)))
    ws = ws_for(batch, 1, 8, max(T - 1, 1), Hq, Hkv, D, sum_L)
    scale = float(scale if scale is not None else 1.0 / np.sqrt(D))
    kcd = conv(kc.reshape(-1, Hkv, D)) if sum_L > 0 else None
    vcd = conv(vc.reshape(-1, Hkv, D)) if sum_L > 0 else None
    out = dd.verify_attn(conv(q.reshape(-1, Hq, D)), kcd, vcd, conv(kt.reshape(-1, Hkv, D)),
                         conv(vt.reshape(-1, Hkv, D)),
                         to_dev(np.ascontiguousarray(mask).view(np.int64).reshape(batch, T, -1)),
                         kv_offset, batch, T, Hq, Hkv, D, scale,
                         dd.DTYPE_BF16 if dtype == "bf16" else dd.DTYPE_FP32, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().reshape(batch, T, Hq, D)


def gpu_accept(target_logits, tokens, parent, depth, n_nodes, B, temperature=None, seed=0):
    x = target_logits if target_logits.ndim == 3 else target_logits[None]
    batch, T, V = x.shape
    f = lambda a: to_dev(np.asarray(a, np.int32).reshape(batch, -1))
    ws = ws_for(batch, B, V, T - 1)
    out = dd.accept(to_dev(x), f(tokens), f(parent), f(depth),
                    to_dev(np.asarray(n_nodes, np.int32).reshape(batch)), B, ws,
                    temperature=temperature, seed=seed)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}
