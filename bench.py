#!/usr/bin/env python3
"""Benchmark of the DDTree draft-tree step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
    ddtree_topk -> ddtree_build -> ddtree_verify_attn -> ddtree_accept
enqueued back to back on one stream (a dependent chain: the attention mask and the walk come
from the tree that the build produced in the same step).  Inputs are resident in HBM before
the timed region starts, and the step rotates over several copies of them so that no step
finds its logits or KV cache in the 256 MB last-level cache.

Prints ONE JSON line: tree steps/s, plus
  roofline      the verify-attention MFMA kernel: algorithmic FLOP / average kernel duration,
                the duration measured with HIP events around that kernel inside the timed loop
  cpu_baseline  the CPU oracle (test infrastructure, untuned) timed on this host on the same
                workload, for context
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import ddtree_inputs as di  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=3, help="workload (ddtree_inputs.CONFIGS), 1..5")
    ap.add_argument("--budget", type=int, default=0,
                    help="override the node budget N of the workload (budget sweep; 0 = the config's own)")
    ap.add_argument("--sets", type=int, default=0, help="input copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-reps", type=int, default=3)
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MiB (not timed): the kernel of "
                         "known traffic that scales the FETCH_SIZE / WRITE_SIZE counters of a "
                         "rocprofv3 --pmc run")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        log(f"bench.py: this build runs on ONE GPU (asked for --gpus {args.gpus}); the path has no "
            "multi-GPU leg (it would shard over the vocabulary for top-K and argmax and over KV heads "
            "for attention, with KB-sized exchanges)")
        sys.exit(2)
    import torch

    import paper_2604_12989_amd as dd

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    c = dict(di.CONFIGS[args.config])
    if args.budget > 0:
        c["N"] = args.budget
        c["name"] = f"{c['name']}, budget {args.budget}"
    seed = di.config_seed(args.config)
    batch, B, V, N, Hq, Hkv, D, L = c["batch"], c["B"], c["V"], c["N"], c["Hq"], c["Hkv"], c["D"], c["L"]
    K, T = min(N, V), N + 1
    # cache lengths: one sequence of L rows, or (batched configuration) seeded ragged lengths
    Ls = np.array([L]) if batch == 1 else di.ragged_lengths(seed, batch, *L)
    kv_off = [int(v) for v in np.concatenate([[0], np.cumsum(Ls)])]
    sum_L = kv_off[-1]
    bf16 = c["dtype"] == "bf16"
    dtype_id = dd.DTYPE_BF16 if bf16 else dd.DTYPE_FP32

    # ------------------------------------------------------------------ inputs (host, seeded)
    t0 = time.time()
    logits_h = np.stack([di.draft_logits(seed, B, V, batch_index=s) for s in range(batch)])
    if batch == 1:
        q_h, kc_h, vc_h, kt_h, vt_h = di.attn_tensors(seed, T, L, Hq, Hkv, D, c["dtype"])
    else:  # queries and tree rows of all sequences, one packed ragged cache
        q_h, _, _, kt_h, vt_h = di.attn_tensors(seed, batch * T, 0, Hq, Hkv, D, c["dtype"])
        _, kc_h, vc_h, _, _ = di.attn_tensors(seed + 1, 1, sum_L, Hq, Hkv, D, c["dtype"])
    log(f"[bench] config {args.config} ({c['name']}): inputs generated in {time.time() - t0:.1f}s")

    def attn_dev(a):
        if bf16:
            bits = di.f32_to_bf16_bits(a).reshape(a.shape)
            return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    ws = dd.Workspace(batch, B, V, N, Hq, Hkv, D, sum_L)
    root = torch.full((batch,), 11, dtype=torch.int32, device=dev)
    logits0 = torch.from_numpy(logits_h).to(dev).contiguous()
    # the tree of this workload (needed to plant the target's argmax); setup, not timed
    tok0, lp0 = dd.topk(logits0, K, ws)
    tree0 = dd.build(tok0, lp0, N, root)
    torch.cuda.synchronize()
    depth_h = tree0["depth"].cpu().numpy()
    top1_h = tok0.cpu().numpy()[:, :, 0]
    tl_h = np.stack([di.target_logits(seed, T, V, di.planted_tokens(seed, depth_h[s], top1_h[s], B, batch_index=s),
                                      batch_index=s) for s in range(batch)])
    log(f"[bench] tree: {int(tree0['n_nodes'][0])} nodes, max depth {int(depth_h.max())}; "
        f"all inputs ready after {time.time() - t0:.1f}s")

    bytes_per_set = logits_h.nbytes + tl_h.nbytes + (2 if bf16 else 4) * (
        q_h.size + kc_h.size + vc_h.size + kt_h.size + vt_h.size)
    n_sets = args.sets or max(2, int(np.ceil(2.2 * 256e6 / bytes_per_set)))
    sets = []
    base = dict(logits=logits0, tl=torch.from_numpy(tl_h).to(dev).contiguous(), q=attn_dev(q_h),
                kc=attn_dev(kc_h), vc=attn_dev(vc_h), kt=attn_dev(kt_h), vt=attn_dev(vt_h))
    for s in range(n_sets):
        sets.append(base if s == 0 else {k: v.clone() for k, v in base.items()})
    # outputs, allocated once
    out_attn = torch.empty_like(base["q"])
    tok = torch.empty((batch, B, K), dtype=torch.int32, device=dev)
    lp = torch.empty((batch, B, K), dtype=torch.float32, device=dev)
    tree = {k: torch.empty_like(v) for k, v in tree0.items()}
    acc = dict(path=torch.empty((batch, B + 1), dtype=torch.int32, device=dev),
               n_accepted=torch.empty((batch,), dtype=torch.int32, device=dev),
               bonus_token=torch.empty((batch,), dtype=torch.int32, device=dev),
               posterior=torch.empty((batch, T), dtype=torch.int32, device=dev))
    scale = 1.0 / float(np.sqrt(D))

    # one pre-marshalled call list per input set: the timed loop is four ctypes calls per step
    steps = []
    for s in sets:
        steps.append([
            dd.topk(s["logits"], K, ws, tok, lp, defer=True),
            dd.build(tok, lp, N, root, ws, tree, defer=True),
            dd.verify_attn(s["q"], s["kc"], s["vc"], s["kt"], s["vt"], tree["ancestor_mask"], kv_off,
                           batch, T, Hq, Hkv, D, scale, dtype_id, ws, out_attn, defer=True),
            dd.accept(s["tl"], tree["tokens"], tree["parent"], tree["depth"], tree["n_nodes"], B, ws,
                      acc, defer=True),
        ])

    def run_step(i):
        for call in steps[i % n_sets]:
            call()

    main_kernel = "attn" if (bf16 and D == 128) else "attn_generic"
    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # ------------------------------------------------------------------ warm-up, then timed
    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    # the main kernel is timed live with HIP events that take the time stamps of its own dispatch
    # (ddtree_profile_enable_every), one launch in `every` of the timed loop
    every = max(1, min(8, args.steps // 32))
    dd.profile_enable([main_kernel], args.steps // every + 1, every)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        run_step(i)
    torch.cuda.synchronize()
    t_stop = time.perf_counter()
    kernel_ms = dd.profile_read(main_kernel)
    dd.profile_enable([], 0)
    elapsed = t_stop - t_start
    ms_per_step = 1e3 * elapsed / args.steps
    steps_per_s = args.steps / elapsed
    n_acc = [int(v) for v in acc["n_accepted"].cpu()]
    n_acc = n_acc[0] if batch == 1 else n_acc

    # ------------------------------------------------------------------ roofline of the main kernel
    depth_now = tree["depth"].cpu().numpy()
    vis_tree = int((depth_now[depth_now >= 0] + 1).sum())
    flops = 4.0 * D * Hq * (float(T) * sum_L + vis_tree)  # algorithmic: QK^T and PV over visible keys
    k_avg_ms = float(kernel_ms.mean())
    achieved = flops / (k_avg_ms * 1e-3) / 1e12
    # HBM bytes per launch from committed rocprofv3 --pmc summaries (FETCH_SIZE + WRITE_SIZE, each
    # scaled by a plain copy of known size); null for workloads that have not been profiled
    traffic = traffic_detail = None
    tpath = os.path.join(ROOT, "profiles", "attn_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic_detail = json.load(open(tpath)).get(f"config{args.config}")
            if traffic_detail:
                traffic = traffic_detail["fetch_bytes"] + traffic_detail["write_bytes"]
        except Exception:  # noqa: BLE001
            traffic = traffic_detail = None
    roofline = dict(bound="mfma", kernel="attn_mfma_kernel" if main_kernel == "attn" else main_kernel,
                    achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS if bf16 else 157.3,
                    unit="TFLOP/s", frac=round(achieved / (PEAK_BF16_TFLOPS if bf16 else 157.3), 4),
                    traffic=traffic, traffic_detail=traffic_detail, flops_per_launch=flops, kernel_avg_us=round(1e3 * k_avg_ms, 2),
                    kernel_launches=int(kernel_ms.size), timed_one_launch_in=every)

    # ------------------------------------------------------------------ per-kernel breakdown (not timed)
    names = ["topk_chunk", "topk_merge", "build", main_kernel, "attn_merge", "accept_argmax",
             "accept_walk"]
    reps = 40
    dd.profile_enable(names, reps)
    for i in range(reps):
        run_step(i)
    torch.cuda.synchronize()
    stages = {}
    for nme in names:
        ms = dd.profile_read(nme)
        if ms.size:
            stages[nme + "_us"] = round(1e3 * float(np.median(ms)), 2)
    dd.profile_enable([], 0)
    if "accept_argmax_us" in stages:
        stages["accept_argmax_GBs"] = round(tl_h.nbytes / (stages["accept_argmax_us"] * 1e-6) / 1e9, 1)
    if "topk_chunk_us" in stages:
        stages["topk_chunk_GBs"] = round(logits_h.nbytes / (stages["topk_chunk_us"] * 1e-6) / 1e9, 1)
    # each stage against the roofline that bounds it (the build is a latency chain: no roofline)
    stages["frac_of_roofline"] = {
        k: v for k, v in (
            ("topk_hbm", round(logits_h.nbytes / (1e-6 * (stages.get("topk_chunk_us", 0) + stages.get("topk_merge_us", 0))
                                                  or float("inf")) / 1e9 / PEAK_HBM_GBS, 4)),
            ("attn_mfma" if main_kernel == "attn" else "attn_fp32_alu",
             round(flops / (stages[main_kernel + "_us"] * 1e-6) / 1e12 / (PEAK_BF16_TFLOPS if main_kernel == "attn" else 157.3), 4)),
            ("accept_hbm", round(tl_h.nbytes / (1e-6 * (stages.get("accept_argmax_us", 0) + stages.get("accept_walk_us", 0))
                                                or float("inf")) / 1e9 / PEAK_HBM_GBS, 4)),
        )}

    # ------------------------------------------------------------------ CPU oracle baseline
    cpu = None
    if not args.no_cpu:
        import oracle
        t_cpu = []
        cpu_reps = args.cpu_reps if batch == 1 else 1
        for _ in range(cpu_reps):
            t1 = time.perf_counter()
            for s in range(batch):
                tok_o, lp_o = oracle.topk(logits_h[s], K)
                tr = oracle.build_tree(tok_o, lp_o, N, 11)
                mask_o = oracle.ancestor_mask(tr["parent"], tr["n_nodes"], T=T)
                oracle.verify_attn(q_h[s * T:(s + 1) * T], kc_h[kv_off[s]:kv_off[s + 1]], vc_h[kv_off[s]:kv_off[s + 1]],
                                   kt_h[s * T:(s + 1) * T], vt_h[s * T:(s + 1) * T], mask_o)
                oracle.accept(tl_h[s], tr["tokens"], tr["parent"], tr["n_nodes"], B)
            t_cpu.append(time.perf_counter() - t1)
        cpu = dict(value=round(1.0 / float(np.mean(t_cpu)), 4), unit="tree steps/s",
                   cores=oracle.num_threads(), kind="oracle",
                   sample=f"{cpu_reps} full steps of the same config-{args.config} inputs "
                          f"(all {batch}x{T}x{Hq} attention rows), mean {np.mean(t_cpu):.2f} s/step")

    result = {
        "metric": ("tree steps/s (topk+build+verify-attn+accept) at N=256, L=8192; % roofline"
                   if args.config == 3 and args.budget == 0 else "tree steps/s (topk+build+verify-attn+accept)"),
        "value": round(steps_per_s, 1),
        "unit": "tree steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"config {args.config} ({c['name']}): B={B} V={V} N={N} Hq={Hq} "
                               f"Hkv={Hkv} D={D} " + (f"L={L}" if batch == 1 else
                               f"batch={batch} ragged L={min(Ls)}..{max(Ls)} (sum {sum_L})"), "input_sets_rotated": n_sets,
                   "launch": "eager, 4 C-ABI calls per step on one stream",
                   "n_accepted": n_acc},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "stages": stages,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
