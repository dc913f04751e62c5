#!/usr/bin/env python3
"""Benchmark of the DDTree draft-tree step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
    ddtree_topk -> ddtree_build -> ddtree_verify_attn -> ddtree_accept
enqueued back to back on one stream (a dependent chain: the attention mask and the walk come
from the tree that the build produced in the same step).  Inputs are resident in HBM before
the timed region starts, and the step rotates over several copies of them so that no step
finds its logits or KV cache in the 256 MB last-level cache.

The timed loop carries no instrumentation at all.  Everything else is measured afterwards, in
passes of their own over the same call lists:
  step_us       p10 / median / p90 of the step, from blocks of 8 steps timed on the host
  roofline      the verify-attention MFMA kernel: algorithmic FLOP / average kernel duration,
                the duration from HIP events that take the time stamps of the kernel's own
                dispatch (one launch in four of a separate loop)
  stages        per-kernel medians (the same kind of events on every launch)
  stages_peaked the same workload with a confident drafter (one token per row holds 90 % of the
                probability): a tree of full depth, where the build and the walk do real work
  cpu_baseline  the CPU oracle (test infrastructure, untuned) timed on this host on the same
                workload, all threads and one thread
Prints ONE JSON line.  --sweep adds the node-budget sweep N = 16 .. 1024 (Section 5's budget
trade-off) to that line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import subprocess
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import ddtree_inputs as di  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3   # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E
KERNEL_NAMES = ["topk_chunk", "topk_merge", "build", "attn", "attn_generic", "attn_merge",
                "accept_argmax", "accept_walk"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=3, help="workload (ddtree_inputs.CONFIGS), 1..5")
    ap.add_argument("--budget", type=int, default=0,
                    help="override the node budget N of the workload (0 = the config's own)")
    ap.add_argument("--sets", type=int, default=0, help="input copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-peaked", action="store_true", help="skip the confident-drafter variant")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the step at node budgets 16 .. 1024 (adds budget_sweep to the line)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MiB (not timed): the kernel of "
                         "known traffic that scales the FETCH_SIZE / WRITE_SIZE counters of a "
                         "rocprofv3 --pmc run")
    return ap.parse_args()


# ---------------------------------------------------------------------------------- workload
class Workload:
    """Device-resident input sets of one (config, budget, drafter kind) and the pre-marshalled
    call lists that run a step over them."""

    def __init__(self, dd, torch, c, N, host, logits_h, tl_h, n_sets, dev="cuda:0"):
        self.c, self.N = c, N
        batch, B, V, Hq, Hkv, D = c["batch"], c["B"], c["V"], c["Hq"], c["Hkv"], c["D"]
        K, T = min(N, V), N + 1
        self.K, self.T = K, T
        bf16 = c["dtype"] == "bf16"
        self.bf16 = bf16
        self.kv_off = host["kv_off"]
        self.sum_L = self.kv_off[-1]
        self.logits_h, self.tl_h = logits_h, tl_h

        def attn_dev(a):
            if bf16:
                bits = di.f32_to_bf16_bits(a).reshape(a.shape)
                return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
            return torch.from_numpy(a).to(dev)

        self.ws = dd.Workspace(batch, B, V, N, Hq, Hkv, D, self.sum_L)
        self.root = torch.full((batch,), 11, dtype=torch.int32, device=dev)
        nq = batch * T
        base = dict(logits=torch.from_numpy(logits_h).to(dev).contiguous(),
                    tl=torch.from_numpy(tl_h).to(dev).contiguous(),
                    q=attn_dev(host["q"][:nq]), kc=attn_dev(host["kc"]), vc=attn_dev(host["vc"]),
                    kt=attn_dev(host["kt"][:nq]), vt=attn_dev(host["vt"][:nq]))
        self.bytes_per_set = sum(v.numel() * v.element_size() for v in base.values())
        self.n_sets = n_sets or max(2, int(np.ceil(2.2 * 256e6 / self.bytes_per_set)))
        self.sets = [base if s == 0 else {k: v.clone() for k, v in base.items()}
                     for s in range(self.n_sets)]
        W = (T + 63) // 64
        self.out_attn = torch.empty_like(base["q"])
        self.tok = torch.empty((batch, B, K), dtype=torch.int32, device=dev)
        self.lp = torch.empty((batch, B, K), dtype=torch.float32, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        self.tree = dict(tokens=torch.empty((batch, T), **i32), parent=torch.empty((batch, T), **i32),
                         depth=torch.empty((batch, T), **i32), rank=torch.empty((batch, T), **i32),
                         node_score=torch.empty((batch, T), dtype=torch.float32, device=dev),
                         ancestor_mask=torch.empty((batch, T, W), dtype=torch.int64, device=dev),
                         n_nodes=torch.empty((batch,), **i32))
        self.acc = dict(path=torch.empty((batch, B + 1), **i32), n_accepted=torch.empty((batch,), **i32),
                        bonus_token=torch.empty((batch,), **i32), posterior=torch.empty((batch, T), **i32))
        scale = 1.0 / float(np.sqrt(D))
        dtype_id = dd.DTYPE_BF16 if bf16 else dd.DTYPE_FP32
        # one pre-marshalled call list per input set: a step is four ctypes calls
        self.steps = []
        for s in self.sets:
            self.steps.append([
                dd.topk(s["logits"], K, self.ws, self.tok, self.lp, defer=True),
                dd.build(self.tok, self.lp, N, self.root, self.ws, self.tree, defer=True),
                dd.verify_attn(s["q"], s["kc"], s["vc"], s["kt"], s["vt"], self.tree["ancestor_mask"],
                               self.kv_off, batch, T, Hq, Hkv, D, scale, dtype_id, self.ws, self.out_attn,
                               defer=True),
                dd.accept(s["tl"], self.tree["tokens"], self.tree["parent"], self.tree["depth"],
                          self.tree["n_nodes"], B, self.ws, self.acc, defer=True),
            ])
        self.main_kernel = "attn" if (bf16 and D == 128) else "attn_generic"

    def run_step(self, i):
        for call in self.steps[i % self.n_sets]:
            call()

    def attn_flops(self):
        """Algorithmic flops of one attention launch: QK^T and PV over the visible keys only."""
        c = self.c
        depth = self.tree["depth"].cpu().numpy()
        vis_tree = int((depth[depth >= 0] + 1).sum())
        return 4.0 * c["D"] * c["Hq"] * (float(self.T) * self.sum_L + vis_tree)


def timed_loop(torch, wl, steps, warmup):
    for i in range(warmup):
        wl.run_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        wl.run_step(i)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def step_distribution(torch, wl, blocks=40, per_block=8):
    """p10 / median / p90 of the step from blocks of `per_block` steps, each block timed on the
    host between two synchronisations (the launch latency exposed at the head of a block is
    shared by its steps: under a microsecond per step)."""
    us = []
    i = 0
    for _ in range(blocks):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(per_block):
            wl.run_step(i)
            i += 1
        torch.cuda.synchronize()
        us.append(1e6 * (time.perf_counter() - t0) / per_block)
    p10, med, p90 = np.percentile(us, [10, 50, 90])
    return dict(p10=round(float(p10), 2), median=round(float(med), 2), p90=round(float(p90), 2),
                method=f"{blocks} blocks of {per_block} steps, host clock between synchronisations")


def kernel_times(dd, torch, wl, names, reps, every=1):
    """Per-launch durations (ms arrays) of the named kernels over `reps` steps, from events that
    take the begin and end time stamps of each dispatch (one launch in `every`)."""
    dd.profile_enable(names, reps // every + 2, every)
    for i in range(reps):
        wl.run_step(i)
    torch.cuda.synchronize()
    out = {n: dd.profile_read(n) for n in names}
    dd.profile_enable([], 0)
    return out


def stage_table(dd, torch, wl, reps=40):
    ms = kernel_times(dd, torch, wl, KERNEL_NAMES, reps)
    st = {n + "_us": round(1e3 * float(np.median(v)), 2) for n, v in ms.items() if v.size}
    return st


def stage_fractions(st, wl, flops):
    """Each stage against the roofline that bounds it (the build is a latency chain: none)."""
    topk_us = st.get("topk_chunk_us", 0) + st.get("topk_merge_us", 0)
    acc_us = st.get("accept_argmax_us", 0) + st.get("accept_walk_us", 0)
    mk = wl.main_kernel
    out = {}
    if topk_us:
        out["topk_hbm"] = round(wl.logits_h.nbytes / (topk_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)
    if st.get(mk + "_us"):
        peak = PEAK_BF16_TFLOPS if mk == "attn" else PEAK_FP32_TFLOPS
        out["attn_mfma" if mk == "attn" else "attn_fp32_alu"] = round(
            flops / (st[mk + "_us"] * 1e-6) / 1e12 / peak, 4)
    if acc_us:
        out["accept_hbm"] = round(wl.tl_h.nbytes / (acc_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)
    return out


# ---------------------------------------------------------------------------------- host side
def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def set_omp_threads(n):
    """Thread count of the OpenMP runtime the oracle library runs on (its own source is untouched)."""
    for name in ("libgomp.so.1", "libgomp.so"):
        try:
            ctypes.CDLL(name).omp_set_num_threads(int(n))
            return True
        except OSError:
            continue
    return False


def oracle_step(oracle, wl, host, s, rows=None):
    """One oracle step on sequence s; rows = (node, head) pairs to restrict the attention to."""
    c, T = wl.c, wl.T
    off = wl.kv_off
    tok_o, lp_o = oracle.topk(wl.logits_h[s], wl.K)
    tr = oracle.build_tree(tok_o, lp_o, wl.N, 11)
    mask_o = oracle.ancestor_mask(tr["parent"], tr["n_nodes"], T=T)
    oracle.verify_attn(host["q"][s * T:(s + 1) * T], host["kc"][off[s]:off[s + 1]], host["vc"][off[s]:off[s + 1]],
                       host["kt"][s * T:(s + 1) * T], host["vt"][s * T:(s + 1) * T], mask_o, pairs=rows)
    oracle.accept(wl.tl_h[s], tr["tokens"], tr["parent"], tr["n_nodes"], c["B"])


def cpu_baseline(wl, host, config, reps):
    import oracle
    batch, T, Hq = wl.c["batch"], wl.T, wl.c["Hq"]
    threads = oracle.num_threads()
    t_all = []
    for _ in range(reps if batch == 1 else 1):
        t1 = time.perf_counter()
        for s in range(batch):
            oracle_step(oracle, wl, host, s)
        t_all.append(time.perf_counter() - t1)
    mean_all = float(np.mean(t_all))
    # one thread: the same step with the attention restricted to every 8th (node, head) row, the
    # other stages in full; the attention time is scaled back by the row count
    single = None
    if set_omp_threads(1):
        pairs = np.array([(i, h) for i in range(T) for h in range(Hq)], np.int32)[::8]
        t1 = time.perf_counter()
        for s in range(batch):
            oracle_step(oracle, wl, host, s, rows=np.zeros((1, 2), np.int32))
        t_rest = time.perf_counter() - t1
        t1 = time.perf_counter()
        for s in range(batch):
            oracle_step(oracle, wl, host, s, rows=pairs)
        t_samp = time.perf_counter() - t1
        set_omp_threads(threads)
        t_one = t_rest + (t_samp - t_rest) * (T * Hq) / len(pairs)
        single = dict(value=round(1.0 / t_one, 4), unit="tree steps/s", cores=1,
                      sample=f"top-K, build and walk in full, attention on {len(pairs)} of {T * Hq} rows per "
                             f"sequence scaled to all rows: {t_one:.1f} s/step")
    try:
        cc = subprocess.run(["gcc", "--version"], capture_output=True, text=True).stdout.splitlines()[0]
    except Exception:  # noqa: BLE001
        cc = "gcc"
    return dict(value=round(1.0 / mean_all, 4), unit="tree steps/s", cores=threads, kind="oracle",
                sample=f"{len(t_all)} full steps of the same config-{config} inputs "
                       f"(all {batch}x{T}x{Hq} attention rows), mean {mean_all:.2f} s/step",
                single_thread=single, cpu_model=cpu_model(), host_cpus=os.cpu_count(),
                compiler=cc, flags=" ".join(getattr(oracle, "CFLAGS", [])))


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
    sweep_budgets = [16, 32, 64, 128, 256, 512, 1024] if args.sweep else []
    if args.sweep and batch != 1:
        log("bench.py: --sweep is for the single-sequence configurations")
        sys.exit(2)
    N_max = max([N] + sweep_budgets)
    T_max = N_max + 1
    T = N + 1
    # cache lengths: one sequence of L rows, or (batched configuration) seeded ragged lengths
    Ls = np.array([L]) if batch == 1 else di.ragged_lengths(seed, batch, *L)
    kv_off = [int(v) for v in np.concatenate([[0], np.cumsum(Ls)])]
    sum_L = kv_off[-1]
    bf16 = c["dtype"] == "bf16"

    # ------------------------------------------------------------------ inputs (host, seeded)
    # Generated once for the largest budget asked for; a smaller budget uses the leading rows
    # (the generator is counter-based, so those are the rows it would have drawn anyway).
    t0 = time.time()
    logits_h = np.stack([di.draft_logits(seed, B, V, batch_index=s) for s in range(batch)])
    if batch == 1:
        q_h, kc_h, vc_h, kt_h, vt_h = di.attn_tensors(seed, T_max, L, Hq, Hkv, D, c["dtype"])
    else:  # queries and tree rows of all sequences, one packed ragged cache
        q_h, _, _, kt_h, vt_h = di.attn_tensors(seed, batch * T, 0, Hq, Hkv, D, c["dtype"])
        _, kc_h, vc_h, _, _ = di.attn_tensors(seed + 1, 1, sum_L, Hq, Hkv, D, c["dtype"])
    host = dict(q=q_h, kc=kc_h, vc=vc_h, kt=kt_h, vt=vt_h, kv_off=kv_off)
    tl_plain = [di.target_logits(seed, T_max if batch == 1 else T, V, np.full(T_max if batch == 1 else T, -1),
                                 batch_index=s) for s in range(batch)]
    log(f"[bench] config {args.config} ({c['name']}): inputs generated in {time.time() - t0:.1f}s")

    use_oracle = not args.no_cpu
    if use_oracle:
        import oracle

    def planted_target(lg_h, n_budget, p):
        """Target logits whose argmax is planted along the tree of these draft logits: the CPU
        oracle's tree (and the GPU's tree is checked to be the same one); with --no-cpu, where
        the oracle stays unloaded, the GPU's own."""
        k, t = min(n_budget, V), n_budget + 1
        ws = dd.Workspace(batch, B, V, n_budget, Hq, Hkv, D, sum_L)
        tok_g, lp_g = dd.topk(torch.from_numpy(lg_h).to(dev).contiguous(), k, ws)
        tree_g = dd.build(tok_g, lp_g, n_budget, torch.full((batch,), 11, dtype=torch.int32, device=dev))
        torch.cuda.synchronize()
        depth_g, top1_g = tree_g["depth"].cpu().numpy(), tok_g.cpu().numpy()[:, :, 0]
        out, depths = [], []
        for s in range(batch):
            depth_s, top1_s = depth_g[s], top1_g[s]
            if use_oracle:
                tok_o, lp_o = oracle.topk(lg_h[s], k)
                tr = oracle.build_tree(tok_o, lp_o, n_budget, 11)
                if not (np.array_equal(tr["depth"], depth_s) and np.array_equal(tok_o[:, 0], top1_s)
                        and np.array_equal(tr["parent"], tree_g["parent"][s].cpu().numpy())):
                    raise SystemExit("bench.py: the GPU tree differs from the oracle's tree")
                depth_s, top1_s = tr["depth"], tok_o[:, 0]
            plant = di.planted_tokens(seed, depth_s, top1_s, B, p=p, batch_index=s)
            x = tl_plain[s][:t].copy()
            rows = np.nonzero(plant >= 0)[0]
            x[rows, plant[rows]] = np.float32(10.0)
            out.append(x)
            depths.append(int(depth_s.max()))
        return np.stack(out), max(depths)

    tl_h, max_depth = planted_target(logits_h, N, 0.8)
    log(f"[bench] tree: max depth {max_depth}; all inputs ready after {time.time() - t0:.1f}s")
    wl = Workload(dd, torch, c, N, host, logits_h, tl_h, args.sets)
    n_sets = wl.n_sets

    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ the step's distribution
    # (the same uninstrumented step in blocks of eight; taken first, so that the timed loop below
    # meets a chip that is already at its working clocks whatever --warmup says)
    step_us = step_distribution(torch, wl)

    # ------------------------------------------------------------------ warm-up, then the timed loop
    elapsed = timed_loop(torch, wl, args.steps, args.warmup)
    ms_per_step = 1e3 * elapsed / args.steps
    steps_per_s = args.steps / elapsed
    n_acc = [int(v) for v in wl.acc["n_accepted"].cpu()]
    n_acc = n_acc[0] if batch == 1 else n_acc

    # ------------------------------------------------------------------ roofline of the main kernel
    flops = wl.attn_flops()
    mk = wl.main_kernel
    k_reps = max(args.steps, 128)
    kernel_ms = kernel_times(dd, torch, wl, [mk], k_reps, every=4)[mk]
    k_avg_ms = float(kernel_ms.mean())
    peak = PEAK_BF16_TFLOPS if mk == "attn" else PEAK_FP32_TFLOPS
    achieved = flops / (k_avg_ms * 1e-3) / 1e12
    # HBM bytes per launch from committed rocprofv3 --pmc summaries (FETCH_SIZE + WRITE_SIZE, each
    # scaled by a plain copy of known size); null for workloads that have not been profiled
    traffic = traffic_detail = None
    tpath = os.path.join(ROOT, "profiles", "attn_traffic.json")
    if os.path.exists(tpath) and args.budget == 0:
        try:
            traffic_detail = json.load(open(tpath)).get(f"config{args.config}")
            if traffic_detail:
                traffic = traffic_detail["fetch_bytes"] + traffic_detail["write_bytes"]
        except Exception:  # noqa: BLE001
            traffic = traffic_detail = None
    roofline = dict(bound="mfma" if mk == "attn" else "alu",
                    kernel="attn_mfma_kernel" if mk == "attn" else "attn_generic_kernel",
                    achieved=round(achieved, 2), peak=peak, unit="TFLOP/s", frac=round(achieved / peak, 4),
                    traffic=traffic, traffic_detail=traffic_detail, flops_per_launch=flops,
                    kernel_avg_us=round(1e3 * k_avg_ms, 2), kernel_launches=int(kernel_ms.size),
                    timing="HIP events on the kernel's own dispatch, one launch in 4 of a separate loop of "
                           f"{k_reps} steps (the timed loop carries none)")

    # ------------------------------------------------------------------ per-kernel breakdown
    stages = stage_table(dd, torch, wl)
    if "accept_argmax_us" in stages:
        stages["accept_argmax_GBs"] = round(tl_h.nbytes / (stages["accept_argmax_us"] * 1e-6) / 1e9, 1)
    if "topk_chunk_us" in stages:
        stages["topk_chunk_GBs"] = round(logits_h.nbytes / (stages["topk_chunk_us"] * 1e-6) / 1e9, 1)
    stages["frac_of_roofline"] = stage_fractions(stages, wl, flops)

    # ------------------------------------------------------------------ confident drafter: a deep tree
    stages_peaked = None
    if batch == 1 and not args.no_peaked:
        lg_p = np.stack([di.peaked_draft_logits(seed, B, V, 0.9, batch_index=s) for s in range(batch)])
        tl_p, depth_p = planted_target(lg_p, N, 0.9)
        wlp = Workload(dd, torch, c, N, host, lg_p, tl_p, args.sets)
        n_steps_p = max(100, min(args.steps, 300))
        el = timed_loop(torch, wlp, n_steps_p, 20)
        stp = stage_table(dd, torch, wlp)
        flops_p = wlp.attn_flops()
        stp["frac_of_roofline"] = stage_fractions(stp, wlp, flops_p)
        stages_peaked = dict(workload="the same shapes, every draft row with one token at probability 0.9",
                             max_depth=depth_p, n_accepted=int(wlp.acc["n_accepted"][0]),
                             ms_per_step=round(1e3 * el / n_steps_p, 5), steps_per_s=round(n_steps_p / el, 1),
                             steps=n_steps_p, **stp)
        del wlp

    # ------------------------------------------------------------------ node-budget sweep
    budget_sweep = None
    if args.sweep:
        budget_sweep = []
        for nb in sweep_budgets:
            tl_b, depth_b = planted_target(logits_h, nb, 0.8)
            wb = Workload(dd, torch, c, nb, host, logits_h, tl_b, 0)
            el = timed_loop(torch, wb, 200, 20)
            stb = stage_table(dd, torch, wb)
            fb = wb.attn_flops()
            row = dict(N=nb, ms_per_step=round(1e3 * el / 200, 5), steps_per_s=round(200 / el, 1),
                       max_depth=depth_b, **stb)
            row["attn_frac"] = stage_fractions(stb, wb, fb).get("attn_mfma")
            budget_sweep.append(row)
            log(f"[bench] budget {nb}: {row['ms_per_step'] * 1e3:.1f} us/step")
            del wb
            torch.cuda.empty_cache()

    # ------------------------------------------------------------------ CPU oracle baseline
    cpu = cpu_baseline(wl, host, args.config, 3) if use_oracle else None

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
                   "n_accepted": n_acc, "tree_max_depth": max_depth,
                   "target_argmax_planted_from": "the oracle's tree (GPU tree checked equal)" if use_oracle
                   else "the GPU's tree (--no-cpu)"},
        "step_us": step_us,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "stages": stages,
        "stages_peaked": stages_peaked,
    }
    if budget_sweep is not None:
        result["budget_sweep"] = budget_sweep
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
