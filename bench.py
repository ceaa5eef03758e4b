#!/usr/bin/env python3
"""Benchmark of the MCSD verification step on one MI355X.

One "step" = one mcsd_verify_step call: tree attention of one layer over the
draft tree (prefix KV cache streamed once) followed by the multi-candidate
accept/reject pass over the vocabulary and the root-to-leaf walk.  Inputs are
seeded synthetic tensors resident in HBM before the timed region starts.

Prints ONE JSON line.  Metric: verified draft-tree nodes per second
(B * N / step time).  `roofline` describes the dominant kernel (tree attention)
from per-kernel execution times (HIP events tied to each dispatch) taken in a second pass
over the same work; `cpu_baseline` is the CPU oracle timed on a bounded sample of the same
workload.  The default run measures the batched workload c4 (headline, bound by HBM) and adds
the long-prompt GQA workload c5 (bound by the matrix cores) as `secondary`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

# HBM traffic per launch of the tree-attention kernel measured with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); see the
# summaries under profiles/.  None = not measured for that workload.
MEASURED_TRAFFIC_BYTES = {"c4": 655631815, "c5": 348566826, "c3": 50875781, "c2": 9534005}   # profiles/step_<workload>.md


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--stage", default="verify_step", choices=["verify_step", "draft_sample", "kv_commit", "no_tree_attention", "paged_attention"],
                    help="verify_step (default): the headline step; draft_sample: the draft-side candidate "
                         "sampler that precedes it; kv_commit: tree build + commit of the accepted path that "
                         "follows it (8 layers); no_tree_attention: the same attention with one private "
                         "prefix-cache copy per candidate sequence (what tree attention replaces), timed next to "
                         "tree attention; paged_attention: tree attention with the prefix cache in a page pool "
                         "(--page-size), timed next to the contiguous layout; each measured on its own")
    ap.add_argument("--page-size", type=int, default=64, help="tokens per page for --stage paged_attention")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="with the default workload (c4), do not also measure c5 for the `secondary` object")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--sets", type=int, default=0, help="rotating input copies (0 = enough for >= 1 GiB)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a few device-to-device copies of 1 GiB (a plain copy kernel of known "
                         "size) for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters, then exit")
    return ap.parse_args()


def cpu_baseline(w, ai, vi, target_seconds):
    """Times the oracle (as it stands) on a bounded sample of the workload with all host
    threads: a random subset of attention rows sized for about 70 % of the time budget (all
    rows if they fit) plus the verification of whole sequences, extrapolated to one step."""
    from oracle import mcsd_oracle as O
    threads = min(O.max_threads(), os.cpu_count() or 1)
    dt = O.FP32 if ai.dtype == "fp32" else O.BF16
    rng = np.random.default_rng(0)
    total_rows = ai.B * ai.N * ai.H_q

    def attn_time(n):
        if n >= total_rows:
            sel = None
        else:
            sel = np.stack([rng.integers(0, ai.B, n), rng.integers(0, ai.N, n), rng.integers(0, ai.H_q, n)],
                           axis=1).astype(np.int32)
        t0 = time.perf_counter()
        O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                    dt, sel=sel, n_threads=threads)
        return time.perf_counter() - t0

    pilot_n = 4 * threads
    per_row = attn_time(pilot_n) / pilot_n
    n_rows = int(min(total_rows, max(pilot_n, 0.7 * target_seconds / max(per_row, 1e-9))))
    t_attn = attn_time(n_rows)

    t0 = time.perf_counter()
    O.verify(vi.target_logits, vi.draft_logits, vi.tree.q_row, vi.tree.parent, vi.cand_tok, vi.u_accept,
             vi.u_endpoint, vi.temperature, vi.variant, gamma_max=vi.tree.gamma, n_threads=threads)
    t_ver = time.perf_counter() - t0
    est_step = t_attn * total_rows / n_rows + t_ver
    # one thread, on a fifth of the budget: attention rows only (the verification of all rows
    # on one thread would not fit the budget for the large workloads; it scales the same way)
    n1 = max(4, int(0.2 * target_seconds / max(per_row * threads, 1e-9)))
    n1 = min(n1, total_rows)
    sel1 = np.stack([rng.integers(0, ai.B, n1), rng.integers(0, ai.N, n1), rng.integers(0, ai.H_q, n1)],
                    axis=1).astype(np.int32)
    t0 = time.perf_counter()
    O.tree_attn(ai.q, ai.k_prefix, ai.v_prefix, ai.prefix_len, ai.k_tree, ai.v_tree, ai.parent, ai.scale,
                dt, sel=sel1, n_threads=1)
    t1_row = (time.perf_counter() - t0) / n1
    return {
        "single_thread_attention_rows_per_s": 1.0 / t1_row,
        "all_threads_attention_rows_per_s": n_rows / t_attn,
        "value": vi.B * vi.N / est_step, "unit": "nodes/s", "cores": threads, "kind": "oracle",
        "sample": f"{n_rows} of {total_rows} attention rows in {t_attn:.3f} s + verification of all "
                  f"{vi.B} sequences in {t_ver:.3f} s; one full step extrapolates to {est_step:.3f} s",
    }


def bench_draft_sample(args, torch, M, D, W):
    """The sampler that produces the candidates the verification step consumes: one launch per
    step over all draft rows of the workload (B x P rows of V fp32 logits, each read once)."""
    w = W.WORKLOADS[args.workload]
    vi = W.gen_verify_inputs(w)
    u = W.open_uniform(np.random.default_rng(w.seed + 7), (vi.B, vi.N))
    design_bytes = vi.B * vi.P * vi.V * 4
    n_sets = args.sets if args.sets > 0 else max(2, int(np.ceil((1 << 30) / design_bytes)))
    n_sets = min(n_sets, 64)
    sets = [D.make_draft_call(vi, u) for _ in range(n_sets)]
    torch.cuda.synchronize()

    def run(n, off=0):
        for i in range(n):
            M.mcsd_draft_sample(sets[(off + i) % n_sets].args)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    M.mcsd_kernel_timing(True)
    run(args.steps, args.warmup + args.steps)
    torch.cuda.synchronize()
    kt = M.mcsd_kernel_timing_read()
    M.mcsd_kernel_timing(False)
    k_us = 1e3 * kt["draft_rows"][0] / kt["draft_rows"][1]
    out = {
        "metric": "draft candidates sampled per second (k per parent from softmax(z_q/T))",
        "value": vi.B * vi.N / (ms * 1e-3), "unit": "candidates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} draft rows: {w.description}", "B": w.B, "draft_rows": vi.P,
                   "nodes": vi.N, "V": vi.V, "input_sets": n_sets,
                   "variant": "without_replacement" if vi.variant else "with_replacement"},
        "roofline": {"kernel": "draft_rows", "bound": "hbm", "achieved": design_bytes / (k_us * 1e-6) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": design_bytes / (k_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "traffic": None, "algorithmic_bytes": design_bytes, "avg_kernel_us": k_us},
    }
    if not args.no_cpu_baseline:
        from oracle import mcsd_oracle as O
        threads = min(O.max_threads(), os.cpu_count() or 1)
        t0 = time.perf_counter()
        O.draft_sample(vi.draft_logits, vi.tree.q_row, vi.tree.parent, u, vi.temperature, vi.variant, n_threads=threads)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": vi.B * vi.N / dt, "unit": "candidates/s", "cores": threads, "kind": "oracle",
                               "sample": f"all {vi.B * vi.P} draft rows of the workload in {dt:.3f} s"}
    print(json.dumps(out))


def bench_kv_commit(args, torch, M, D, W):
    """mcsd_tree_build + mcsd_kv_commit for the workload's shape with 8 layers of cache: the accepted
    paths come from one verification of the workload; prefix_len is reset on the device between steps."""
    from oracle import mcsd_oracle as O
    w = W.WORKLOADS[args.workload]
    ai, vi = W.gen_attn_inputs(w), W.gen_verify_inputs(w)
    n_layers, dev = 8, "cuda:0"
    ref = O.verify(vi.target_logits, vi.draft_logits, vi.tree.q_row, vi.tree.parent, vi.cand_tok, vi.u_accept,
                   vi.u_endpoint, vi.temperature, vi.variant, gamma_max=vi.tree.gamma, n_threads=16)
    B, N, H_kv, d, Ls, G = ai.B, ai.N, ai.H_kv, ai.d, ai.k_prefix.shape[2], vi.tree.gamma
    bf = torch.bfloat16
    kp = torch.zeros((n_layers, B, H_kv, Ls, d), dtype=bf, device=dev)
    vp = torch.zeros_like(kp)
    kt = torch.randn((n_layers, B, H_kv, N, d), device=dev).to(bf)
    vt = torch.randn((n_layers, B, H_kv, N, d), device=dev).to(bf)
    L0 = torch.from_numpy(np.minimum(ai.prefix_len, Ls - G).astype(np.int32)).to(dev)
    L = L0.clone()
    i32 = dict(dtype=torch.int32, device=dev)
    n_acc = torch.from_numpy(ref.n_accepted).to(dev)
    path = torch.from_numpy(ref.accepted_path).to(dev)
    otok = torch.from_numpy(ref.out_tokens).to(dev)
    nxt, fl = torch.empty((B,), **i32), torch.empty((B,), **i32)
    parent, depth = torch.empty((N,), **i32), torch.empty((N,), **i32)
    q_row, pos = torch.empty((N + 1,), **i32), torch.empty((B, N), **i32)
    cargs = M.commit_args(kp, vp, kt, vt, n_acc, path, otok, L, nxt, fl)
    moved = int(ref.n_accepted.sum()) * H_kv * d * 2 * 2 * 2 * n_layers      # K and V, read + write

    def run(n):
        for _ in range(n):
            L.copy_(L0)
            M.mcsd_tree_build(w.kconfig, parent, depth, q_row, prefix_len=L, position_ids=pos)
            M.mcsd_kv_commit(cargs)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    M.mcsd_kernel_timing(True)
    run(args.steps)
    torch.cuda.synchronize()
    kt_ = M.mcsd_kernel_timing_read()
    M.mcsd_kernel_timing(False)
    kernels = {k: 1e3 * ms_ / n for k, (ms_, n) in kt_.items() if n}
    out = {
        "metric": "tree build + KV commit of the accepted paths (8 layers) per second", "value": 1e3 / ms,
        "unit": "commits/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name} commit: {w.description}", "B": B, "layers": n_layers, "H_kv": H_kv, "d": d,
                   "accepted_total": int(ref.n_accepted.sum()), "bytes_moved": moved,
                   "note": "ms_per_step includes the device-side reset of prefix_len (one small copy)"},
        "roofline": {"kernel": "kv_copy", "bound": "hbm", "achieved": moved / (kernels["kv_copy"] * 1e-6) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": moved / (kernels["kv_copy"] * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "traffic": None, "algorithmic_bytes": moved, "avg_kernel_us": kernels["kv_copy"]},
        "kernels_us": kernels,
    }
    if not args.no_cpu_baseline:
        kph, vph = kp.view(torch.int16).cpu().numpy().view(np.uint16), vp.view(torch.int16).cpu().numpy().view(np.uint16)
        kth, vth = kt.view(torch.int16).cpu().numpy().view(np.uint16), vt.view(torch.int16).cpu().numpy().view(np.uint16)
        Lh = L0.cpu().numpy()
        import ctypes
        lib, P_ = O.lib(), O._ptr
        nr, full = np.empty(B, np.int32), np.empty(B, np.int32)
        t0 = time.perf_counter()
        reps = 20
        for _ in range(reps):
            Lc = Lh.copy()
            O.tree_build(w.kconfig)
            lib.mcsd_oracle_kv_commit(n_layers, B, N, H_kv, d, 2, Ls, G, 0, P_(kph), P_(vph), P_(kth), P_(vth),
                                      P_(ref.n_accepted), P_(ref.accepted_path), P_(ref.out_tokens), P_(Lc), P_(nr), P_(full))
        dt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": 1.0 / dt, "unit": "commits/s", "cores": 1, "kind": "oracle",
                               "sample": f"the same commit, in place on host copies of the caches, {reps} repetitions"}
    print(json.dumps(out))


def bench_no_tree_attention(args, torch, M, D, W):
    """Tree attention against the arrangement it replaces (Sec. 3.3): every root-to-leaf candidate
    sequence as a sequence of its own with a private copy of the prefix cache, run through the same
    kernel as a chain.  One input set each (the replicated caches are n_leaves times larger)."""
    w = W.WORKLOADS[args.workload]
    ai = W.gen_attn_inputs(w)
    tree = D.make_attn_call(ai)
    rep = D.make_replicated_attn_call(tree, ai)
    n_leaves, depth = len(rep.paths), len(rep.paths[0])
    e = 2 if ai.dtype == "bf16" else 4
    rep_bytes = 2 * ai.H_kv * ai.d * e * n_leaves * (int(ai.prefix_len.sum()) + ai.B * depth) \
        + 2 * ai.B * n_leaves * depth * ai.H_q * ai.d * e
    res = {}
    for name, call in (("tree", tree), ("replicated", rep)):
        for _ in range(args.warmup):
            M.mcsd_tree_attn(call.args)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            M.mcsd_tree_attn(call.args)
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) * 1e6 / args.steps
    out = {
        "metric": "attention time without / with tree attention (same candidates, same kernel)",
        "value": res["replicated"] / res["tree"], "unit": "x", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["tree"] * 1e-3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if ai.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} attention: {w.description}", "candidate_sequences": ai.B * n_leaves,
                   "depth": depth, "tree_nodes": ai.N, "input_sets": 1},
        "tree_us": res["tree"], "replicated_us": res["replicated"],
        "tree_bytes": ai.algorithmic_bytes(), "replicated_bytes": rep_bytes,
        "tree_gbs": ai.algorithmic_bytes() / res["tree"] / 1e3, "replicated_gbs": rep_bytes / res["replicated"] / 1e3,
        "roofline": {"kernel": "tree_attn_mfma (replicated sequences)", "bound": "hbm",
                     "achieved": rep_bytes / res["replicated"] / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": rep_bytes / res["replicated"] / 1e3 / HBM_PEAK_GBS, "traffic": None},
    }
    print(json.dumps(out))


def bench_paged_attention(args, torch, M, D, W):
    """mcsd_tree_attn_paged (prefix cache scattered over a page pool in random page order) next to
    mcsd_tree_attn on the same data; rotating input sets as in the headline benchmark."""
    w = W.WORKLOADS[args.workload]
    ai = W.gen_attn_inputs(w)
    n_sets = args.sets if args.sets > 0 else max(2, int(np.ceil((1 << 30) / ai.algorithmic_bytes())))
    n_sets = min(n_sets, 64)
    cont = [D.make_attn_call(ai) for _ in range(n_sets)]
    paged = [D.make_paged_attn_call(c, ai, args.page_size, seed=i)[:2] for i, c in enumerate(cont)]
    torch.cuda.synchronize()
    res = {}
    for name in ("contiguous", "paged"):
        def run(n, off=0):
            for i in range(n):
                j = (off + i) % n_sets
                if name == "contiguous":
                    M.mcsd_tree_attn(cont[j].args)
                else:
                    M.mcsd_tree_attn_paged(paged[j][0].args, paged[j][1])
        run(args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps, args.warmup)
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) * 1e6 / args.steps
    b = ai.algorithmic_bytes()
    out = {
        "metric": "tree attention over a paged prefix cache: achieved HBM GB/s (attention + combine)",
        "value": b / res["paged"] / 1e3, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["paged"] * 1e-3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if ai.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} attention: {w.description}", "page_size": args.page_size, "input_sets": n_sets},
        "paged_us": res["paged"], "contiguous_us": res["contiguous"], "contiguous_gbs": b / res["contiguous"] / 1e3,
        "roofline": {"kernel": "tree_attn_mfma (paged) + combine", "bound": "hbm", "achieved": b / res["paged"] / 1e3,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": b / res["paged"] / 1e3 / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes": b},
    }
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build measures one GPU only (got --gpus {args.gpus}); the path shards by "
              "sequence / KV head without any exchange", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2401_06706_amd import binding as M
    from paper_2401_06706_amd import device as D
    from paper_2401_06706_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    M.lib()     # fails loudly if libmcsd.so is not built
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": src.numel() * 4, "copies": 4}))
        return
    if args.stage == "draft_sample":
        bench_draft_sample(args, torch, M, D, W)
        return
    if args.stage == "kv_commit":
        bench_kv_commit(args, torch, M, D, W)
        return
    if args.stage == "no_tree_attention":
        bench_no_tree_attention(args, torch, M, D, W)
        return
    if args.stage == "paged_attention":
        bench_paged_attention(args, torch, M, D, W)
        return
    out = measure_step(args, args.workload, torch, M, D, W, with_cpu_baseline=not args.no_cpu_baseline)
    if args.workload == "c4" and not args.no_secondary:
        # the second long-prefix workload, bound by the matrix cores instead of HBM
        torch.cuda.empty_cache()
        sec = measure_step(args, "c5", torch, M, D, W, with_cpu_baseline=False)
        out["secondary"] = {k: sec[k] for k in ("value", "unit", "ms_per_step", "dtype", "config", "step_ms_event_p10_p50_p90",
                                                 "hot_cache_ms_per_step", "step_hbm_gbs", "step_hbm_frac", "roofline",
                                                 "verify_roofline", "kernels", "kernels_sum_us")}
    print(json.dumps(out))


def measure_step(args, workload, torch, M, D, W, with_cpu_baseline):
    """Times mcsd_verify_step on one workload: wall clock over back-to-back steps on rotating
    input sets, then per-kernel execution times from the events of each dispatch."""
    dev = "cuda:0"
    w = W.WORKLOADS[workload]
    ai = W.gen_attn_inputs(w)
    vi = W.gen_verify_inputs(w)

    attn_bytes = ai.algorithmic_bytes()
    verify_bytes = vi.design_bytes()
    footprint = attn_bytes + verify_bytes
    n_sets = args.sets if args.sets > 0 else max(2, int(np.ceil((1 << 30) / footprint)))
    n_sets = min(n_sets, 128)
    sets = []
    for s in range(n_sets):
        # every set holds the same values at different addresses, so no cache level can
        # serve one step's reads from the previous step
        sets.append((D.make_attn_call(ai, dev), D.make_verify_call(vi, dev, want_ratio=False)))
    torch.cuda.synchronize()

    def run(n_steps, offset=0):
        for i in range(n_steps):
            a, v = sets[(offset + i) % n_sets]
            M.mcsd_verify_step(a.args, v.args)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # second pass, same work: every kernel dispatch carries its own start / stop events, so the
    # durations are kernel execution times (as in a kernel trace) and add up to less than a step
    M.mcsd_kernel_timing(True)
    run(args.steps, args.warmup + args.steps)
    torch.cuda.synchronize()
    ktimes = M.mcsd_kernel_timing_read()
    M.mcsd_kernel_timing(False)
    kernels = {k: {"avg_us": 1e3 * ms / n, "launches": n} for k, (ms, n) in ktimes.items() if n > 0}
    kernels_sum_us = sum(v["avg_us"] * v["launches"] for v in kernels.values()) / args.steps

    # third pass: one event pair per step for the spread, then the same step on ONE input set
    # (the 256 MB memory-side cache then serves part of the reads): labelled, never the headline
    def per_step_times(n_steps, offset, one_set=False):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_steps)]
        for i, (e0, e1) in enumerate(evs):
            a, v = sets[0 if one_set else (offset + i) % n_sets]
            e0.record()
            M.mcsd_verify_step(a.args, v.args)
            e1.record()
        torch.cuda.synchronize()
        return np.array([e0.elapsed_time(e1) for e0, e1 in evs])

    n_spread = min(args.steps, 100)
    spread = per_step_times(n_spread, 0)
    hot = per_step_times(n_spread, 0, one_set=True)

    dom = "tree_attn_mfma"
    dom_us = kernels[dom]["avg_us"]
    achieved = attn_bytes / (dom_us * 1e-6) / 1e9
    flops = ai.flops()
    tflops = flops / (dom_us * 1e-6) / 1e12
    # the roof that binds: matrix cores where the arithmetic intensity (flops per algorithmic byte)
    # lies above the ridge of the two published peaks, HBM below it; both fractions are reported
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    if flops / attn_bytes > ridge:
        roofline = {"kernel": dom, "bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": tflops / MFMA_BF16_PEAK_TFLOPS}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS}
    roofline.update({"traffic": MEASURED_TRAFFIC_BYTES.get(workload),
                     "traffic_source": f"profiles/step_{workload}.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, a run of its own)",
                     "algorithmic_bytes": attn_bytes,
                     "algorithmic_flops": flops, "avg_kernel_us": dom_us,
                     "hbm_gbs": achieved, "hbm_frac": achieved / HBM_PEAK_GBS,
                     "mfma_tflops": tflops, "mfma_frac": tflops / MFMA_BF16_PEAK_TFLOPS})
    ver_us = kernels["verify_rows"]["avg_us"]
    # path-only minimum next to the design bytes: the rows a sequential walk would touch at most
    # (gamma + 1 target rows, and gamma draft rows for a sampled sequence)
    g = vi.tree.gamma
    path_rows = sum((g + 1) + (0 if T == 0.0 else g) for T in vi.temperature)
    verify_roof = {"kernel": "verify_rows", "bound": "hbm", "achieved": verify_bytes / (ver_us * 1e-6) / 1e9,
                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": verify_bytes / (ver_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                   "algorithmic_bytes": verify_bytes, "design_bytes_every_row": verify_bytes,
                   "path_only_bytes": int(path_rows) * vi.V * 4, "avg_kernel_us": ver_us}

    out = {
        "metric": "verified draft-tree nodes/sec (tree-attn + MCSD sample); achieved HBM GB/s",
        "value": w.B * ai.N / (ms_per_step * 1e-3),
        "unit": "nodes/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.description}", "B": w.B, "tree": "x".join(map(str, w.kconfig)),
                   "nodes": ai.N, "H_q": w.H_q, "H_kv": w.H_kv, "d": w.d, "V": w.V,
                   "prefix_tokens_total": int(ai.prefix_len.sum()), "input_sets": n_sets,
                   "variant": "without_replacement" if vi.variant else "with_replacement"},
        "step_ms_event_p10_p50_p90": [float(x) for x in np.percentile(spread, [10, 50, 90])],
        "hot_cache_ms_per_step": float(np.median(hot)),
        "step_hbm_gbs": footprint / (ms_per_step * 1e-3) / 1e9,
        "step_hbm_frac": footprint / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": roofline,
        "verify_roofline": verify_roof,
        "kernels": kernels,
        "kernels_sum_us": kernels_sum_us,
    }
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, ai, vi, args.cpu_seconds)
    del sets
    return out


if __name__ == "__main__":
    main()
