#!/usr/bin/env python3
"""Benchmark of the CUSA decode hot path on one MI355X.

A "step" is the attention part of one decode step of the paper's Alg. 1 over all layers of
the workload: full-attention layers, the selection layer (full attention that also emits the
scores + per-head top-k + cross-head union + window) and the sparse-attention layers that reuse rho.  Inputs are
seeded, synthetic and resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

Prints ONE JSON line: the step time, a `roofline` object for the kernel that takes most of the
step (algorithmic bytes / its HIP-event duration against the 8 TB/s HBM peak), per-kernel
figures, the speedup over this library's own full attention on every layer, and `cpu_baseline`,
the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "loop"],
                    help="c1..c5: one decode step at fixed lengths (c2 is the configuration the metric is quoted on); "
                         "loop: consecutive decode steps, every sequence one token longer after each")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step into one HIP graph and time its replays (the library only enqueues kernels)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--rank-study", action="store_true",
                    help="also compare the three readings of the global ranking and the per-head sets: overlap of rho "
                         "and attention recall (Eq. 3) on the selection layer and on the last sparse layer")
    ap.add_argument("--head-overlap", type=float, default=None, metavar="S",
                    help="redraw the workload with a rank-8 component of scale S shared by all heads of a sequence "
                         "(0 = independent heads, 4 = nearly identical picks): sets how much the heads' top-k sets overlap")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-baseline", action="store_true")
    ap.add_argument("--no-per-head", action="store_true",
                    help="skip the head-to-head comparison (every head attends its own top-k instead of the unified set)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the HIP-event pass (use under rocprofv3 to keep the trace to the timed steps)")
    return ap.parse_args()


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def kernel_bytes(w, lens, acc):
    """Algorithmic bytes of ONE launch of each bandwidth-bound kernel (all sequences of the batch)."""
    G, K, W = w.n_kv_heads, w.budget, w.window
    return {
        "attn_kernel<full>": sum(acc.full_attn_bytes(G, L) for L in lens),
        "attn_kernel<sparse>": sum(acc.sparse_attn_bytes(G, K, L) for L in lens),
        "score_kernel": sum(acc.score_bytes(G, L, K, W) for L in lens),
        # the selection layer's pass: K and V once, the scores come from the same K rows
        "attn_kernel<full+score>": sum(acc.full_attn_bytes(G, L) for L in lens),
    }


def per_head_comparison(r, w, sched, lens, steps, torch, cb, acc):
    """The sparse layers of the step with per-head token sets (head-to-head selection, the variant the
    paper's kernel comparison is against) next to the same layers with the unified set."""
    sel = sched.index(1)
    sparse_layers = [i for i, k in enumerate(sched) if k == 2]
    idx_head = r.make_idx_head()
    r.select_per_head(sel, idx_head)
    r.select(sel)
    torch.cuda.synchronize()
    g = w.n_q_heads // w.n_kv_heads
    n = min(w.budget, min(lens))
    # distinct rows a KV group's heads ask for, relative to one head's list (1 = identical lists, g = disjoint)
    grp = idx_head[:, :, :n].reshape(w.batch * w.n_kv_heads, g * n)
    distinct = sum(int(torch.unique(row).numel()) for row in grp[: 64]) / (min(64, grp.shape[0]) * n)

    def unified():
        for i in sparse_layers:
            r.sparse(i)

    def per_head():
        for i in sparse_layers:
            r.sparse_per_head(i, idx_head)

    t_uni = time_steps(unified, steps, 2, torch)
    t_ph = time_steps(per_head, steps, 2, torch)
    cb.profile_reset()
    cb.profile_enable(True)
    for _ in range(steps):
        unified()
        per_head()
    torch.cuda.synchronize()
    prof = cb.profile_read()
    cb.profile_enable(False)
    ku = prof["attn_kernel<sparse>"]
    kp = prof["attn_kernel<per-head>"]
    ku_us, kp_us = ku["total_ms"] * 1e3 / ku["calls"], kp["total_ms"] * 1e3 / kp["calls"]
    b_uni = sum(acc.sparse_attn_bytes(w.n_kv_heads, w.budget, L) for L in lens)
    b_ph = sum(acc.per_head_sparse_attn_bytes(w.n_q_heads, w.budget, L) for L in lens)
    return {"sparse_layers": len(sparse_layers), "unified_us": round(t_uni * 1e6, 2), "per_head_us": round(t_ph * 1e6, 2),
            "per_head_over_unified": round(t_ph / t_uni, 3),
            "kernel_us": {"unified": round(ku_us, 3), "per_head": round(kp_us, 3), "ratio": round(kp_us / ku_us, 3)},
            "kernel_bytes": {"unified": b_uni, "per_head": b_ph},
            "per_head_GBs": round(b_ph / (kp_us * 1e-6) / 1e9, 1),
            "distinct_rows_per_group_over_list": round(distinct, 3), "gqa_group": g}


def rank_study(inp, w, sched, torch, StepRunner):
    """How much the readings of "globally ranked" differ on this workload: |rho ∩ rho_first| / |rho| and the
    recall of Eq. 3 (mean and minimum over sequences and heads), on the selection layer's own q, K and on the
    last sparse layer's (rho reused there); per-head sets (every head its own top-k) for comparison."""
    sel = sched.index(1)
    last = max(i for i, k in enumerate(sched) if k == 2)
    names = {0: "first_occurrence", 1: "votes", 2: "max_score"}
    res, base = {}, None

    def stats(t):
        return {"mean": round(float(t.mean()), 5), "min": round(float(t.min()), 5)}

    for mode in (0, 1, 2):
        r = StepRunner(inp, sched, rank_mode=mode)
        r.select(sel)
        torch.cuda.synchronize()
        rho = [set(r.idx[b, : int(r.cnt[b])].tolist()) for b in range(w.batch)]
        if base is None:
            base = rho
        same = sum(len(a & b) for a, b in zip(rho, base)) / sum(len(a) for a in rho)
        res[names[mode]] = {"share_of_rho_in_first_occurrence_rho": round(same, 5),
                            "recall_select_layer": stats(r.recall(sel)), "recall_last_sparse_layer": stats(r.recall(last))}
        if mode == 0:
            idx_head = r.make_idx_head()
            r.select_per_head(sel, idx_head)
            res["per_head_sets"] = {"recall_select_layer": stats(r.recall(sel, idx_head)),
                                    "recall_last_sparse_layer": stats(r.recall(last, idx_head))}
        del r
    return res


def cpu_baseline(inp, w, sched):
    """Oracle wall time for one step on the host cores.

    One layer of each kind is timed on sequence 0 first; if that projects to at most 30 s the whole
    step (every layer, every sequence) is run and its measured time reported, otherwise the
    projection is."""
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import host_view

    def timed(fn):
        t0 = time.perf_counter()
        r = fn()
        return time.perf_counter() - t0, r

    sel = sched.index(1)
    q, K, V = host_view(inp, sel, 0)
    t_full, _ = timed(lambda: oracle.attention(q, K, V))
    t_sel, rho0 = timed(lambda: oracle.select(q, K, w.budget, w.window, w.topk_per_head))
    sp = sched.index(2)
    q, K, V = host_view(inp, sp, 0)
    t_sparse, _ = timed(lambda: oracle.attention(q, K, V, rho0))
    n_full = sum(1 for k in sched if k in (0, 1))
    n_sparse = sum(1 for k in sched if k == 2)
    scale = sum(inp.seq_lens_host) / inp.seq_lens_host[0]          # other sequences, by length
    projected = (n_full * t_full + t_sel) * scale + n_sparse * t_sparse * w.batch
    base = {"unit": "us", "cores": oracle.num_threads(), "kind": "oracle"}
    if projected > 30.0:
        base.update(value=projected * 1e6,
                    sample=(f"sequence 0 of {w.batch}: one full-attention layer ({t_full:.3f} s), one selection "
                            f"({t_sel:.3f} s), one sparse layer ({t_sparse:.4f} s); projected to {n_full} full + 1 select + "
                            f"{n_sparse} sparse layers and to all sequences by length"))
        return base
    total = 0.0
    rho = [None] * w.batch
    for i, kind in enumerate(sched):
        for b in range(w.batch):
            q, K, V = host_view(inp, i, b)                            # device -> host copy, not timed
            if kind == 2:
                dt, _ = timed(lambda: oracle.attention(q, K, V, rho[b]))
            else:
                dt, _ = timed(lambda: oracle.attention(q, K, V))
                if kind == 1:
                    d2, rho[b] = timed(lambda: oracle.select(q, K, w.budget, w.window, w.topk_per_head))
                    dt += d2
            total += dt
    base.update(value=total * 1e6,
                sample=f"the whole step: all {len(sched)} layers of all {w.batch} sequences, oracle calls only (host copies of the inputs not timed)")
    return base


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the hot path shards by sequence "
              "and KV head without communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    from paper_2508_07101_amd import accounting as acc
    from paper_2508_07101_amd import binding as cb
    from paper_2508_07101_amd import workloads as wl
    from paper_2508_07101_amd.runner import StepRunner

    w = wl.WORKLOADS[args.workload]
    if args.head_overlap is not None:
        w = wl.scaled(w, lowrank=8, lowrank_scale=args.head_overlap, n_planted=0)
    inp = wl.make_inputs(w, "cuda:0")
    sched = list(w.schedule)
    lens = inp.seq_lens_host
    r = StepRunner(inp, sched)
    torch.cuda.synchronize()

    run_step = r.run
    if w.grow_room > 0:
        if args.graph or args.steps + args.warmup > w.grow_room:
            print(f"workload {w.name}: at most {w.grow_room} steps (warm-up included), and no --graph", file=sys.stderr)
            sys.exit(2)

        def run_step():                           # one decode step, then the sequences are one token longer
            r.run()
            r.grow(1)
    if args.graph:
        r.run()                                   # warm the library before capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            r.run()
        run_step = graph.replay
    step_s = time_steps(run_step, args.steps, args.warmup, torch)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    full_s = None
    if not args.no_full_baseline:
        rf = StepRunner(inp, [0] * len(sched))
        full_s = time_steps(rf.run, max(3, args.steps // 4), 1, torch)
        del rf

    kernels, roofline = {}, None
    if not args.no_kernel_timing:
        cb.profile_reset()
        cb.profile_enable(True)
        for _ in range(args.steps):
            r.run()
        torch.cuda.synchronize()
        prof = cb.profile_read()
        cb.profile_enable(False)
        kb = kernel_bytes(w, lens, acc)
        for name, p in prof.items():
            if p["calls"] == 0:
                continue
            avg_us = p["total_ms"] * 1e3 / p["calls"]
            k = {"launches_per_step": p["calls"] // args.steps, "avg_us": round(avg_us, 3),
                 "us_per_step": round(p["total_ms"] * 1e3 / args.steps, 3)}
            if name in kb and kb[name] > 0:
                k["bytes_per_launch"] = kb[name]
                k["achieved_GBs"] = round(kb[name] / (avg_us * 1e-6) / 1e9, 1)
                k["frac_of_hbm_peak"] = round(k["achieved_GBs"] / HBM_PEAK_GBS, 4)
            kernels[name] = k
        hot = max((n for n in kernels if "achieved_GBs" in kernels[n]), key=lambda n: kernels[n]["us_per_step"])
        traffic = None                            # HBM bytes per launch from rocprofv3 counters, if a summary is committed
        tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch", {}).get(hot)
        roofline = {"kernel": hot, "bound": "hbm", "achieved": kernels[hot]["achieved_GBs"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": kernels[hot]["frac_of_hbm_peak"], "traffic": traffic,
                    "bytes_per_launch": kernels[hot]["bytes_per_launch"], "avg_us": kernels[hot]["avg_us"]}

    sb = acc.step_bytes(sched, lens, w.n_kv_heads, w.budget, w.window)
    out = {
        "metric": "us_per_decode_step_select_plus_sparse_attn",
        "value": round(step_s * 1e6, 2), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_s * 1e3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_layers} layers, batch {w.batch}, {w.n_q_heads}q/{w.n_kv_heads}kv heads, "
                               f"d {w.head_dim}, L {min(lens)}..{max(lens)}, budget {w.budget}, window {w.window}, "
                               f"top-k/head {w.k_eff}, {'paged' if w.paged else 'contiguous'} KV",
                   "schedule": "".join("FSs"[k] for k in sched), "launch": "hip_graph" if args.graph else "stream",
                   "sinks": w.n_sink, "lengths": "grow by one token per step" if w.grow_room > 0 else "fixed",
                   **({"head_overlap": args.head_overlap} if args.head_overlap is not None else {})},
        "step_algorithmic_bytes": sb["total"],
        "step_achieved_GBs": round(sb["total"] / step_s / 1e9, 1),
        "roofline": roofline,
        "kernels": kernels,
    }
    if full_s is not None:
        out["full_attention_all_layers_us"] = round(full_s * 1e6, 2)
        out["speedup_vs_full_attention"] = round(full_s / step_s, 3)
    if not args.no_per_head and 2 in sched:
        out["per_head_comparison"] = per_head_comparison(r, w, sched, lens, max(3, args.steps // 2), torch, cb, acc)
    if args.rank_study and 2 in sched:
        out["rank_study"] = rank_study(inp, w, sched, torch, StepRunner)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, w, sched)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
