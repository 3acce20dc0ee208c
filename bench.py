#!/usr/bin/env python3
"""Benchmark of the CUSA decode hot path on one MI355X.

A "step" is the attention part of one decode step of the paper's Alg. 1 over all layers of a
workload: full-attention layers, the selection layer (full attention whose pass over K also emits
the scores, then per-head top-k, cross-head union and the recency window) and the sparse-attention
layers that reuse rho.  Inputs are seeded, synthetic and resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workloads c1,c2,c3,c4,c5]

One invocation measures every listed workload (default: the five quoted configurations, in that
order) and prints ONE JSON line.  The top-level figures (`value`, `config`, `roofline`,
`cpu_baseline`) are those of the LAST workload listed -- by default c5, the largest configuration
one GPU holds (21.5 GB of KV cache, 6.5 GB moved per step); `configs` carries one record per
workload with

  * us_per_step: mean over the K timed steps (wall clock around exactly K steps) and the median and
    minimum of the K step durations taken from events recorded between the steps;
  * kernels: per kernel, launches per step and the dispatch duration (begin to end time stamp, what a
    kernel trace reports), mean / median-free average over all launches of the K steps;
  * rooflines: for every bandwidth-bound kernel of the step (sparse attention, the selection layer's
    pass, plain full attention) algorithmic bytes per launch / its average duration against the
    8 TB/s HBM peak;
  * the same stack with full attention on every layer, and the speed-up over it;
  * cpu_baseline: the CPU oracle timed on a bounded sample (sequence 0: one full-attention layer,
    one selection, one sparse layer; whole step when that is short), split by stage, with the
    core count; c1 also single-threaded.

`traffic_probes` are the read rates of kernels that only move data, measured in the same run: a plain
streaming read, gathered 256-byte rows, and a streaming read with a few per cent of writes (scattered,
and in workgroup bursts) -- the practical ceilings to set beside the nominal peak for full attention,
sparse attention and the selection layer's pass.
"""
import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
QUOTED = ["c1", "c2", "c3", "c4", "c5"]
BANDWIDTH_KERNELS = ("attn_kernel<sparse>", "attn_kernel<full+score>", "attn_kernel<full>", "attn_kernel<scores only>")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workloads", "--workload", dest="workloads", default=",".join(QUOTED),
                    help="comma-separated list of c1..c5 and loop (consecutive decode steps, every sequence one "
                         "token longer after each); the last one listed supplies the top-level figures")
    ap.add_argument("--entry", default="step", choices=["step", "select"],
                    help="what a timed call is: the whole decode step (cusa_decode_step), or cusa_select on the selection "
                         "layer alone (the stand-alone scoring kernel + top-k + union; for kernel traces of that path)")
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
    ap.add_argument("--no-probe", action="store_true", help="skip the traffic probes")
    return ap.parse_args()


def time_steps(fn, steps, warmup, torch):
    """Wall clock around exactly `steps` calls, after `warmup` untimed ones; seconds per call."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def step_durations(fn, steps, torch):
    """Duration of each of `steps` back-to-back calls (microseconds) from events recorded between
    them on the stream the library launches on; nothing synchronises inside the loop."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    marks[0].record()
    for i in range(steps):
        fn()
        marks[i + 1].record()
    torch.cuda.synchronize()
    return [marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(steps)]


def cold_step_durations(fn, steps, torch, cb):
    """Durations of `steps` calls (microseconds), each after a streaming read of 1 GiB that turns the caches
    over (the 256 MB last-level cache included); the read is outside the timed interval."""
    junk = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    junk.fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for a, b in ev:
        cb.probe_stream_read(junk, sink)
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    out = [a.elapsed_time(b) * 1e3 for a, b in ev]
    del junk
    torch.cuda.empty_cache()
    return out


def kernel_bytes(w, lens, acc):
    """Algorithmic bytes of ONE launch of each bandwidth-bound kernel (all sequences of the batch)."""
    G, K, W = w.n_kv_heads, w.budget, w.window
    return {
        "attn_kernel<full>": sum(acc.full_attn_bytes(G, L) for L in lens),
        "attn_kernel<sparse>": sum(acc.sparse_attn_bytes(G, K, L) for L in lens),
        "attn_kernel<scores only>": sum(acc.score_bytes(G, L, K, W) for L in lens),
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


def _host_view(inp, layer_pos, b):
    """Logical (q, K, V) bf16 bit patterns of sequence b on the host, for the oracle (input marshalling only)."""
    import numpy as np
    import torch

    import oracle
    from paper_2508_07101_amd.workloads import bf16_bits
    lay = inp.layers[layer_pos]
    L = inp.seq_lens_host[b]
    q = bf16_bits(lay.q[b])
    if inp.block_table is None:
        return q, bf16_bits(lay.k[b, :, :L]), bf16_bits(lay.v[b, :, :L])
    n = (L + inp.workload.page_size - 1) // inp.workload.page_size
    bt = inp.block_table[b, :n].cpu().numpy()
    sel = torch.as_tensor(bt, device=lay.k.device, dtype=torch.long)      # this sequence's pages, in logical order
    local = np.arange(n, dtype=np.int32)
    return q, oracle.resolve_paged(bf16_bits(lay.k[sel]), local, L), oracle.resolve_paged(bf16_bits(lay.v[sel]), local, L)


def _set_omp_threads(n):
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def cpu_baseline(inp, w, sched, single_thread_too=False):
    """Oracle wall time for one step on the host cores, split by stage.

    One layer of each kind is timed on sequence 0 (full attention, selection = scores + per-head
    top-k + union + window, sparse attention over the rho just selected).  If that projects to at
    most 20 s the whole step (every layer, every sequence) is run and its measured time reported,
    otherwise the projection is (other sequences scaled by length, other layers by count)."""
    import oracle

    def timed(fn):
        t0 = time.perf_counter()
        r = fn()
        return time.perf_counter() - t0, r

    sel = sched.index(1)
    sp = sched.index(2)
    q, K, V = _host_view(inp, sel, 0)
    q2, K2, V2 = _host_view(inp, sp, 0)
    t_full, _ = timed(lambda: oracle.attention(q, K, V))
    t_sel, rho0 = timed(lambda: oracle.select(q, K, w.budget, w.window, w.topk_per_head))
    t_sparse, _ = timed(lambda: oracle.attention(q2, K2, V2, rho0))
    cores = oracle.num_threads()
    n_full = sum(1 for k in sched if k in (0, 1))
    n_sparse = sum(1 for k in sched if k == 2)
    scale = sum(inp.seq_lens_host) / inp.seq_lens_host[0]          # other sequences, by length
    stage = {"full_attention_s": n_full * t_full * scale, "selection_s": t_sel * scale,
             "sparse_attention_s": n_sparse * t_sparse * w.batch}
    projected = sum(stage.values())
    base = {"unit": "us", "cores": cores, "kind": "oracle",
            "sequence0_one_layer_s": {"full_attention": round(t_full, 4), "selection": round(t_sel, 4),
                                      "sparse_attention": round(t_sparse, 5), "context": inp.seq_lens_host[0]}}

    def single_thread(base):
        """Last, because changing the thread count makes the OpenMP runtime rebuild its pool."""
        if not single_thread_too:
            return base
        _set_omp_threads(1)
        s_full, _ = timed(lambda: oracle.attention(q, K, V))
        s_sel, _ = timed(lambda: oracle.select(q, K, w.budget, w.window, w.topk_per_head))
        s_sparse, _ = timed(lambda: oracle.attention(q2, K2, V2, rho0))
        _set_omp_threads(cores)
        base["single_thread_s"] = {"full_attention": round(s_full, 4), "selection": round(s_sel, 4),
                                   "sparse_attention": round(s_sparse, 5),
                                   "step": round(n_full * s_full + s_sel + n_sparse * s_sparse, 4)}
        return base

    if projected > 20.0:
        base.update(value=round(projected * 1e6, 1), stage_seconds={k: round(v, 4) for k, v in stage.items()},
                    sample=(f"sequence 0 of {w.batch}: one full-attention layer, one selection, one sparse layer; "
                            f"projected to {n_full} full + 1 select + {n_sparse} sparse layers and to all sequences by length"))
        return single_thread(base)
    stage = {"full_attention_s": 0.0, "selection_s": 0.0, "sparse_attention_s": 0.0}
    rho = [None] * w.batch
    for i, kind in enumerate(sched):
        for b in range(w.batch):
            qi, Ki, Vi = _host_view(inp, i, b)                       # device -> host copy, not timed
            if kind == 2:
                dt, _ = timed(lambda: oracle.attention(qi, Ki, Vi, rho[b]))
                stage["sparse_attention_s"] += dt
            else:
                dt, _ = timed(lambda: oracle.attention(qi, Ki, Vi))
                stage["full_attention_s"] += dt
                if kind == 1:
                    d2, rho[b] = timed(lambda: oracle.select(qi, Ki, w.budget, w.window, w.topk_per_head))
                    stage["selection_s"] += d2
    base.update(value=round(sum(stage.values()) * 1e6, 1), stage_seconds={k: round(v, 4) for k, v in stage.items()},
                sample=f"the whole step: all {len(sched)} layers of all {w.batch} sequences, oracle calls only "
                       f"(host copies of the inputs not timed)")
    return single_thread(base)


def traffic_probes(torch, cb):
    """What the memory system gives the access patterns of the attention kernels without their arithmetic
    (4 GiB each, far beyond the 256 MB last-level cache): a plain streaming read (grid-stride, and in the 32 KiB
    tiles per wave the other probes use); 256-byte rows gathered with
    irregular gaps (sparse attention); a streaming read with 1/32 of its volume written back as scattered
    256-byte runs, and with the same volume written in workgroup bursts (the selection layer's pass, which
    stores the scores)."""
    n = 1 << 32
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    src.fill_(1)
    dst = torch.zeros((n >> 5) + (1 << 20), dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    runs = {"stream_read": (lambda: cb.probe_stream_read(src, sink), "probe_stream_read_kernel", n),
            "stream_read_in_tiles": (lambda: cb.probe_traffic(0, src, dst), "probe_traffic_kernel<stream>", n),
            "gathered_rows_read": (lambda: cb.probe_traffic(1, src, dst), "probe_traffic_kernel<gather>", n >> 2),
            "stream_read_with_scattered_writes": (lambda: cb.probe_traffic(2, src, dst), "probe_traffic_kernel<scattered writes>", n),
            "stream_read_with_burst_writes": (lambda: cb.probe_traffic(3, src, dst), "probe_traffic_kernel<burst writes>", n)}
    out = {}
    reps = 10
    for label, (fn, kname, nbytes) in runs.items():
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        cb.profile_reset()
        cb.profile_enable(True)
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        p = cb.profile_read()[kname]
        cb.profile_enable(False)
        cb.profile_reset()
        us = p["total_ms"] * 1e3 / p["calls"]
        gbs = nbytes / (us * 1e-6) / 1e9
        out[label] = {"kernel": kname, "bytes_read": nbytes, "avg_us": round(us, 2), "read_GBs": round(gbs, 1),
                      "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "launches": reps}
    del src, dst
    torch.cuda.empty_cache()
    return out


def measure(name, args, torch, acc, cb, wl, StepRunner):
    """Everything reported for one workload."""
    w = wl.WORKLOADS[name]
    if args.head_overlap is not None:
        w = wl.scaled(w, lowrank=8, lowrank_scale=args.head_overlap, n_planted=0)
    inp = wl.make_inputs(w, "cuda:0")
    sched = list(w.schedule)
    lens = inp.seq_lens_host
    r = StepRunner(inp, sched)
    torch.cuda.synchronize()

    run_step = r.run
    if args.entry == "select":
        sel_layer = sched.index(1)

        def run_step():
            r.select(sel_layer)
    steps, warmup = args.steps, args.warmup
    if w.grow_room > 0:
        if args.graph or 2 * steps + warmup > w.grow_room:
            raise SystemExit(f"workload {w.name}: at most {w.grow_room} steps (warm-up and both timing passes "
                             f"included), and no --graph")

        def run_step():                           # one decode step, then the sequences are one token longer
            r.run()
            r.grow(1)
    if args.graph:
        r.run()                                   # the first call on a device does the library's set-up
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            r.run()
        run_step = graph.replay
    step_s = time_steps(run_step, steps, warmup, torch)
    durs = step_durations(run_step, steps, torch)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    full_s = None
    if not args.no_full_baseline and w.grow_room == 0:
        rf = StepRunner(inp, [0] * len(sched))
        full_s = time_steps(rf.run, max(3, steps // 4), 1, torch)
        del rf

    kernels, rooflines = {}, []
    if not args.no_kernel_timing and w.grow_room == 0:
        cb.profile_reset()
        cb.profile_enable(True)
        for _ in range(steps):
            run_step()
        torch.cuda.synchronize()
        prof = cb.profile_read()
        cb.profile_enable(False)
        kb = kernel_bytes(w, lens, acc)
        tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.json")
        counted = json.load(open(tpath)).get("hbm_bytes_per_launch", {}) if os.path.exists(tpath) else {}
        # A selection layer on the filtered fast path launches the scores-only pass and topk_kernel only as the second
        # chance of heads whose threshold failed; with none flagged they exit at once and move no bytes.
        fast_path = args.entry == "step" and prof.get("sample_threshold_kernel", {}).get("calls", 0) > 0
        for kname, p in prof.items():
            if p["calls"] == 0:
                continue
            avg_us = p["total_ms"] * 1e3 / p["calls"]
            k = {"launches_per_step": p["calls"] // steps, "avg_us": round(avg_us, 3),
                 "us_per_step": round(p["total_ms"] * 1e3 / steps, 3)}
            if fast_path and kname in ("attn_kernel<scores only>", "topk_kernel"):
                k["role"] = "second chance of the filtered selection (exits at once when no head is flagged)"
            elif kname in kb and kb[kname] > 0:
                k["bytes_per_launch"] = kb[kname]
                k["achieved_GBs"] = round(kb[kname] / (avg_us * 1e-6) / 1e9, 1)
                k["frac_of_hbm_peak"] = round(k["achieved_GBs"] / HBM_PEAK_GBS, 4)
            kernels[kname] = k
        for kname in BANDWIDTH_KERNELS:
            if kname in kernels and "achieved_GBs" in kernels[kname]:
                k = kernels[kname]
                # traffic: HBM bytes per launch from rocprofv3 counters, where a summary of them is committed
                rooflines.append({"kernel": kname, "bound": "hbm", "achieved": k["achieved_GBs"], "peak": HBM_PEAK_GBS,
                                  "unit": "GB/s", "frac": k["frac_of_hbm_peak"], "traffic": counted.get(kname),
                                  "bytes_per_launch": k["bytes_per_launch"], "avg_us": k["avg_us"],
                                  "us_per_step": k["us_per_step"]})

    sb = acc.step_bytes(sched, lens, w.n_kv_heads, w.budget, w.window)
    # A step over less than a few last-level caches' worth of KV finds part of it cached from the step before
    # (c1, c4: one layer, repeated): those figures are warm.  The cold figure beside them has the caches turned
    # over before every step.
    kv_bytes = int(sum(2 * w.n_kv_heads * L * w.head_dim * 2 for L in lens) * (1 if w.same_layer_sparse else w.n_layers))
    cold = None
    if kv_bytes < (1 << 30) and w.grow_room == 0 and not args.graph:
        cd = cold_step_durations(run_step, steps, torch, cb)
        cold = {"median": round(statistics.median(cd), 2), "min": round(min(cd), 2), "steps": steps,
                "how": "1 GiB streaming read before every step, outside the timed interval"}
    rec = {
        "us_per_step": {"mean": round(step_s * 1e6, 2), "median": round(statistics.median(durs), 2),
                        "min": round(min(durs), 2), "steps": steps, "warmup": warmup},
        "config": {"workload": f"{w.name}: {w.n_layers} layers, batch {w.batch}, {w.n_q_heads}q/{w.n_kv_heads}kv heads, "
                               f"d {w.head_dim}, L {min(lens)}..{max(lens)}, budget {w.budget}, window {w.window}, "
                               f"top-k/head {w.k_eff}, {'paged' if w.paged else 'contiguous'} KV",
                   "schedule": "".join("FSs"[k] for k in sched), "launch": "hip_graph" if args.graph else "stream",
                   "timed_call": "cusa_decode_step" if args.entry == "step" else "cusa_select on the selection layer",
                   "sinks": w.n_sink, "lengths": "grow by one token per step" if w.grow_room > 0 else "fixed",
                   "kv_cache_bytes": int(sum(2 * w.n_kv_heads * L * w.head_dim * 2 for L in lens) *
                                         (1 if w.same_layer_sparse else w.n_layers)),
                   **({"head_overlap": args.head_overlap} if args.head_overlap is not None else {})},
        "cache": "warm (the step's KV fits the last-level cache in part; see cold_us_per_step)" if cold else "cold",
        **({"cold_us_per_step": cold} if cold else {}),
        "step_algorithmic_bytes": sb["total"],
        "step_achieved_GBs": round(sb["total"] / step_s / 1e9, 1),
        "rooflines": rooflines,
        "kernels": kernels,
    }
    if args.entry == "step" and 1 in sched and r.filtered_select():
        # the selection layer kept only the candidates above sampled thresholds; heads whose threshold failed
        # were scored and ranked again the ordinary way (the result is the same either way)
        run_step()
        torch.cuda.synchronize()
        rec["filtered_selection"] = {"second_chance_heads": r.second_chance_heads(), "heads": w.batch * w.n_q_heads}
    if full_s is not None and args.entry == "step":
        rec["full_attention_all_layers_us"] = round(full_s * 1e6, 2)
        rec["speedup_vs_full_attention"] = round(full_s / step_s, 3)
    if not args.no_per_head and 2 in sched and w.grow_room == 0 and args.entry == "step":
        rec["per_head_comparison"] = per_head_comparison(r, w, sched, lens, max(3, steps // 2), torch, cb, acc)
    if args.rank_study and 2 in sched:
        rec["rank_study"] = rank_study(inp, w, sched, torch, StepRunner)
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(inp, w, sched, single_thread_too=(w.name == "c1"))
    del r, inp
    torch.cuda.empty_cache()
    return rec


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

    names = [n for n in args.workloads.split(",") if n]
    for n in names:
        if n not in wl.WORKLOADS:
            raise SystemExit(f"unknown workload {n}: choose from {sorted(wl.WORKLOADS)}")
    t_start = time.perf_counter()
    probe = None if args.no_probe else traffic_probes(torch, cb)
    configs = {}
    for n in names:
        t0 = time.perf_counter()
        configs[n] = measure(n, args, torch, acc, cb, wl, StepRunner)
        configs[n]["bench_seconds"] = round(time.perf_counter() - t0, 1)
        print(f"[bench] {n}: {configs[n]['us_per_step']['mean']} us/step ({configs[n]['bench_seconds']} s)",
              file=sys.stderr, flush=True)
    head = configs[names[-1]]
    # the headline roofline: the bandwidth kernel that takes most of the headline workload's step
    roofline = max(head["rooflines"], key=lambda k: k["us_per_step"]) if head["rooflines"] else None
    out = {
        "metric": "us_per_decode_step_select_plus_sparse_attn",
        "value": head["us_per_step"]["mean"], "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["us_per_step"]["mean"] / 1e3, 5), "higher_is_better": False, "scaling": "none (one GPU)",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": head["config"],
        "step_algorithmic_bytes": head["step_algorithmic_bytes"],
        "step_achieved_GBs": head["step_achieved_GBs"],
        "roofline": roofline,
        "cpu_baseline": head.get("cpu_baseline"),
        "traffic_probes": probe,
        "configs": configs,
        "bench_seconds": round(time.perf_counter() - t_start, 1),
    }
    if "speedup_vs_full_attention" in head:
        out["full_attention_all_layers_us"] = head["full_attention_all_layers_us"]
        out["speedup_vs_full_attention"] = head["speedup_vs_full_attention"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
