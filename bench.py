#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is already resident in
HBM: hs_draft_entropy_topk on every expanded draft row, hs_tree_prune on the candidate tree,
hs_tree_attention on the kept rows (for the single-sequence workloads: all decoder layers of the
model the layer is shaped after, each with its own Q and K/V cache, in one batched launch) and
hs_verify_accept on the kept rows' target logits.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--layers N] [--accept greedy]
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published


def cpu_baseline(w, step, layers, seed, budget_s=9.0):
    """The CPU checker, as it stands, on a bounded sample of the same step, each stage scaled to the full step:
    once with the host's BLAS threads as they are (about `budget_s` seconds of CPU work: the sample is
    repeated until that much time has passed) and once more limited to one thread."""
    import numpy as np
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import draft_entropy_topk, tree_prune, tree_attention, verify_accept

    h = step.host
    rows_total = int(step.t["draft_rows"].shape[0])
    n_rows = min(64, rows_total)
    x = step.t["draft_rows"][:n_rows].cpu().numpy()
    prune_in = [step.t[k].cpu().numpy() for k in ("cand_parent", "cand_logc", "cand_offsets", "d_max", "theta", "max_nodes")]
    no, po = h["attn_node_offsets"].numpy(), h["attn_prefix_offsets"].numpy()

    def np_store(t):
        import torch
        return t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()
    es = 4 if w.dtype == "f32" else 2
    # attention: leading batch entries (layers / sequences) up to about 64 MB of K/V, scaled by bytes
    n_ent, bytes_sample = 0, 0
    while n_ent < len(no) - 1 and (n_ent == 0 or bytes_sample < 64e6):
        M, L = int(no[n_ent + 1] - no[n_ent]), int(po[n_ent + 1] - po[n_ent])
        bytes_sample += (2 * (L + M) * w.Hkv * w.D + 2 * M * w.Hq * w.D) * es
        n_ent += 1
    n1, p1 = int(no[n_ent]), int(po[n_ent])
    q, kp, vp = np_store(step.t["q"][:n1]), np_store(step.t["k_prefix"][:p1]), np_store(step.t["v_prefix"][:p1])
    kt, vt = np_store(step.t["k_tree"][:n1]), np_store(step.t["v_tree"][:n1])
    par = step.t["attn_parent"][:n1].cpu().numpy()
    # accept walk: the checker's verify_accept on the step's own inputs; leading sequences of the
    # batch up to 256 rows of logits, scaled by rows
    oo = h["out_offsets"]
    n_seq = 1
    while n_seq < len(oo) - 1 and int(oo[n_seq + 1]) <= 256:
        n_seq += 1
    n4 = int(oo[n_seq])
    tl = step.t["target_logits"][:n4].cpu().numpy()
    tok = step.t["token"][:n4].cpu().numpy()
    par4 = step.t["s2_out"]["out_parent"][:n4].cpu().numpy()

    def sample(budget):
        t1 = t2 = t3 = t4 = 0.0
        reps = 0
        start = time.perf_counter()
        while reps == 0 or time.perf_counter() - start < budget:
            t0 = time.perf_counter()
            draft_entropy_topk(x, w.topk, w.temperature)
            t1 += time.perf_counter() - t0
            t0 = time.perf_counter()
            tree_prune(*prune_in)
            t2 += time.perf_counter() - t0
            t0 = time.perf_counter()
            tree_attention(q, kp, vp, kt, vt, par, no[:n_ent + 1], po[:n_ent + 1], h["scale"])
            t3 += time.perf_counter() - t0
            t0 = time.perf_counter()
            verify_accept(tl, None, tok, par4, oo[:n_seq + 1], 0, w.temperature, None, h["max_depth"])
            t4 += time.perf_counter() - t0
            reps += 1
        spent = time.perf_counter() - start
        st = {"entropy_topk": t1 / reps * rows_total / n_rows, "prune": t2 / reps,
              "attention": t3 / reps * step.bytes_stage3() / bytes_sample, "accept": t4 / reps * h["NNp"] / n4}
        return st, reps, spent

    stages, reps, spent = sample(budget_s)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    with threadpool_limits(limits=1):
        stages1, reps1, spent1 = sample(budget_s)
    total, total1 = sum(stages.values()), sum(stages1.values())
    return {"value": h["kept_draft_nodes"] / total, "unit": "tree-tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d repetitions (%.1f s of CPU work) of: stage1 on %d of %d rows, stage2 whole, stage3 on %d of %d "
                      "batch entries (scaled by bytes), stage4 = the checker's greedy accept walk on %d of %d rows "
                      "(%d of %d sequences); each scaled to the full step; then %d repetitions (%.1f s) limited to "
                      "one thread" % (reps, spent, n_rows, rows_total, n_ent, len(no) - 1, n4, h["NNp"], n_seq,
                                      len(oo) - 1, reps1, spent1),
            "seconds_per_step": total, "stage_seconds": stages,
            "one_thread": {"value": h["kept_draft_nodes"] / total1, "cores": 1, "seconds_per_step": total1,
                           "stage_seconds": stages1}}


def adaptive_main(args, w, layers):
    """K adaptive steps whose entropy bin changes from step to step: the drafting graph, one host read of
    the bin, the graph cached for that bin (Section 4.3, Dynamic Computational Adaptation).  The draft
    rows of a step are the workload's at one of four draft temperatures (exact power-of-two scalings of
    the same rows), the synthetic bin boundaries are placed so that the four land in four different
    bins; swapping the rows stands in for the draft model and is not timed."""
    import numpy as np
    import torch
    from paper_2505_13254_amd import harness
    edges = [e * args.edge_scale for e in (1.0, 3.0, 8.0, 11.0, 12.0, 13.0, 14.0)]
    temps = [1.0, 0.125, 0.5, 0.25]
    st = harness.build_adaptive(w, args.seed, layers=layers, edges=edges)
    st.capture()                      # the drafting graph and one graph per distinct (d', N')
    per_bin = {}
    results = {}
    for k in range(args.warmup + args.steps):
        T = temps[k % len(temps)]
        st.set_temperature(T)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        b = st.step_graph()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) * 1e3
        if k >= args.warmup:
            per_bin.setdefault(b, []).append(dt)
            results[b] = st.result(b)
    all_ms = [x for v in per_bin.values() for x in v]
    tokens = float(np.mean([results[b]["n_prime"] for b, v in per_bin.items() for _ in v]))
    # the same bins with eager launches, for the value of the graphs
    eager = {}
    for T in temps:
        st.set_temperature(T)
        for rep in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            b = st.step_eager()
            torch.cuda.synchronize()
            eager[b] = (time.perf_counter() - t0) * 1e3
    ms = float(np.mean(all_ms))
    print(json.dumps({
        "metric": "verified tree-tokens/sec per step + tree-attn HBM GB/s (% of peak), 1 GPU",
        "value": tokens / (ms * 1e-3), "unit": "tree-tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "configs[%d] %s, adaptive step on the device (expansion level by level, complexity "
                               "decision, extended drafting, one cached HIP graph per entropy bin), the bin changing "
                               "from step to step" % (w.wid - 1, w.name),
                   "attention_layers_per_step": layers, "d_base": st.d_base, "alpha": st.alpha,
                   "n_default": st.n_default, "bin_edges": st.edges, "gamma": st.gamma, "draft_temperatures": temps,
                   "graphs_cached": len({id(g) for g in st.graphs.values()})},
        "per_bin": {str(b): {"steps": len(v), "ms_per_step_median": float(np.median(v)), "ms_per_step_eager": eager.get(b),
                             **results[b]} for b, v in sorted(per_bin.items())}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, help="1..5, the configs of BASELINE.json in order")
    ap.add_argument("--layers", type=int, default=0, help="attention layers per step (0 = the model's)")
    ap.add_argument("--accept", default="greedy", choices=["greedy", "stochastic", "pointmass"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--theta", type=float, default=None,
                    help="prune threshold on the cumulative log-probability (default: the workload's first; "
                         "-inf keeps every node the depth cap and the node budget allow)")
    ap.add_argument("--pause-ms", type=float, default=0.0,
                    help="--only attention: host pause after every launch (the chip's clocks recover between launches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--head-dim", type=int, default=0,
                    help="--only attention: the workload's attention shape with this head dimension (64: the "
                         "matrix-core kernel's paired-head path); not a bench line")
    ap.add_argument("--only", default="", choices=["", "attention"],
                    help="attention: nothing but W + K attention launches of the workload (for profiler passes); "
                         "prints a short line, not the bench line")
    ap.add_argument("--adaptive", action="store_true",
                    help="the device-driven adaptive step (level-by-level expansion, complexity decision, extended "
                         "drafting, per-bin HIP graphs) instead of the four-call step; not the headline line")
    ap.add_argument("--edge-scale", type=float, default=1.0, help="--adaptive: scales the synthetic bin boundaries")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU hot path (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2505_13254_amd as hs
    from paper_2505_13254_amd import harness
    from synth import workloads as W

    if not os.path.exists(hs.LIB_PATH):
        from paper_2505_13254_amd.build import build
        build(verbose=False)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = W.WORKLOADS[args.workload]
    if args.head_dim:
        assert args.only == "attention", "--head-dim goes with --only attention"
        w = W.small(w, D=args.head_dim)
    layers = args.layers or (w.layers if w.B == 1 else 1)
    mode = {"greedy": 0, "stochastic": 1, "pointmass": 2}[args.accept]
    if args.adaptive:
        return adaptive_main(args, w, layers)
    step = harness.build_step(w, args.seed, layers=layers, accept_mode=mode, theta=args.theta)
    torch.cuda.synchronize()
    if args.only == "attention":
        # W + K attention launches (each carrying events on its dispatch) with a 2 ms pause between them,
        # and one 1 GiB device copy, whose known size calibrates the profiler's byte counters
        n = args.warmup + args.steps
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]
        for pair in ev:
            for e in pair:
                e.record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for a_, b_ in ev:
            hs.hs_time_next_attention(a_, b_)
            step.stage3()
            if args.pause_ms > 0:
                torch.cuda.synchronize()
                time.sleep(args.pause_ms * 1e-3)
        torch.cuda.synchronize()
        call_ms = (time.perf_counter() - t0) * 1e3 / n
        big = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(big)
        dst.copy_(big)
        torch.cuda.synchronize()
        ts = np.array([a_.elapsed_time(b_) for a_, b_ in ev][args.warmup:])
        print(json.dumps({"only": "attention", "workload": w.wid, "head_dim": w.D, "layers": layers, "launches": n,
                          "kernel": {0: "none", 1: "matrix cores", 2: "vector ALUs"}[hs.hs_tree_attention_last_kernel()],
                          "verified_rows": step.host["NNp"],
                          "pause_ms_between_launches": args.pause_ms,
                          "kernel_ms_median": float(np.median(ts)), "kernel_ms_mean": float(ts.mean()),
                          "kernel_ms_min": float(ts.min()), "call_to_call_ms": call_ms,
                          "algorithmic_bytes_per_launch": step.bytes_stage3(),
                          "algorithmic_flops_per_launch": step.flops_stage3(),
                          "note": "kernel_ms is the attention kernel alone (a combine launch that follows split keys "
                                  "is not in it)"}))
        return
    n_sets = step.rotate_logits()     # consecutive steps read different copies: the scans stream from HBM

    for _ in range(args.warmup):
        step.run()
    torch.cuda.synchronize()
    K = args.steps
    # Timed region: K steps and nothing else on the stream.
    t0 = time.perf_counter()
    for k in range(K):
        step.stage1()
        step.stage2()
        step.stage3()
        step.stage4()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    # The same K steps once more, each attention launch carrying a pair of events on its own dispatch
    # (hs_time_next_attention: stamped when that kernel begins and ends on the stream it is launched
    # on): the kernel's duration for the roofline.  Not inside the region above, because a dispatch
    # that carries events costs the stream about 6 us more than one that does not.
    KE = max(K, 50)             # at least 50 launches, whatever --steps says
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(KE)]
    for pair in ev:
        for e in pair:
            e.record()          # torch creates the HIP event at the first record
    torch.cuda.synchronize()
    te0 = time.perf_counter()
    for k in range(KE):
        step.stage1()
        step.stage2()
        hs.hs_time_next_attention(ev[k][0], ev[k][1])
        step.stage3()
        step.stage4()
    torch.cuda.synchronize()
    ms_per_step_with_events = (time.perf_counter() - te0) * 1e3 / KE
    attn = [a.elapsed_time(b) for a, b in ev]

    # Per-stage breakdown: a third pass of K steps with an event recorded at every stage boundary
    # (recorded events cost about 5 us a pair, which is why they stay out of the timed region above;
    # gaps[2] is the attention call bracketed that way, combine kernel included when there is one).
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(KE)]
    for k in range(KE):
        ev2[k][0].record()
        step.stage1()
        ev2[k][1].record()
        step.stage2()
        ev2[k][2].record()
        step.stage3()
        ev2[k][3].record()
        step.stage4()
        ev2[k][4].record()
    torch.cuda.synchronize()
    gaps = [[ev2[k][i].elapsed_time(ev2[k][i + 1]) for k in range(KE)] for i in range(4)]
    stage_ms = [float(np.mean(gaps[0])), float(np.mean(gaps[1])), float(np.mean(attn)), float(np.mean(gaps[3]))]
    stage_med = [float(np.median(gaps[0])), float(np.median(gaps[1])), float(np.median(attn)), float(np.median(gaps[3]))]
    attn_bracketed_ms = float(np.mean(gaps[2]))

    # what a pair of events costs by itself on the busy stream (it is inside every figure above)
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2 * 20)]
    step.run()
    for i in range(20):
        pe[2 * i].record()
        pe[2 * i + 1].record()
        step.stage2()
    torch.cuda.synchronize()
    event_pair_ms = float(np.median([pe[2 * i].elapsed_time(pe[2 * i + 1]) for i in range(20)]))

    # streaming-copy ceiling of this device, for context
    big = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")   # 1 GiB
    dst = torch.empty_like(big)
    for _ in range(2):
        dst.copy_(big)
    torch.cuda.synchronize()
    c0 = torch.cuda.Event(enable_timing=True)
    c1 = torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(big)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * big.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9

    # One layer of the same workload by itself (what a single hs_tree_attention call of a model's
    # layer loop sees): warm (same buffers, resident in the last-level cache when they fit) and cold
    # (a 1 GiB copy streams through the caches before every call).
    single = None
    if layers > 1:
        one = harness.build_step(w, args.seed, layers=1, accept_mode=0, theta=args.theta)
        for _ in range(5):
            one.stage3()
        torch.cuda.synchronize()
        ev3 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(30)]
        for a, b in ev3[:20]:
            a.record()
            one.stage3()
            b.record()
        torch.cuda.synchronize()
        warm = float(np.median([a.elapsed_time(b) for a, b in ev3[:20]]))
        for a, b in ev3[20:]:
            dst.copy_(big)
            a.record()
            one.stage3()
            b.record()
        torch.cuda.synchronize()
        cold = float(np.median([a.elapsed_time(b) for a, b in ev3[20:]]))
        b1 = one.bytes_stage3()
        single = {"algorithmic_bytes": b1, "warm_ms": warm, "cold_ms": cold,
                  "warm_gbps": b1 / (warm * 1e-3) / 1e9, "cold_gbps": b1 / (cold * 1e-3) / 1e9,
                  "note": "event pairs cost about %.0f us each" % (event_pair_ms * 1e3)}
        del one
    del big, dst

    # The same step under the sampling rule (ratio rule, seeded uniforms): reported beside the headline
    # line, which keeps the accept rule asked for.
    sampling = None
    if mode == 0:
        st2 = harness.build_step(w, args.seed, layers=layers, accept_mode=1, theta=args.theta)
        for _ in range(max(args.warmup, 3)):
            st2.run()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(K):
            st2.run()
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t2) * 1e3 / K
        acc2 = st2.t["s4_out"]
        sampling = {"accept": "stochastic", "ms_per_step": ms2,
                    "tree_tokens_per_s": st2.host["kept_draft_nodes"] / (ms2 * 1e-3),
                    "accept_len": [int(x) for x in acc2["accept_len"].cpu().numpy()][:16]}
        del st2

    h = step.host
    tokens = h["kept_draft_nodes"]
    bytes3 = step.bytes_stage3()
    # A launch with split keys is followed by the combine kernel, which the events attached to the attention
    # kernel do not cover: the roofline then takes the whole call as bracketed by recorded events (less
    # what an empty pair of those costs), so that the merge of the splits is paid for in the figure.
    call_ms = attn_bracketed_ms - event_pair_ms
    with_combine = call_ms > 1.05 * stage_ms[2]
    launch_ms = call_ms if with_combine else stage_ms[2]
    achieved = bytes3 / (launch_ms * 1e-3) / 1e9
    flops3 = step.flops_stage3()
    # the attention launch is bound by the matrix cores when its arithmetic intensity lies above the
    # ridge of the two published peaks (workload 4: 776 rows share every K/V byte)
    mfma_bound = w.dtype == "bf16" and flops3 / bytes3 > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_tree_attention_w%d.json" % w.wid)
    if os.path.exists(tpath) and args.theta is None and not args.layers:   # (measured on the configured launch only)
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
    out = {
        "metric": "verified tree-tokens/sec per step + tree-attn HBM GB/s (% of peak), 1 GPU",
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tree-tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "configs[%d] %s" % (w.wid - 1, w.name), "sequences": w.B, "heads": "%d/%d" % (w.Hq, w.Hkv),
                   "head_dim": w.D, "vocab": w.V, "prefix_tokens": int(h["attn_prefix_offsets"][1]) if w.B == 1 else
                   [int(x) for x in np.diff(h["attn_prefix_offsets"].numpy())],
                   "attention_layers_per_step": layers, "candidate_nodes": h["cand_nodes"],
                   "verified_rows": h["NNp"], "verified_draft_nodes": tokens,
                   "draft_rows_quantified": int(step.t["draft_rows"].shape[0]), "accept": args.accept,
                   "prune_threshold": float(step.t["theta"][0])},
        "stage_ms": {"entropy_topk": stage_med[0], "prune": stage_med[1], "attention": stage_med[2], "accept": stage_med[3],
                     "statistic": "median of %d steps (attention: the kernel between the events attached to its "
                                  "dispatch; the other stages between recorded events, which add about one "
                                  "empty_event_pair each)" % KE,
                     "attention_call_bracketed_by_events": attn_bracketed_ms,
                     "empty_event_pair": event_pair_ms, "step_with_events_on_the_attention_launch": ms_per_step_with_events},
        "stage_ms_mean": {"entropy_topk": stage_ms[0], "prune": stage_ms[1], "attention": stage_ms[2],
                          "accept": stage_ms[3]},
        "stage_gbps": {"entropy_topk": step.bytes_stage1() / (stage_med[0] * 1e-3) / 1e9,
                       "attention": achieved, "accept": step.bytes_stage4() / (stage_med[3] * 1e-3) / 1e9,
                       "logits_copies_rotated": n_sets,
                       "note": "consecutive steps read different copies of the logits (%d copies, %.0f MB in all), so the "
                               "scans' rates are HBM rates, not last-level-cache rates" %
                               (n_sets, n_sets * (step.bytes_stage1() + step.bytes_stage4()) / 1e6)},
        "tree_attn_hbm_gbps": achieved, "tree_attn_pct_of_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "copy_ceiling_gbps": copy_gbps,
        "tree_attn_single_layer": single,
        "step_with_sampling_accept": sampling,
        "roofline": {"kernel": "hs_tree_attention", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": bytes3, "algorithmic_flops_per_launch": flops3,
                     "launch_ms": launch_ms, "launch_ms_median": stage_med[2], "launches_timed": len(attn),
                     "launch_covers": "attention kernel + combine kernel (recorded events around the call, less an empty pair)"
                                      if with_combine else "attention kernel (events attached to its dispatch)",
                     "attention_kernel_alone_ms": stage_ms[2]},
    }
    if mfma_bound:
        tf = flops3 / (launch_ms * 1e-3) / 1e12
        out["roofline"].update({"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "hbm_gbps": achieved})
    acc = step.t["s4_out"]
    out["result"] = {"accept_len": [int(x) for x in acc["accept_len"].cpu().numpy()][:16],
                     "bonus_token": [int(x) for x in acc["bonus_token"].cpu().numpy()][:16]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, step, layers, args.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
