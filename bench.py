#!/usr/bin/env python3
"""Benchmark of the verification hot path on one MI355X.

One step = one full verification step of a Llama-3.1-8B-shaped target model at
a 16384-token prefix: 32 layers of Hybrid Tree Attention (prefix pass + tree
pass + merge; each layer has its own bf16 K/V cache, 2.147 GB in total, so
every layer streams cold from HBM), then chunk scores from the last layer,
top-32-of-512 chunk selection and the draft-KV gather.  Inputs are synthetic
and resident in HBM before the timed region.  The whole step is captured once
in a HIP graph and replayed, so the host launch path is not what is timed.

Prints one JSON line.  `roofline` prices the dominant kernel (the prefix pass)
by its algorithmic bytes (one layer's K+V prefix) over its average launch
duration, measured with HIP events around a graph that holds only the 32
prefix-pass launches.  `cpu_baseline` times the fp64 oracle on the host cores
for a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "prefix_rows_kernel_config4_hbm_traffic.txt")


def measured_traffic():
    """HBM bytes per launch of the dominant kernel at the default workload, from the summary of the latest
    FETCH_SIZE / WRITE_SIZE counter passes (written by `python -m paper_2505_20776_amd.profile_summary traffic`,
    which records the commit it was measured at).  None when there is no summary."""
    try:
        fields = dict(line.strip().split("=", 1) for line in open(TRAFFIC_FILE) if "=" in line and not line.startswith("#"))
        return {"bytes": float(fields["traffic_bytes_per_launch"]), "commit": fields.get("commit", "?"),
                "fetch_bytes": float(fields["fetch_bytes_per_launch"]), "write_bytes": float(fields["write_bytes_per_launch"])}
    except (OSError, KeyError, ValueError):
        return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 300 steps are 0.3 s of timed work: the first steps behind the synchronisation that opens the timed region run
    # below the clock the power management settles on, and with 30 steps they are 2 % of the mean
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default 300; 10 for --workload prefill)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", choices=["2", "3", "4", "5wide", "5chain", "draft", "draft68m"], default="4",
                    help="numbered workload: 4 (default) = 32 layers at a 16K prefix, the headline metric; 2 / 3 / 5 = "
                         "the single-layer shapes (2K, 8K, 32K-37 with a 128-node wide tree or a 16-node chain), run "
                         "over enough distinct K/V copies (>= 768 MB) that every launch streams cold (a second figure, "
                         "labelled hot, comes from one copy that stays in the caches); draft = the draft model's side "
                         "(Sec. 3.2.1): one EAGLE-style layer of the same shape over a compacted working cache of "
                         "2048 tokens; draft68m = a Vicuna-68M-shaped draft layer (12 heads of 64, no grouping) over "
                         "a working cache of 1024 tokens")
    ap.add_argument("--valu-prefix", action="store_true",
                    help="prefix pass on the vector ALUs (SPECEXT_FLAG_VALU_PREFIX) instead of the matrix cores")
    ap.add_argument("--kv-heads", type=int, default=8,
                    help="KV heads (8 = Llama-3.1-8B's grouped queries; 32 = multi-head attention as in the "
                         "Vicuna-7B / LongChat-7B targets of the paper)")
    ap.add_argument("--layers", type=int, default=0, help="distinct K/V copies per step (0 = the config's own)")
    ap.add_argument("--prefix", type=int, default=0, help="prefix length (0 = the config's own)")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--last-layer", choices=["fused", "materialized"], default="fused",
                    help="how the last layer (the one the chunk scores come from) is computed: fused (default) or as "
                         "standard attention with the probability matrix written out, as Sec. 3.2.1 words it")
    ap.add_argument("--workload", choices=["verify", "prefill"], default="verify",
                    help="verify (default): the verification step the headline metric is quoted on; prefill: causal "
                         "self-attention of a --prefix token prompt on all layers (Sec. 3.1), its own JSON line")
    ap.add_argument("--merge", choices=["two-launch", "fused"], default="two-launch",
                    help="tree pass + merge as their own launch (default) or as the tail of the prefix launch "
                         "(SPECEXT_FLAG_FUSED_MERGE)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hold", type=float, default=0.0,
                    help="instead of the benchmark: keep the GPU busy with --hold-what for this many seconds (so that "
                         "power and clocks can be sampled from outside, e.g. with rocm-smi) and print the rate it ran at")
    ap.add_argument("--hold-what", choices=["stream", "mfma", "prefix", "step"], default="step",
                    help="stream: the HBM read calibration kernel; mfma: the matrix-core calibration kernel; prefix: "
                         "the prefix-pass kernel alone over all layers; step: whole verification steps")
    ap.add_argument("--issue-probe", action="store_true",
                    help="instead of the benchmark: time the library's probe of how matrix and vector instructions share "
                         "a SIMD (specext_calib_issue_mix) and print one JSON line")
    ap.add_argument("--no-calibrate", action="store_true",
                    help="skip the two calibration kernels (pure HBM read stream, pure bf16 matrix-core loop) whose rates "
                         "are reported as measured_* next to the published peaks")
    ap.add_argument("--operands", choices=["recipe", "zeros", "unit"], default="recipe",
                    help="values of Q, K and V: recipe (default; N(0, 1/d), the workload the metric is quoted on), "
                         "zeros or N(0, 1) - the same instruction stream on other bits, to show how much of the time is "
                         "the power management's answer to the data; such a line is labelled and is not the metric")
    ap.add_argument("--cpu-layers", type=int, default=32, help="layers the oracle is timed on (32 = the whole step, about 10 s)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.steps <= 0:
        args.steps = 10 if args.workload == "prefill" else 300
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "prefill":
        return bench_prefill(args)

    import numpy as np
    import torch

    import paper_2505_20776_amd as sx
    from paper_2505_20776_amd import harness
    from workloads import config_tree

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    Hq, Hkv, d = (12, 12, 64) if args.config == "draft68m" else (32, args.kv_heads, 128)
    L, B, topk, parent_np = {"2": (2048, 32, 32, config_tree(2)), "3": (8192, 32, 32, config_tree(3)),
                             "4": (16384, 32, 32, config_tree(4)), "5wide": (32768 - 37, 64, 16, config_tree(5, "wide")),
                             "5chain": (32768 - 37, 64, 16, config_tree(5, "chain")),
                             "draft": (2048, 32, 32, config_tree(2)), "draft68m": (1024, 32, 32, config_tree(2))}[args.config]
    L = args.prefix or L
    T = len(parent_np)
    layer_bytes = 2 * Hkv * L * d * 2
    single = args.config != "4"
    # Cold means cold: the distinct K/V copies of a step add up to three times the 256 MB last-level cache (with
    # little more than one cache size, launches that follow one another directly still found part of their K/V there)
    cold_layers = -(-768_000_000 // layer_bytes)
    n_layers = args.layers or (max(32, cold_layers) if args.config == "4" else cold_layers)
    n_chunks = (L + B - 1) // B

    gen = torch.Generator(device=dev)
    gen.manual_seed(4000)
    std = 1.0 / np.sqrt(d)

    def randn(*shape):
        if args.operands == "zeros":
            return torch.zeros(*shape, device=dev, dtype=torch.bfloat16)
        scale = 1.0 if args.operands == "unit" else std
        return (torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32) * scale).to(torch.bfloat16)

    q = [randn(T, Hq, d) for _ in range(n_layers)]
    kp = [randn(Hkv, L, d) for _ in range(n_layers)]
    vp = [randn(Hkv, L, d) for _ in range(n_layers)]
    kt = [randn(Hkv, T, d) for _ in range(n_layers)]
    vt = [randn(Hkv, T, d) for _ in range(n_layers)]
    draft_k = randn(1, Hkv, L, d)
    draft_v = randn(1, Hkv, L, d)
    parent = torch.from_numpy(parent_np).to(dev)

    merge_flag = (sx.SPECEXT_FLAG_FUSED_MERGE if args.merge == "fused" else 0) | \
                 (sx.SPECEXT_FLAG_VALU_PREFIX if args.valu_prefix else 0)
    plain = harness.make_buffers(dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, prefix_len=L, n_tree=T,
                                 num_splits=args.num_splits, flags=merge_flag)
    last = harness.make_buffers(dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, prefix_len=L, n_tree=T,
                                chunk_size=B, want_scores=True, num_splits=args.num_splits, flags=merge_flag)
    only = harness.make_buffers(dtype="bf16", n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, prefix_len=L, n_tree=T,
                                num_splits=args.num_splits, flags=sx.SPECEXT_FLAG_PREFIX_ONLY |
                                (sx.SPECEXT_FLAG_VALU_PREFIX if args.valu_prefix else 0))
    outs = [torch.empty((T, Hq, d), dtype=torch.bfloat16, device=dev) for _ in range(n_layers)]
    scores = torch.empty((n_chunks,), dtype=torch.float32, device=dev)
    idx = torch.empty((topk,), dtype=torch.int32, device=dev)
    n_out = torch.empty((1,), dtype=torch.int32, device=dev)
    topk = min(topk, n_chunks)
    cap = topk * B
    ck = torch.empty((1, Hkv, cap, d), dtype=torch.bfloat16, device=dev)
    cv = torch.empty((1, Hkv, cap, d), dtype=torch.bfloat16, device=dev)
    pos = torch.empty((cap,), dtype=torch.int32, device=dev)
    length = torch.empty((1,), dtype=torch.int32, device=dev)

    materialized = args.last_layer == "materialized"
    if materialized:
        mat_ws = torch.empty(sx.materialized_bytes(last.desc), dtype=torch.uint8, device=dev)

    def score_select():
        # chunk scores of the root row and their top-k, one launch (two beyond 1024 chunks)
        sx.chunk_scores_select(last.desc, last.workspace, 0, topk, idx, n_out, scores=scores)

    def gather():
        sx.gather_draft_kv(draft_k, draft_v, ck, cv, idx, n_out, topk, 1, Hkv, L, cap, d, B, 2, pos, length)

    def layers(first, count, buffers=None):
        for l in range(first, first + count):
            buf = buffers or (last if l == n_layers - 1 else plain)
            sx.verify_attn(buf.desc, q[l], kp[l], vp[l], kt[l], vt[l], parent, outs[l], buf.lse, buf.workspace)

    def step():
        layers(0, n_layers - 1 if materialized else n_layers)
        if materialized:
            l = n_layers - 1
            sx.attn_materialized(last.desc, q[l], kp[l], vp[l], kt[l], vt[l], parent, outs[l], last.lse, mat_ws)
            sx.chunk_scores_materialized(last.desc, mat_ws, 0, scores)
            sx.select_chunks(scores, n_chunks, topk, idx, n_out)
        else:
            score_select()
        gather()

    stream = torch.cuda.Stream()

    def graphed(fn):
        """fn captured once in a HIP graph (or fn itself with --no-graph)."""
        if args.no_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            fn()
        return g.replay

    def event_time_us(run, reps):
        """Average GPU time of `run` over `reps` back-to-back calls, HIP events on the launch stream."""
        run()
        stream.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            run()
        e1.record(stream)
        stream.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    with torch.cuda.stream(stream):
        for _ in range(max(args.warmup, 1)):
            step()
        layers(0, n_layers, only)
        stream.synchronize()
        run_step = graphed(step)
        run_prefix = graphed(lambda: layers(0, n_layers, only))
        for _ in range(2):
            run_step()
        stream.synchronize()

        if args.issue_probe:
            return issue_probe(sx, event_time_us)
        if args.hold > 0:
            return hold(args, sx, torch, stream, run_step, run_prefix, n_layers, layer_bytes,
                        4.0 * d * T * (Hq // Hkv) * Hkv * L)

        # ---- timed region: exactly K steps ----
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps

        # ---- the same K steps once more, each between its own pair of events: median and minimum ----
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for a, b in evs:
            a.record(stream)
            run_step()
            b.record(stream)
        stream.synchronize()
        per_step = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)

        # ---- dominant kernel: prefix pass, HIP events on the launch stream ----
        prefix_us = event_time_us(run_prefix, args.steps) / n_layers

        # ---- the retrieval steps on their own (32 calls per graph, so that launch gaps count as they do in a step) ----
        reps = 32
        a45_us = event_time_us(graphed(lambda: [score_select() for _ in range(reps)]), 10) / reps
        a6_us = event_time_us(graphed(lambda: [gather() for _ in range(reps)]), 10) / reps

        # ---- hot figures for the single-layer workloads: one K/V copy, resident in the caches ----
        hot = None
        if single:
            hot_layer_us = event_time_us(graphed(lambda: [layers(0, 1, plain) for _ in range(reps)]), 10) / reps
            hot_prefix_us = event_time_us(graphed(lambda: [layers(0, 1, only) for _ in range(reps)]), 10) / reps
            hot = {"label": "hot: one K/V copy re-read from the caches by every launch",
                   "us_per_layer": round(hot_layer_us, 3), "prefix_us_per_launch": round(hot_prefix_us, 3),
                   "prefix_GBps": round(layer_bytes / (hot_prefix_us * 1e-6) / 1e9, 1)}

        # ---- measured ceilings of this GPU, same run ----
        calib = None
        if not args.no_calibrate:
            calib = calibrate(sx, torch, stream, event_time_us)

    assert int(n_out.item()) == topk and cap - B < int(length.item()) <= cap

    bytes_per_launch = layer_bytes                             # one layer's K and V prefix, bf16
    flops_per_launch = 4.0 * d * T * (Hq // Hkv) * Hkv * L     # QK^T and PV, 2 flops per MAC
    achieved_gbs = bytes_per_launch / (prefix_us * 1e-6) / 1e9
    achieved_tf = flops_per_launch / (prefix_us * 1e-6) / 1e12
    step_us = ms_per_step * 1e3
    gather_bytes = 2 * 2 * Hkv * cap * d * 2                   # K and V, read + written
    default_workload = (args.config == "4" and L == 16384 and Hkv == 8 and args.num_splits == 0 and
                        args.merge == "two-launch" and args.operands == "recipe")
    traffic = measured_traffic() if default_workload else None
    result = {
        "metric": "us per verification step (all layers) at 16K prefix" if (args.config == "4" and L == 16384 and Hkv == 8)
                  else f"us per verification step ({n_layers} layers) at prefix {L}",
        "value": round(step_us, 2),
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic" if args.operands == "recipe" else
                f"synthetic, {args.operands} operands: a probe of data-dependent power, not the metric's workload",
        "config": {
            "workload": f"config {args.config}: {n_layers} layers x (Hq={Hq}, Hkv={Hkv}, d={d}) bf16, prefix {L}, {T}-node tree, "
                        f"chunk {B}, top-{topk} of {n_chunks}, draft gather 1x{Hkv}x{cap}x{d}"
                        + (" (every layer its own K/V copy: cold)" if single else ""),
            "arithmetic": "bf16 inputs, fp32 accumulation on the matrix cores; split partials cross HBM as fp16 "
                          "after a per-row power-of-two rescale",
            "us_per_layer": round(step_us / n_layers, 2),
            "step_us_median": round(per_step[len(per_step) // 2], 2),
            "step_us_min": round(per_step[0], 2),
            "num_splits": sx.num_splits(plain.desc),
            "graph_replay": not args.no_graph,
            "last_layer": args.last_layer,
            "merge": args.merge,
            "step_hbm_GBps": round(n_layers * bytes_per_launch / (step_us * 1e-6) / 1e9, 1),
            "step_mfma_TFLOPs": round(n_layers * flops_per_launch / (step_us * 1e-6) / 1e12, 1),
            "a1_prefix_us_per_layer": round(prefix_us, 3),
            "a2a3_tree_merge_us_per_layer": round((step_us - a45_us - a6_us) / n_layers - prefix_us, 3),
            "a4a5_scores_select_us": round(a45_us, 3),
            "a6_gather_us": round(a6_us, 3),
            "gather_GBps": round(gather_bytes / (a6_us * 1e-6) / 1e9, 1),
            "gather_copy_frac": round(gather_bytes / (a6_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        },
        "roofline": {
            "kernel": ("prefix_generic_kernel (split-K prefix pass on the vector ALUs" if args.valu_prefix else
                       ("prefix_rows_kernel" if (T * (Hq // Hkv) > 32 or d == 64) else "prefix_mfma_kernel") +
                       " (split-K prefix pass on the matrix cores") + ", one layer per launch)",
            "bound": "hbm",
            "achieved": round(achieved_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
            "traffic": traffic["bytes"] if traffic else None,
            "algorithmic_bytes": bytes_per_launch,
            "us_per_launch": round(prefix_us, 3),
            "mfma_TFLOPs": round(achieved_tf, 1),
            "mfma_frac": round(achieved_tf / MFMA_BF16_PEAK_TFLOPS, 4),
        },
    }
    rf = result["roofline"]
    if traffic:
        rf.update({"traffic_over_algorithmic": round(traffic["bytes"] / bytes_per_launch, 3),
                   "traffic_fetch_bytes": traffic["fetch_bytes"], "traffic_write_bytes": traffic["write_bytes"],
                   "traffic_measured_at_commit": traffic["commit"]})
    if hot:
        result["config"]["hot"] = hot
    if calib:
        rf.update({"measured_hbm_GBps": calib["hbm_GBps"], "measured_mfma_TFLOPs": calib["mfma_TFLOPs"],
                   "frac_of_measured": round(achieved_gbs / calib["hbm_GBps"], 4),
                   "mfma_frac_of_measured": round(achieved_tf / calib["mfma_TFLOPs"], 4),
                   # the share of each measured ceiling the kernel uses; on this part the two draw on one power
                   # budget, so their sum (not either alone) says how close the kernel is to what the chip gives
                   "sum_of_measured_fracs": round(achieved_gbs / calib["hbm_GBps"] + achieved_tf / calib["mfma_TFLOPs"], 4),
                   "calibration": calib["how"]})
        result["config"]["gather_copy_frac_of_measured"] = round(gather_bytes / (a6_us * 1e-6) / 1e9 / calib["hbm_GBps"], 4)

    if T * (Hq // Hkv) * 1.0 > MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS:
        # more flops per K/V byte than the ridge point: the matrix roof is the binding one
        rf.update({"bound": "mfma", "achieved": rf["mfma_TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                   "frac": rf["mfma_frac"], "hbm_GBps": round(achieved_gbs, 1)})
        if calib:
            rf["frac_of_measured"] = rf["mfma_frac_of_measured"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, n_layers, L, B, topk)
    print(json.dumps(result))


def hold(args, sx, torch, stream, run_step, run_prefix, n_layers, layer_bytes, layer_flops):
    """Loop one kind of work for args.hold seconds and report the rate it sustained."""
    nbytes = 2 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1) if args.hold_what == "stream" else None
    flops = [0]

    def mfma():
        flops[0] = sx.calib_mfma(20000, 32, 512)

    run = {"stream": lambda: sx.calib_stream_read(buf, nbytes), "mfma": mfma, "prefix": run_prefix, "step": run_step}[args.hold_what]
    run()
    stream.synchronize()
    n = 0
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < args.hold:
        for _ in range(20):
            run()
        stream.synchronize()
        n += 20
    dt = time.perf_counter() - t0
    us = dt / n * 1e6
    out = {"hold": args.hold_what, "seconds": round(dt, 2), "launches": n, "us_per_launch": round(us, 2)}
    if args.hold_what == "stream":
        out["GBps"] = round(nbytes / us / 1e3, 1)
    elif args.hold_what == "mfma":
        out["TFLOPs"] = round(flops[0] / us / 1e6, 1)
    else:
        per = us / n_layers if args.hold_what == "prefix" else us / n_layers
        out.update({"us_per_layer": round(per, 2), "GBps": round(layer_bytes / per / 1e3, 1),
                    "TFLOPs": round(layer_flops / per / 1e6, 1)})
    print(json.dumps(out))


def issue_probe(sx, event_time_us):
    """How the matrix and the vector instructions of the two waves of a SIMD share it: 256 workgroups of eight waves
    (w and w + 4 on one SIMD), 2000 iterations of 16 matrix instructions and / or 16 x n vector instructions per wave."""
    iters, wgs = 2000, 256
    out = {"issue_probe": "specext_calib_issue_mix", "iters": iters, "workgroups": wgs, "us": {}}
    for n in (4, 8):
        for mode, name in ((1, "matrix_waves_alone"), (2, "vector_waves_alone"), (3, "matrix_waves_and_vector_waves")):
            if mode == 1 and n == 8:
                continue
            out["us"][f"{name}_n{n}"] = round(event_time_us(lambda: sx.calib_issue_mix(mode, n, iters, wgs), 5), 1)
    for n in (0, 4, 8):
        out["us"][f"all_waves_in_turns_n{n}"] = round(event_time_us(lambda: sx.calib_issue_mix(4, n, iters, wgs), 5), 1)
    print(json.dumps(out))


def calibrate(sx, torch, stream, event_time_us):
    """What this GPU sustains: a pure HBM read stream over 2 GiB (eight times the last-level cache) and a pure
    dense bf16 matrix-core loop, both from the library's calibration kernels, timed like everything else here."""
    nbytes = 2 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    t_read = event_time_us(lambda: sx.calib_stream_read(buf, nbytes), 10)
    del buf
    flops = [0]

    def mfma():
        flops[0] = sx.calib_mfma(20000, 32, 512)

    t_mfma = event_time_us(mfma, 3)
    return {"hbm_GBps": round(nbytes / (t_read * 1e-6) / 1e9, 1), "mfma_TFLOPs": round(flops[0] / (t_mfma * 1e-6) / 1e12, 1),
            "how": "specext_calib_stream_read over 2 GiB x 10; specext_calib_mfma (v_mfma_f32_32x32x16_bf16 only, "
                   "2 waves per SIMD) 12 ms x 3; same process, same stream"}


def bench_prefill(args):
    """Prefill attention of a prompt of --prefix tokens on all layers (each layer its own Q/K/V in HBM)."""
    import numpy as np
    import torch

    import paper_2505_20776_amd as sx

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    Hq, Hkv, d, L, n_layers = 32, 8, 128, args.prefix or 16384, args.layers or 32
    gen = torch.Generator(device=dev)
    gen.manual_seed(4100)
    randn = lambda *shape: torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = [randn(L, Hq, d) for _ in range(n_layers)]
    k = [randn(Hkv, L, d) for _ in range(n_layers)]
    v = [randn(Hkv, L, d) for _ in range(n_layers)]
    out = torch.empty((L, Hq, d), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((Hq, L), dtype=torch.float32, device=dev)

    def step():
        for l in range(n_layers):
            sx.prefill_attn(q[l], k[l], v[l], out, lse, Hq, Hkv, d, L, L)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(max(args.warmup, 1)):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / (args.steps * n_layers)
    flops = 4.0 * d * Hq * L * (L + 1) / 2                    # QK^T and PV over the causal half, 2 flops per MAC
    tflops = flops / (kernel_ms * 1e-3) / 1e12
    result = {
        "metric": "ms per prefill attention pass (all layers)", "value": round(ms_per_step, 4), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"prefill: {n_layers} layers x (Hq=32, Hkv=8, d=128) bf16, prompt {L}, causal"},
        "roofline": {"kernel": "prefill_rows_kernel (causal attention on the matrix cores, one layer per launch)",
                     "bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                     "algorithmic_flops": flops, "ms_per_launch": round(kernel_ms, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle as orc
        from workloads import quantize
        rng = np.random.default_rng(4100)
        mk = lambda *shape: quantize(rng.standard_normal(shape).astype(np.float32), "bf16")
        qs, ks, vs = mk(L, Hq, d), mk(Hkv, L, d), mk(Hkv, L, d)
        rows = sorted(int(x) for x in rng.integers(0, L, size=3000))
        t0 = time.perf_counter()
        orc.prefill_attention(qs, ks, vs, rows=rows)
        t = time.perf_counter() - t0
        mean_keys = float(np.mean([r + 1 for r in rows]))
        scaled = t * (L * (L + 1) / 2) / (mean_keys * len(rows)) * n_layers
        result["cpu_baseline"] = {"value": round(scaled * 1e3, 1), "unit": "ms", "cores": int(os.cpu_count() or 1),
                                  "kind": "oracle",
                                  "sample": f"fp64 numpy oracle on {len(rows)} random query rows of one layer "
                                            f"({t:.1f} s), scaled by key count to all rows and {n_layers} layers"}
    print(json.dumps(result))


def cpu_baseline(args, n_layers, L, B, topk):
    """The fp64 oracle, as it stands, on the host cores for a bounded sample."""
    import numpy as np

    import oracle as orc
    from workloads import config_tree, config_workload

    sample_layers = max(1, min(args.cpu_layers, n_layers))
    t_attn = 0.0
    wl = None
    for l in range(sample_layers):
        if args.config == "draft68m":
            from workloads import make_workload
            wl = make_workload("draft68m", seed=6800 + l, dtype="bf16", n_q_heads=12, n_kv_heads=12, head_dim=64,
                               prefix_len=L, parent=config_tree(2), chunk_size=B, top_k=topk, n_needles=0)
        else:
            cfg = 2 if args.config == "draft" else int(args.config[0])
            wl = config_workload(cfg, item=l, prefix_len=L, variant="" if args.config == "draft" else args.config[1:])
        t0 = time.perf_counter()
        orc.verify_attention(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent)
        t_attn += time.perf_counter() - t0
    t0 = time.perf_counter()
    sc = orc.chunk_scores(wl.q, wl.k_prefix, wl.v_prefix, wl.k_tree, wl.v_tree, wl.parent, B)
    sel = orc.select_chunks(sc[0], topk)
    src = wl.k_prefix[None]
    orc.gather_draft_kv(src, src, sel, B)
    t_tail = time.perf_counter() - t0
    step_s = t_attn / sample_layers * n_layers + t_tail
    try:
        import threadpoolctl
        threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        threads = os.cpu_count() or 1
    return {
        "value": round(step_s * 1e6, 1),
        "unit": "us",
        "cores": int(threads),
        "kind": "oracle",
        "sample": f"fp64 numpy oracle: attention of {sample_layers} of {n_layers} layers timed "
                  f"({t_attn:.1f} s) and scaled to {n_layers}, plus chunk scores + select + gather once "
                  f"({t_tail:.1f} s)",
    }


if __name__ == "__main__":
    main()
