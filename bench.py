#!/usr/bin/env python3
"""Benchmark of the FloE decode hot path on one MI355X.

A "step" is one pass of the whole path (router, quantized up GEMV, threshold selection, gathered
gate/down GEMVs, top-2 combine) for one decode token through one Mixtral-shaped MoE layer:
8 experts of d=4096, f=14336, up projection INT2 with group 64, thresholds set for 90 % channel
sparsity, softmax top-2 renormalised.  Inputs are seeded and synthetic (floe_synth), weights and
tokens are resident in HBM before the timed region, and consecutive steps rotate over several copies
of the layer so that weights come from HBM and not from the 256 MB last-level cache.

Prints ONE JSON line: metric = microseconds per MoE layer-token (lower is better), plus
  "roofline":     achieved algorithmic GB/s of the dominant kernel against the 8 TB/s HBM peak,
                  its duration read with HIP events around that kernel on the launch stream,
  "cpu_baseline": the CPU oracle timed on a bounded sample of the same tokens.
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

HBM_PEAK_GBS = 8000.0
D, F_INT, BITS, GROUP, N_EXPERTS, TOP_K, PCT = 4096, 14336, 2, 64, 8, 2, 90
CONFIG_ID, SEED = 3, 0
N_TOKENS = 16          # distinct decode tokens the steps cycle through
TRAFFIC_PROFILE = os.path.join("profiles", "layer_decode_config3_T1_hbm_traffic.md")


def measured_traffic():
    """HBM bytes per launch of each kernel of THIS workload as the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    summary states them (hardware counters cannot be read from inside this process).  Returns ({kernel: bytes}, note);
    the note names the file and the kernel-source state it was taken at, so a reader can tell whether it is current."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    out, note = {}, None
    try:
        for line in open(path):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 7 and cells[1].startswith("fused_ffn_kernel"):
                out["fused_ffn"] = float(cells[6]) * 1e6
            elif len(cells) > 7 and cells[1].startswith("combine_kernel"):
                out["combine"] = float(cells[6]) * 1e6
            elif line.lower().startswith("kernel sources at"):
                note = line.strip()
    except (OSError, ValueError):
        return {}, None
    return out, f"{TRAFFIC_PROFILE}" + (f" ({note})" if note else "")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def stable_tokens(S, wr, n):
    """Seeded tokens whose top-k routing does not hinge on rounding (gap between the k-th and (k+1)-th
    logit above 1e-3 relative); decided from fp64 logits computed here with numpy (harness logic)."""
    import numpy as np
    out, i = [], 0
    w64 = wr.astype(np.float64)
    while len(out) < n:
        x = S.tokens(SEED, CONFIG_ID, 1, D, layer=1000 + i)[0]
        i += 1
        lg = np.sort(w64 @ x.astype(np.float64))[::-1]
        p = np.exp(lg - lg[0])
        if (p[TOP_K - 1] - p[TOP_K]) > 1e-3 * p[TOP_K - 1]:
            out.append(x)
    return np.stack(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=80)
    ap.add_argument("--copies", type=int, default=8, help="layer copies rotated over (HBM, not cache, reads)")
    ap.add_argument("--launch", choices=["graph", "stream"], default="graph",
                    help="graph: the K steps are replayed from one HIP graph; stream: plain launches")
    ap.add_argument("--workload", choices=["layer", "expert", "stage", "stack", "batch", "variants"], default="layer",
                    help="layer: the headline metric (default); expert: single-expert sweep over bit widths and "
                         "sparsity levels (Table 1 protocol); stage: host->HBM transfer of selected channels; "
                         "stack: 32 offloaded layers per token, gate/down matrices in pinned host memory; "
                         "batch: decode batches of configs[2] (T=1,4,16) and configs[4] (T=1,8,32); "
                         "variants: the three sparsification candidates of Sec. 3.2.1 on one expert")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy five times (reference for hardware-counter runs)")
    ap.add_argument("--batch-cases", default="", help="batch workload only: cases to run as config:T,... "
                                                      "(e.g. 2:16,4:32; empty = all)")
    ap.add_argument("--union-kernels", type=int, default=0, help="floe_tuning(FLOE_TUNE_UNION_KERNELS): 0 = library default")
    ap.add_argument("--stack-parts", default="plain,budget,cache,prefetch",
                    help="stack workload only: which measurements to run (a short list makes a short profile)")
    ap.add_argument("--grouped-gemv", type=int, default=0, help="floe_tuning(FLOE_TUNE_GROUPED_GEMV): 0 = library default")
    ap.add_argument("--fused-tasks", type=int, default=0, help="floe_tuning(FLOE_TUNE_FUSED_TASKS): 0 = library default")
    ap.add_argument("--copy-workgroups", type=int, default=0, help="floe_tuning(FLOE_TUNE_STAGE_WORKGROUPS): 0 = library default")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import floe_synth as S
    import paper_2505_05950_amd as FL

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    FL.load()
    if args.union_kernels:
        FL.floe_tuning(FL.TUNE_UNION_KERNELS, args.union_kernels)
    if args.grouped_gemv:
        FL.floe_tuning(FL.TUNE_GROUPED_GEMV, args.grouped_gemv)
    if args.fused_tasks:
        FL.floe_tuning(FL.TUNE_FUSED_TASKS, args.fused_tasks)
    if args.copy_workgroups:
        FL.floe_tuning(FL.TUNE_STAGE_WORKGROUPS, args.copy_workgroups)
    K, W, R = args.steps, args.warmup, max(1, args.copies)
    if args.workload == "expert":
        return bench_expert(args, np, torch, S, FL, dev)
    if args.workload == "stage":
        return bench_stage(args, np, torch, S, FL, dev)
    if args.workload == "stack":
        return bench_stack(args, np, torch, S, FL, dev)
    if args.workload == "batch":
        return bench_batch(args, np, torch, S, FL, dev)
    if args.workload == "variants":
        return bench_variants(args, np, torch, S, FL, dev)

    # ---------------------------------------------------------------- inputs (seeded, synthetic)
    t0 = time.time()
    wr = S.router_weights(SEED, CONFIG_ID, N_EXPERTS, D)
    xs = stable_tokens(S, wr, N_TOKENS)
    w_ups, gds = [], []
    for e in range(N_EXPERTS):
        w_up, gd = S.expert_weights(SEED, CONFIG_ID, D, F_INT, 0, e)
        w_ups.append(w_up)
        gds.append(gd)
    log(f"[bench] generated 8 experts in {time.time() - t0:.1f}s")

    # S0 on the GPU (offline step, timed on its own)
    base = []
    q_ms = []
    for e in range(N_EXPERTS):
        w_dev = torch.from_numpy(w_ups[e]).to(dev)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        codes, scale, zero = FL.floe_quantize_expert(w_dev, BITS, GROUP)
        b.record()
        torch.cuda.synchronize()
        q_ms.append(a.elapsed_time(b))
        base.append((codes, scale, zero, torch.from_numpy(gds[e]).to(dev)))
        del w_dev
    x_dev = torch.from_numpy(xs).to(dev)
    wr_dev = torch.from_numpy(wr).to(dev)

    # thresholds: per (token, expert) the ceil(f*pct/100)-th smallest |v| of the library's own v
    # (calibration is harness work: the paper derives its thresholds offline from an empirical CDF)
    z = -(-F_INT * PCT // 100)
    tau = torch.empty((N_TOKENS, N_EXPERTS), dtype=torch.float32, device=dev)
    for e in range(N_EXPERTS):
        v = FL.floe_up_gemv(base[e][0], base[e][1], base[e][2], x_dev, D, BITS, GROUP)
        tau[:, e] = torch.kthvalue(v.abs(), z, dim=1).values
    torch.cuda.synchronize()

    layers = []
    for r in range(R):
        experts = []
        for e in range(N_EXPERTS):
            c, s, zz, gd = base[e] if r == 0 else tuple(t.clone() for t in base[e])
            experts.append(FL.Expert(D, F_INT, BITS, GROUP, c, s, zz, gd))
        layers.append(FL.Layer(experts, 0, TOP_K, True, wr_dev if r == 0 else wr_dev.clone(), tau[0:1], True))
    tau_rows = [tau[i:i + 1].contiguous() for i in range(N_TOKENS)]
    x_rows = [x_dev[i:i + 1].contiguous() for i in range(N_TOKENS)]
    y = torch.empty((1, D), dtype=torch.float16, device=dev)
    ws = layers[0].workspace(1)
    stats = torch.zeros((1, TOP_K, 4), dtype=torch.int32, device=dev)

    def step(i, st=None):
        L = layers[i % R]
        L.set_tau(tau_rows[i % N_TOKENS], True)
        FL.floe_moe_layer_decode(L, x_rows[i % N_TOKENS], y, st, ws)

    # K per (token, slot): needed for the byte model
    Ks = np.zeros((N_TOKENS, TOP_K), np.int64)
    for i in range(N_TOKENS):
        step(i, stats)
        torch.cuda.synchronize()
        Ks[i] = stats.cpu().numpy().reshape(TOP_K, 4)[:, 1]
    log(f"[bench] selected channels per (token, slot): min {Ks.min()} mean {Ks.mean():.1f} max {Ks.max()}")

    # ---------------------------------------------------------------- timed region
    stream = torch.cuda.Stream()
    graph = None
    with torch.cuda.stream(stream):
        for i in range(W):
            step(i)
        stream.synchronize()
        if args.launch == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(K):
                    step(W + i)
            graph.replay()          # one untimed replay after instantiation
            stream.synchronize()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_wall = time.perf_counter()
        e0.record(stream)
        if graph is not None:
            graph.replay()
        else:
            for i in range(K):
                step(W + i)
        e1.record(stream)
        torch.cuda.synchronize()
        t_wall = time.perf_counter() - t_wall
    ms_total = max(e0.elapsed_time(e1), 0.0)
    ms_per_step = ms_total / K
    us_per_layer_token = ms_per_step * 1e3      # T = 1

    # spread of the same metric: the K steps again in chunks of 10 consecutive steps, every chunk timed on its own
    # (a second pass: the value above stays the plain total over K steps)
    chunk = 10
    n_chunks = max(1, K // chunk)
    chunk_us = []
    with torch.cuda.stream(stream):
        graphs = []
        if args.launch == "graph":
            for c in range(n_chunks):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(chunk):
                        step(W + c * chunk + i)
                graphs.append(g)
            for g in graphs:
                g.replay()
            stream.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_chunks)]
        for c in range(n_chunks):
            evs[c][0].record(stream)
            if graphs:
                graphs[c].replay()
            else:
                for i in range(chunk):
                    step(W + c * chunk + i)
            evs[c][1].record(stream)
        stream.synchronize()
        chunk_us = [a.elapsed_time(b) * 1e3 / chunk for a, b in evs]
        del graphs
    spread = {"median": round(float(np.median(chunk_us)), 3), "p10": round(float(np.percentile(chunk_us, 10)), 3),
              "p90": round(float(np.percentile(chunk_us, 90)), 3),
              "over": f"{n_chunks} chunks of {chunk} consecutive steps, each replayed and timed on its own"}

    # ---------------------------------------------------------------- per-kernel durations (HIP events)
    # A pair of events around one kernel reads the kernel's duration plus a fixed cost o of the two markers.
    # In the timed graph the kernels of a step run back to back (each waits for the one before it), so a
    # step lasts the sum of their durations: o = (sum of the bracketed reads - graph step time) / number of kernels.
    # With --launch stream there is no such step time, and o comes from a copy kernel instead: a bracket around
    # one launch reads t + o, one around nine launches 9t + o.
    # (At T = 1 the layer is two kernels: router, up GEMV, selection and gate/down in one, then the combine.)
    raw, raw_spread = {}, {}
    with torch.cuda.stream(stream):
        for name in ("fused_ffn", "combine"):
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
            for a, b in pairs:          # torch creates the hipEvent_t on first record
                a.record(stream)
                b.record(stream)
            stream.synchronize()
            for i in range(K):
                FL.floe_profile_kernel(name, pairs[i][0], pairs[i][1])
                step(W + i)
            FL.floe_profile_kernel("none")
            stream.synchronize()
            reads = [a.elapsed_time(b) * 1e3 for a, b in pairs]
            raw[name] = float(np.mean(reads))
            raw_spread[name] = [float(np.median(reads)), float(np.percentile(reads, 10)), float(np.percentile(reads, 90))]
        if args.launch == "graph":
            bracket_us = (sum(raw.values()) - ms_per_step * 1e3) / len(raw)
        else:
            src = torch.empty(8 << 20, dtype=torch.uint8, device=dev)
            dst = torch.empty_like(src)
            reads = {1: [], 9: []}
            for rep in range(60):
                for n in (1, 9):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record(stream)
                    for _ in range(n):
                        dst.copy_(src)
                    b.record(stream)
                    stream.synchronize()
                    if rep >= 10:
                        reads[n].append(a.elapsed_time(b) * 1e3)
            e1, e9 = float(np.mean(reads[1])), float(np.mean(reads[9]))
            bracket_us = e1 - (e9 - e1) / 8.0
        bracket_us = min(max(bracket_us, 0.0), 0.75 * min(raw.values()))
    per_kernel = {n: raw[n] - bracket_us for n in raw}
    torch.cuda.synchronize()

    # ---------------------------------------------------------------- byte model (algorithmic bytes)
    # what the method has to move per layer-token: the routed experts' codes, scales and zeros; the [gate | down]
    # chunks of the selected channels; the router matrix, x; one fp32 result per routed expert and the fp16 output.
    # (v, the mask and the index list stay inside the compute unit and are not counted.)
    codes_meta = D * F_INT * BITS // 8 + 4 * F_INT * (D // GROUP)
    k_steps = np.array([Ks[(W + i) % N_TOKENS] for i in range(K)])          # [K][TOP_K]
    k_mean = float(np.mean(k_steps.sum(axis=1)))
    bytes_router = N_EXPERTS * D * 2 + 2 * D
    bytes_fused = TOP_K * codes_meta + k_mean * 2 * 2 * D + bytes_router + TOP_K * 4 * D
    bytes_combine = TOP_K * 4 * D + 2 * D
    bytes_step = bytes_fused + bytes_combine
    kernel_bytes = {"fused_ffn": bytes_fused, "combine": bytes_combine}
    traffic, traffic_note = measured_traffic()
    dominant = max(per_kernel, key=lambda n: per_kernel[n])
    dom_gbs = kernel_bytes[dominant] / (per_kernel[dominant] * 1e-6) / 1e9
    kernels = {n: {"us": round(per_kernel[n], 3), "algorithmic_bytes": int(kernel_bytes[n]),
                   "GBps": round(kernel_bytes[n] / (per_kernel[n] * 1e-6) / 1e9, 1),
                   "us_median_p10_p90": [round(v - bracket_us, 3) for v in raw_spread[n]]} for n in per_kernel}
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(dom_gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get(dominant), "traffic_source": traffic_note,
                "kernel_us": round(per_kernel[dominant], 3), "kernels": kernels,
                "layer_bytes": int(bytes_step),
                "layer_frac": round(bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "event_bracket_overhead_us": round(bracket_us, 3),
                "timing": "hipEvent pair recorded around each launch of the kernel in a second pass over the same K steps, "
                          "minus the cost of the two markers (live: the share per kernel of what the bracketed reads sum to beyond the graph's step time)"}

    if args.calib_copy:
        src = torch.ones((64 << 20,), dtype=torch.float32, device=dev)     # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as O
        threads = max(1, min(16, os.cpu_count() or 1))
        O.set_threads(threads)
        ex_np = []
        for e in range(N_EXPERTS):
            ex_np.append(O.quantize(w_ups[e], BITS, GROUP) + (gds[e],))
        done, spent, n_tok = 0, 0.0, 0
        while spent < args.cpu_seconds and n_tok < N_TOKENS:
            xt = xs[n_tok:n_tok + 1]
            ids, _, _ = O.router(wr, xt[0], TOP_K, True)
            tau_np = np.zeros((1, N_EXPERTS), np.float32)
            for e in ids:      # calibration, not timed
                tau_np[0, e] = O.threshold_for_sparsity(O.up_gemv(*ex_np[e][:3], D, BITS, GROUP, xt[0]), PCT)
            t1 = time.perf_counter()
            O.moe_layer(ex_np, 0, TOP_K, True, wr, xt, tau_np, BITS, GROUP)
            spent += time.perf_counter() - t1
            if n_tok == 0:
                tau_first = tau_np
            n_tok += 1
        cpu = {"value": round(spent / n_tok * 1e6, 1), "unit": "us per MoE layer-token", "cores": threads, "kind": "oracle",
               "sample": f"{n_tok} of the {N_TOKENS} benchmark tokens through the same layer (router, up GEMV, select, "
                         f"gate/down, combine); threshold calibration not timed"}
        # the same call on one thread (the oracle as its definition reads), on the first token only
        O.set_threads(1)
        t1 = time.perf_counter()
        O.moe_layer(ex_np, 0, TOP_K, True, wr, xs[0:1], tau_first, BITS, GROUP)
        cpu["one_thread_us"] = round((time.perf_counter() - t1) * 1e6, 1)

    out = {
        "metric": "us per MoE layer-token (Mixtral-shape compressed sparse expert layer, decode)",
        "value": round(us_per_layer_token, 3), "unit": "us", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "int2 codes x fp16, fp32 accumulate", "data": "synthetic",
        "config": {"workload": "BASELINE configs[2] at T=1: one Mixtral-shaped MoE layer, 8 experts d=4096 f=14336, "
                               "INT2 group 64 up projection, 90% channel sparsity, softmax top-2 renormalised, 1 decode token",
                   "launch": args.launch, "layer_copies_rotated": R, "tokens_cycled": N_TOKENS,
                   "mean_selected_channels": round(float(Ks.mean()), 1),
                   "quantize_ms_per_expert": round(float(np.mean(q_ms[1:])), 3),
                   "wall_ms_per_step": round(t_wall * 1e3 / K, 6), "us_per_step_spread": spread},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


def _graph_time(torch, stream, fn, K, W, reps=1, spread=None):
    """W warm-up calls, then K calls replayed from one HIP graph (reps timed replays); returns the mean ms per call and
    fills `spread` (median, p10, p90 over the replays) when given."""
    with torch.cuda.stream(stream):
        for i in range(W):
            fn(i)
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for i in range(K):
                fn(W + i)
        g.replay()
        stream.synchronize()
        reads = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            g.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            reads.append(e0.elapsed_time(e1) / K)
    if spread is not None:
        import numpy as np
        spread.update({"median": float(np.median(reads)), "p10": float(np.percentile(reads, 10)),
                       "p90": float(np.percentile(reads, 90)), "replays": reps})
    return reads[0] if reps == 1 else float(sum(reads) / len(reads))


def bench_expert(args, np, torch, S, FL, dev):
    """BASELINE configs[1]: one Mixtral-shaped expert, 1 token, bit widths 2/3/4 and sparsity 0/50/80/90 %
    (the shape of the paper's Table 1: dense up GEMV + fused SiLU + sparse gate and down GEMVs)."""
    K, W = args.steps, args.warmup
    w_up, gd = S.expert_weights(SEED, 2, D, F_INT)
    x = torch.from_numpy(S.tokens(SEED, 2, 1, D)).to(dev)
    w_dev = torch.from_numpy(w_up).to(dev)
    gd_dev = torch.from_numpy(gd).to(dev)
    copies = 4                                        # 4 x (235 MB + codes) > last-level cache
    gds = [gd_dev] + [gd_dev.clone() for _ in range(copies - 1)]
    stream = torch.cuda.Stream()
    rows = []
    for bits in (2, 3, 4):
        q = [FL.floe_quantize_expert(w_dev, bits, GROUP)]
        q += [tuple(t.clone() for t in q[0]) for _ in range(copies - 1)]
        experts = [FL.Expert(D, F_INT, bits, GROUP, q[c][0], q[c][1], q[c][2], gds[c]) for c in range(copies)]
        v = FL.floe_up_gemv(q[0][0], q[0][1], q[0][2], x, D, bits, GROUP)
        for pct in (0, 50, 80, 90):
            z = -(-F_INT * pct // 100)
            tau = torch.full((1,), -1.0, device=dev) if z == 0 else torch.kthvalue(v.abs(), z, dim=1).values.contiguous()
            y = torch.zeros((1, D), dtype=torch.float32, device=dev)
            idx = torch.empty((1, F_INT), dtype=torch.int32, device=dev)
            cnt = torch.zeros((1,), dtype=torch.int32, device=dev)
            ws = torch.empty((FL.floe_expert_workspace_bytes(D, F_INT, bits, GROUP, 1) + 512,), dtype=torch.uint8, device=dev)

            FL.floe_expert_ffn_sparse(experts[0], x, tau, None, y, idx, cnt, ws)      # once with the list: K
            torch.cuda.synchronize()
            Ksel = int(cnt.item())

            def call(i):            # timed: y only (the index list is not needed for the result)
                FL.floe_expert_ffn_sparse(experts[i % copies], x, tau, None, y, None, None, ws, want_list=False)
            ms = _graph_time(torch, stream, call, K, W)
            # codes + scales + zeros, the selected [gate | down] chunks, x, y (v and the list stay on chip)
            nbytes = D * F_INT * bits // 8 + 4 * F_INT * (D // GROUP) + 2 * Ksel * 2 * D + 2 * D + 4 * D
            rows.append({"bits": bits, "sparsity_pct": pct, "K": Ksel, "us_per_expert_ffn": round(ms * 1e3, 3),
                         "algorithmic_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
            log(f"[bench] expert bits={bits} sparsity={pct}% K={Ksel}: {ms * 1e3:.2f} us, {rows[-1]['GBps']} GB/s")
    head = next(r for r in rows if r["bits"] == 2 and r["sparsity_pct"] == 90)
    print(json.dumps({"metric": "us per expert-FFN (Mixtral-shape expert, 1 token)", "value": head["us_per_expert_ffn"],
                      "unit": "us", "n_gpus": 1, "steps": K, "warmup": W, "higher_is_better": False, "data": "synthetic",
                      "config": {"workload": "BASELINE configs[1]: d=4096 f=14336 group 64, bits 2/3/4 x sparsity 0/50/80/90 %, "
                                             "4 weight copies rotated, HIP-graph replay"},
                      "sweep": rows}), flush=True)


def bench_variants(args, np, torch, S, FL, dev):
    """The three candidates for sparsification of Sec. 3.2.1 on one Mixtral-shaped expert, 1 token: S_t on a_up (FloE),
    on a_gate or on a_down, thresholds for 80 % and 90 % of the compared activation (Eq. 6 on this token).  Reports
    time and the bytes each candidate HAS to read: with a_gate / a_down the whole gate projection comes first."""
    K, W = args.steps, args.warmup
    w_up, gd = S.expert_weights(SEED, 2, D, F_INT)
    x = torch.from_numpy(S.tokens(SEED, 2, 1, D)).to(dev)
    copies = 4
    gd0 = torch.from_numpy(gd).to(dev)
    q0 = FL.floe_quantize_expert(torch.from_numpy(w_up).to(dev), BITS, GROUP)
    experts = [FL.Expert(D, F_INT, BITS, GROUP, *(q0 if c == 0 else tuple(t.clone() for t in q0)), gd0 if c == 0 else gd0.clone())
               for c in range(copies)]
    stream = torch.cuda.Stream()
    codes_meta = D * F_INT * BITS // 8 + 4 * F_INT * (D // GROUP)
    rows = []
    names = {FL.SPARSIFY_UP: "a_up", FL.SPARSIFY_GATE: "a_gate", FL.SPARSIFY_DOWN: "a_down"}
    for pct in (80, 90):
        z = -(-F_INT * pct // 100)
        for which in (FL.SPARSIFY_UP, FL.SPARSIFY_GATE, FL.SPARSIFY_DOWN):
            y = torch.zeros((1, D), dtype=torch.float32, device=dev)
            # the activation that is compared: run once with a threshold below zero and read it back from the lists
            tau0 = torch.full((1,), -1.0, device=dev)
            v = FL.floe_up_gemv(*q0, x, D, BITS, GROUP)
            if which == FL.SPARSIFY_UP:
                act = v
            else:
                g = (x.float() @ gd0[:, 0, :].float().t())
                a_gate = g / (1 + torch.exp(-g))
                act = a_gate if which == FL.SPARSIFY_GATE else a_gate * v      # harness-side calibration only
            tau = torch.kthvalue(act.abs(), z, dim=1).values.contiguous()
            _, _, cnt = FL.floe_expert_ffn_sparsified(experts[0], which, x, tau, None, y)
            torch.cuda.synchronize()
            Ksel = int(cnt.item())
            ws = torch.empty((1 << 26,), dtype=torch.uint8, device=dev)

            def call(i):
                FL.floe_expert_ffn_sparsified(experts[i % copies], which, x, tau, None, y, workspace=ws)
            ms = _graph_time(torch, stream, call, K, W)
            if which == FL.SPARSIFY_UP:
                need = codes_meta + 2 * Ksel * 2 * D                         # codes, then gate and down of the kept channels
            elif which == FL.SPARSIFY_GATE:
                need = F_INT * 2 * D + codes_meta * Ksel // F_INT + Ksel * 2 * D   # all of gate, codes and down of the kept
            else:
                need = F_INT * 2 * D + codes_meta + Ksel * 2 * D             # all of gate, all codes, down of the kept
            rows.append({"thresholded": names[which], "sparsity_pct": pct, "K": Ksel, "us_per_expert_ffn": round(ms * 1e3, 2),
                         "bytes_the_candidate_must_read": int(need), "MB": round(need / 1e6, 1)})
            log(f"[bench] S_t on {names[which]:6s} at {pct} %: K={Ksel}, {ms * 1e3:.1f} us, must read {need / 1e6:.1f} MB")
    print(json.dumps({"metric": "us per expert-FFN for the three sparsification candidates (Sec. 3.2.1)", "value": rows[3]["us_per_expert_ffn"],
                      "unit": "us", "n_gpus": 1, "higher_is_better": False, "data": "synthetic",
                      "config": {"workload": "one Mixtral-shaped expert (d=4096 f=14336, INT2 g64 up projection), 1 token, 4 weight "
                                             "copies rotated, HIP-graph replay"}, "results": rows}), flush=True)


def bench_stage(args, np, torch, S, FL, dev):
    """Transfer experiment of Sec. 4.1 / Sec. 3.4.2 (random 20 % of one expert's channels, 20 trials) plus the 10 %
    case of the decode path.  Selected channels go from pinned host memory to HBM by
      gather_compact : floe_stage_channels on the compact [gate | down] layout (one 4d-byte chunk per channel),
      gather_split   : the same kernel on two separate matrices (two 2d-byte chunks per channel: no compact layout),
      gather_chunk_* : the same bytes cut into smaller chunks (8 KiB, 4 KiB),
      cpu_pack       : rows packed by the host's threads into a pinned buffer, then one asynchronous copy
                       (the list has to come back to the host first; timed with and without that),
      per_row_copies : one asynchronous copy per selected chunk (the naive way),
    beside one plain pinned copy of the same number of bytes."""
    trials = 20
    _, gd = S.expert_weights(SEED, 4, D, F_INT)
    host = torch.from_numpy(gd).pin_memory()
    host_gate = torch.from_numpy(np.ascontiguousarray(gd[:, 0, :])).pin_memory()
    host_down = torch.from_numpy(np.ascontiguousarray(gd[:, 1, :])).pin_memory()
    side = torch.cuda.Stream()
    torch.set_num_threads(max(1, min(16, os.cpu_count() or 1)))

    def timed(fn, n=trials, warm=3):
        ts = []
        for tr in range(n + warm):
            prep = fn(tr, None)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            a.record(side)
            fn(tr, prep)
            b.record(side)
            b.synchronize()
            wall = (time.perf_counter() - t0) * 1e3
            if tr >= warm:
                ts.append((a.elapsed_time(b), wall))
        return float(np.mean([t[0] for t in ts])), float(np.mean([t[1] for t in ts]))

    out = []
    for frac in (0.2, 0.1):
        Ksel = int(F_INT * frac)
        nbytes = Ksel * 4 * D
        dst = torch.empty((Ksel, 2, D), dtype=torch.float16, device=dev)
        cnt = torch.tensor([Ksel], dtype=torch.int32, device=dev)
        res = {"fraction": frac, "channels": Ksel, "bytes": nbytes}

        def sel_dev(tr):
            return torch.from_numpy(S.random_channel_subset(SEED, 4, F_INT, Ksel, salt=tr)).to(dev)

        # --- gather kernel, compact layout
        def gather_compact(tr, idx):
            if idx is None:
                return sel_dev(tr)
            FL.floe_stage_channels(host, idx, cnt, Ksel, dst, None, side, None)
        ms, _ = timed(gather_compact)
        res["gather_compact_GBps"] = round(nbytes / ms / 1e6, 2)

        # --- gather kernel, gate and down in two matrices
        dst_g = torch.empty((Ksel, 2, D // 2), dtype=torch.float16, device=dev)
        dst_d = torch.empty((Ksel, 2, D // 2), dtype=torch.float16, device=dev)
        hg, hd = host_gate.view(F_INT, 2, D // 2), host_down.view(F_INT, 2, D // 2)

        def gather_split(tr, idx):
            if idx is None:
                return sel_dev(tr)
            FL.floe_stage_channels(hg, idx, cnt, Ksel, dst_g, None, side, None)
            FL.floe_stage_channels(hd, idx, cnt, Ksel, dst_d, None, side, None)
        ms, _ = timed(gather_split)
        res["gather_split_GBps"] = round(nbytes / ms / 1e6, 2)

        # --- gather kernel, smaller chunks: the matrix seen as [f * c][2][d / c], c x as many rows selected
        for c in (2, 4):
            hv = host.view(F_INT * c, 2, D // c)
            dstc = torch.empty((Ksel * c, 2, D // c), dtype=torch.float16, device=dev)
            cntc = torch.tensor([Ksel * c], dtype=torch.int32, device=dev)

            def gather_chunk(tr, idx, c=c, hv=hv, dstc=dstc, cntc=cntc):
                if idx is None:
                    base = S.random_channel_subset(SEED, 4, F_INT, Ksel, salt=tr).astype(np.int64)
                    fine = (base[:, None] * c + np.arange(c)[None, :]).reshape(-1).astype(np.int32)
                    return torch.from_numpy(fine).to(dev)
                FL.floe_stage_channels(hv, idx, cntc, Ksel * c, dstc, None, side, None)
            ms, _ = timed(gather_chunk)
            res[f"gather_chunk_{16 // c}KiB_GBps"] = round(nbytes / ms / 1e6, 2)

        # --- host threads pack into pinned memory, one copy
        packed = torch.empty((Ksel, 2, D), dtype=torch.float16).pin_memory()

        def cpu_pack(tr, idx):
            if idx is None:
                return sel_dev(tr)
            idx_h = idx.cpu().long()                    # the list lives on the device: it has to come back first
            torch.index_select(host, 0, idx_h, out=packed)
            with torch.cuda.stream(side):
                dst.copy_(packed, non_blocking=True)
        _, wall = timed(cpu_pack, n=10)
        res["cpu_pack_GBps"] = round(nbytes / wall / 1e6, 2)

        def cpu_pack_list_on_host(tr, idx_h):
            if idx_h is None:
                return torch.from_numpy(S.random_channel_subset(SEED, 4, F_INT, Ksel, salt=tr)).long()
            torch.index_select(host, 0, idx_h, out=packed)
            with torch.cuda.stream(side):
                dst.copy_(packed, non_blocking=True)
        _, wall = timed(cpu_pack_list_on_host, n=10)
        res["cpu_pack_list_on_host_GBps"] = round(nbytes / wall / 1e6, 2)

        # --- one copy per chunk
        def per_row(tr, idx_h):
            if idx_h is None:
                return S.random_channel_subset(SEED, 4, F_INT, Ksel, salt=tr).tolist()
            with torch.cuda.stream(side):
                for k, j in enumerate(idx_h):
                    dst[k].copy_(host[j], non_blocking=True)
        _, wall = timed(per_row, n=3, warm=1)
        res["per_row_copies_GBps"] = round(nbytes / wall / 1e6, 2)

        # --- plain contiguous pinned copy of the same size
        flat = host.view(-1)[: nbytes // 2]
        dflat = torch.empty_like(flat, device=dev)

        def plain(tr, prep):
            if prep is None:
                return 1
            with torch.cuda.stream(side):
                dflat.copy_(flat, non_blocking=True)
        ms, _ = timed(plain)
        res["memcpy_GBps"] = round(nbytes / ms / 1e6, 2)
        res["gather_compact_frac_of_memcpy"] = round(res["gather_compact_GBps"] / res["memcpy_GBps"], 3)
        out.append(res)
        log(f"[bench] stage {frac:.0%}: " + ", ".join(f"{k}={v}" for k, v in res.items() if k.endswith("GBps")))
    print(json.dumps({"metric": "host->HBM GB/s for selected channel chunks (compact layout)", "value": out[0]["gather_compact_GBps"],
                      "unit": "GB/s", "n_gpus": 1, "higher_is_better": True, "data": "synthetic",
                      "config": {"workload": "one Mixtral-shaped expert's [gate|down] matrix in pinned host memory, random "
                                             "20 % / 10 % of channels, 20 trials each (Sec. 4.1 protocol); kernel-gather timed "
                                             "with hipEvents on the side stream, host-driven variants by wall clock",
                                 "host_threads": torch.get_num_threads()},
                      "results": out}), flush=True)


def bench_stack(args, np, torch, S, FL, dev):
    """BASELINE configs[3]: a 32-layer stack of the Mixtral-shaped layer at 1 decode token with the gate/down
    matrices in pinned host memory.  Resident in HBM: all quantized up projections (32 x 8 x 18.35 MB = 4.7 GB),
    routers, one staging slab per (token, slot).  Per layer the selected [gate|down] chunks of the two routed
    experts are pulled over the bus on a side stream (floe_moe_layer_decode_offloaded).  The 32 layer slots alias
    a pool of `--copies` distinct pinned layers (60 GB of pinned memory would be needed otherwise); bus traffic is
    not affected, nothing is cached on the way.  No attention exists here: between layers x <- y / std(y)."""
    n_layers, pool = 32, max(1, min(args.copies, 8))
    n_tok, n_warm = 5, 2
    wr = S.router_weights(SEED, 4, N_EXPERTS, D)
    wr_dev = torch.from_numpy(wr).to(dev)
    t0 = time.time()
    base = []
    for e in range(N_EXPERTS):
        w_up, gd = S.expert_weights(SEED, 4, D, F_INT, 0, e)
        q = FL.floe_quantize_expert(torch.from_numpy(w_up).to(dev), BITS, GROUP)
        base.append((q, gd))
    log(f"[bench] generated and quantized 8 experts in {time.time() - t0:.1f}s")
    pinned = [[torch.from_numpy(base[e][1]).clone().pin_memory() for e in range(N_EXPERTS)] for _ in range(pool)]
    log(f"[bench] pinned {pool} layer copies ({pool * N_EXPERTS * base[0][1].nbytes / 1e9:.1f} GB)")
    # per-expert constant thresholds, calibrated offline on 16 N(0,1) tokens (Eq. 6 on a small sample)
    cal = torch.from_numpy(S.tokens(SEED, 4, 16, D, layer=7)).to(dev)
    z = -(-16 * F_INT * PCT // 100)
    tau_e = torch.empty((N_EXPERTS,), dtype=torch.float32, device=dev)
    for e in range(N_EXPERTS):
        v = FL.floe_up_gemv(*base[e][0], cal, D, BITS, GROUP)
        tau_e[e] = torch.kthvalue(v.abs().flatten(), z).values
    layers = []
    for l in range(n_layers):
        experts = []
        for e in range(N_EXPERTS):
            c, s_, zz = (t.clone() for t in base[e][0])
            experts.append(FL.Expert(D, F_INT, BITS, GROUP, c, s_, zz, pinned[l % pool][e]))
        layers.append(FL.Layer(experts, 0, TOP_K, True, wr_dev.clone(), tau_e, False, gd_on_host=True))
    # resident twins of the layers for the VRAM-budget sweep (Sec. 4.2: more memory = more layers kept whole in HBM);
    # they alias a small pool of device copies: 4 x 1.88 GB is beyond any cache, HBM reads are what they would be
    pool_dev = 4
    gd_dev = [[torch.from_numpy(base[e][1]).to(dev) for e in range(N_EXPERTS)] for _ in range(pool_dev)]
    layers_res = []
    for l in range(n_layers):
        ex = layers[l].experts
        experts = [FL.Expert(D, F_INT, BITS, GROUP, ex[e].up_codes, ex[e].up_scale, ex[e].up_zero, gd_dev[l % pool_dev][e])
                   for e in range(N_EXPERTS)]
        layers_res.append(FL.Layer(experts, 0, TOP_K, True, layers[l].router_cm, tau_e, False))
    cap = 2048
    staging = torch.empty((TOP_K, cap, 2, D), dtype=torch.float16, device=dev)
    overflow = torch.zeros((TOP_K,), dtype=torch.int32, device=dev)
    stats = torch.zeros((n_layers, 1, TOP_K, 4), dtype=torch.int32, device=dev)
    side = torch.cuda.Stream()
    ev_a, ev_b = torch.cuda.Event(), torch.cuda.Event()
    ws = layers[0].workspace(1)
    ws_res = layers_res[0].workspace(1)
    y = torch.empty((1, D), dtype=torch.float16, device=dev)
    toks = torch.from_numpy(S.tokens(SEED, 4, n_tok + n_warm, D, layer=9)).to(dev)
    layer_gb = N_EXPERTS * F_INT * 2 * D * 2 / 1e9
    fixed_gb = (n_layers * N_EXPERTS * (D * F_INT * BITS // 8 + 4 * F_INT * (D // GROUP)) + staging.numel() * 2) / 1e9

    def run(n_res):
        """n_res leading layers resident, the rest offloaded; returns (ms per token, staged bytes per token, overflows)"""
        lat, staged, ovf = [], [], 0
        for i in range(n_tok + n_warm):
            x = toks[i:i + 1].contiguous()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for l in range(n_layers):
                if l < n_res:
                    FL.floe_moe_layer_decode(layers_res[l], x, y, stats[l], ws_res)
                else:
                    FL.floe_moe_layer_decode_offloaded(layers[l], x, staging, cap, side, ev_a, ev_b, y=y, stats=stats[l],
                                                       overflow=overflow, workspace=ws)
                yf = y.float()
                x = (yf / yf.std()).half()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            ovf += int(overflow.sum().item())
            if i >= n_warm:
                lat.append(dt)
                ks = stats.cpu().numpy().reshape(n_layers, TOP_K, 4)[n_res:, :, 1]
                staged.append(int(np.minimum(ks, cap).sum()) * 4 * D)
        return float(np.median(lat)) * 1e3, float(np.mean(staged)), ovf   # median: a token that touches host pages for the first time pays for it once

    parts = set(args.stack_parts.split(","))
    ms, nbytes, ovf = run(0) if "plain" in parts else (float("nan"), 0.0, 0)
    sweep = []
    for budget in (12, 16, 20, 24, 32, 48, 66) if "budget" in parts else ():
        n_res = int(max(0, min(n_layers, (budget - fixed_gb) // layer_gb)))
        b_ms, b_bytes, _ = run(n_res)
        sweep.append({"vram_budget_GB": budget, "resident_layers": n_res, "ms_per_token": round(b_ms, 3),
                      "tokens_per_s": round(1e3 / b_ms, 1), "staged_MB_per_token": round(b_bytes / 1e6, 1)})
        log(f"[bench] budget {budget} GB: {n_res} layers resident, {b_ms:.2f} ms/token, {b_bytes / 1e6:.0f} MB staged")
    # ---- the same budgets spent on resident CHANNELS instead of whole layers: per expert the channels that the
    # calibration tokens selected most often stay in HBM (a policy of this harness; the paper names none), every layer
    # keeps the same share, and a token copies only the selected channels that are not resident
    cal_counts = []
    for e in range(N_EXPERTS):
        vcal = FL.floe_up_gemv(*base[e][0], cal, D, BITS, GROUP)
        cal_counts.append((vcal.abs() > tau_e[e]).sum(dim=0))
    M_cache = FL.MissPath(torch.cuda.Stream(), TOP_K, dev)
    cstats = torch.zeros((n_layers, TOP_K, 4), dtype=torch.int32, device=dev)
    cache_sweep = []
    for budget in (12, 16, 20, 24, 32, 48) if "cache" in parts else ():
        share = max(0.0, min(1.0, (budget - fixed_gb) / (n_layers * layer_gb)))
        r_per = int(share * F_INT)
        caches = []
        for p_ in range(pool):                     # one cache per distinct pinned layer (the 32 slots alias them)
            c = FL.ChannelCache(layers[p_], 1, N_EXPERTS * r_per, cap)
            for e in range(N_EXPERTS):
                if r_per == 0:
                    break
                hot = torch.argsort(cal_counts[e], descending=True, stable=True)[:r_per].sort().values.to(torch.int32).contiguous()
                cnt = torch.tensor([r_per], dtype=torch.int32, device=dev)
                FL.floe_channel_cache_load(layers[p_], c, e, hot, cnt, e * r_per, r_per)
            caches.append(c)
        torch.cuda.synchronize()
        lat, staged_b, hits, total = [], [], 0, 0
        for i in range(n_tok + n_warm):
            x = toks[i:i + 1].contiguous()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for l in range(n_layers):
                FL.floe_moe_layer_decode_cached(layers[l], caches[l % pool], M_cache, x, y=y, stats=stats[l],
                                                cache_stats=cstats[l], workspace=ws)
                yf = y.float()
                x = (yf / yf.std()).half()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            if i >= n_warm:
                lat.append(dt)
                rec = stats.cpu().numpy().reshape(n_layers, TOP_K, 4)
                staged_b.append(int(rec[:, :, 3].sum()) * 4 * D)
                hits += int(cstats.cpu().numpy().reshape(n_layers, TOP_K, 4)[:, :, 2].sum())
                total += int(rec[:, :, 1].sum())
        row = {"vram_budget_GB": budget, "resident_share_of_channels": round(share, 3), "ms_per_token": round(float(np.median(lat)) * 1e3, 3),
               "staged_MB_per_token": round(float(np.mean(staged_b)) / 1e6, 1), "hit_rate": round(hits / max(total, 1), 3)}
        cache_sweep.append(row)
        log(f"[bench] channel cache, budget {budget} GB: {row}")
        del caches
    # ---- prefetch of the next layer from the current hidden state (intra-expert reuse, Sec. 3.3).  Hidden states of
    # neighbouring layers are made alike on purpose: x_{l+1} = (x_l + beta * y_l / std(y_l)) / std(...), which gives a
    # cosine similarity of about 1 / sqrt(1 + beta^2) (0.95 at beta = 0.33; the paper reports > 0.95 on Mixtral).
    pre_stream, miss_stream = torch.cuda.Stream(), torch.cuda.Stream()
    P2 = [FL.Prefetch(layers[0], 1, cap, pre_stream), FL.Prefetch(layers[0], 1, cap, pre_stream)]
    M = FL.MissPath(miss_stream, TOP_K, dev)
    ws_pre = layers[0].new_workspace(1)
    pstats = torch.zeros((n_layers, TOP_K, 4), dtype=torch.int32, device=dev)
    def run_prefetch(beta, extra):
        lat, cosines, agg = [], [], np.zeros(5)
        all_rows = torch.zeros((), dtype=torch.int64, device=dev)      # every row the prefetches copied, used or not
        for i in range(-extra, n_tok + n_warm):
            i = max(i, 0)
            x = toks[i:i + 1].contiguous()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            FL.floe_moe_layer_prefetch(layers[0], P2[0], x, ws_pre)
            for l in range(n_layers):
                if l + 1 < n_layers:
                    FL.floe_moe_layer_prefetch(layers[l + 1], P2[(l + 1) % 2], x, ws_pre)
                FL.floe_moe_layer_decode_prefetched(layers[l], P2[l % 2], M, x, y=y, stats=stats[l],
                                                    prefetch_stats=pstats[l], workspace=ws)
                if i >= n_warm:
                    all_rows += P2[l % 2].pred_count.clamp(max=cap).sum()
                xf, yf = x.float(), y.float()
                xn = xf + beta * yf / yf.std()
                xn = xn / xn.std()
                if i >= n_warm:
                    cosines.append(torch.nn.functional.cosine_similarity(xf, xn).reshape(()))
                x = xn.half()
            torch.cuda.synchronize()
            if i >= n_warm:
                lat.append(time.perf_counter() - t1)
                ps = pstats.cpu().numpy().reshape(n_layers, TOP_K, 4)[1:]        # layer 0 is predicted from its own input
                agg += np.array([ps[..., 0].sum(), ps[..., 1].sum(), ps[..., 2].sum(), ps[..., 3].sum(), ps[..., 0].size])
        hits, misses, predicted = agg[2], agg[3], agg[1]
        copied = (float(all_rows.item()) + misses) / n_tok * 4 * D
        row = {"beta": beta, "cosine_similarity": round(float(torch.stack(cosines).mean().item()), 4),
               "expert_prediction_rate": round(float(agg[0] / agg[4]), 4),
               "channel_recall": round(float(hits / max(hits + misses, 1)), 4),
               "channel_precision": round(float(hits / max(predicted, 1)), 4),
               "ms_per_token": round(float(np.median(lat)) * 1e3, 3),
               "prefetched_MB_per_token": round(float(all_rows.item()) / n_tok * 4 * D / 1e6, 1),
               "prefetched_for_the_right_expert_MB_per_token": round(float(predicted) / n_tok * 4 * D / 1e6, 1),
               "missed_MB_per_token": round(float(misses) / n_tok * 4 * D / 1e6, 1),
               "copied_MB_per_token": round(float(copied) / 1e6, 1),
               "link_GBps": round(float(copied) / float(np.median(lat)) / 1e9, 2)}
        return row, lat

    prefetch_rows = []
    first = True
    for beta in (0.33, 0.2) if "prefetch" in parts else ():
        row, lat = run_prefetch(beta, 4 if first else 0)    # the first pass also warms the spare slabs and both streams
        first = False
        prefetch_rows.append(row)
        log(f"[bench] prefetch: {row} per-token ms {[round(v * 1e3, 1) for v in lat]}")
    # ---- how many copy workgroups: host reads in flight beyond what the link needs delay the HBM reads of the kernels
    # that run beside the copy (the up GEMV of the layer being decoded while the next layer is prefetched)
    wg_sweep = []
    for wgs in (256, 128, 64, 32, 16, 8) if "copywgs" in parts else ():
        FL.floe_tuning(FL.TUNE_STAGE_WORKGROUPS, wgs)
        p_ms, _, _ = run(0)
        row, _ = run_prefetch(0.33, 4 if first else 0)
        first = False
        wg_sweep.append({"copy_workgroups": wgs, "plain_ms_per_token": round(p_ms, 3), "prefetch_ms_per_token": row["ms_per_token"]})
        log(f"[bench] copy workgroups {wgs}: plain {p_ms:.2f} ms/token, prefetched (beta 0.33) {row['ms_per_token']:.2f} ms/token")
    FL.floe_tuning(FL.TUNE_STAGE_WORKGROUPS, 0)

    # plain pinned copy of the same volume for reference
    flat = pinned[0][0].view(-1)
    dflat = torch.empty((flat.numel(),), dtype=torch.float16, device=dev)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(4):
        dflat.copy_(flat, non_blocking=True)
    torch.cuda.synchronize()
    peak = 4 * flat.numel() * 2 / (time.perf_counter() - t1) / 1e9
    print(json.dumps({"metric": "ms per decode token, 32 offloaded MoE layers (selected channels streamed host->HBM)",
                      "value": round(ms, 3), "unit": "ms", "n_gpus": 1, "higher_is_better": False, "data": "synthetic",
                      "config": {"workload": "BASELINE configs[3]: 32 x (8 experts d=4096 f=14336, INT2 g64, top-2), gate/down "
                                             "in pinned host memory, per-expert constant thresholds for 90 % sparsity, 1 token",
                                 "pinned_layer_pool": pool, "staging_capacity_rows": cap, "tokens_timed": n_tok, "statistic": "median over the timed tokens",
                                 "overflowed_lists": ovf},
                      "staged_bytes_per_token": int(nbytes), "staged_GBps": round(nbytes / (ms * 1e-3) / 1e9, 2),
                      "pinned_memcpy_GBps": round(peak, 2), "tokens_per_s": round(1e3 / ms, 2),
                      "resident_hbm_GB": round(fixed_gb, 2),
                      "vram_budget_sweep": sweep, "resident_channel_cache_sweep": cache_sweep,
                      "prefetch_next_layer": prefetch_rows, "copy_workgroups_sweep": wg_sweep}), flush=True)


def bench_batch(args, np, torch, S, FL, dev):
    """Decode batches (each token routed on its own, own thresholds): BASELINE configs[2] at T = 1, 4, 16 and
    configs[4] (64 routed + 2 shared experts, d=2048, f=1408, INT3 group 32, top-6, 85 %) at T = 1, 8, 32.
    Per-expert constant thresholds calibrated on 8 tokens; one layer copy (what a call touches beyond T = 1 is larger
    than the last-level cache anyway).  Fractions are over the algorithmic bytes: rows counted once per expert."""
    K, W = max(20, args.steps // 4), max(5, args.warmup // 8)
    out = []

    def make_layer(cfg, d, f, bits, group, n, n_shared, top_k, renorm, pct):
        experts = []
        for e in range(n + n_shared):
            w_up, gd = S.expert_weights(SEED, cfg, d, f, 0, e)
            c, s_, z = FL.floe_quantize_expert(torch.from_numpy(w_up).to(dev), bits, group)
            experts.append(FL.Expert(d, f, bits, group, c, s_, z, torch.from_numpy(gd).to(dev)))
        wr = torch.from_numpy(S.router_weights(SEED, cfg, n, d)).to(dev)
        cal = torch.from_numpy(S.tokens(SEED, cfg, 8, d, layer=7)).to(dev)
        tau = torch.empty((n + n_shared,), dtype=torch.float32, device=dev)
        zq = -(-8 * f * pct // 100)
        for e in range(n + n_shared):
            v = FL.floe_up_gemv(experts[e].up_codes, experts[e].up_scale, experts[e].up_zero, cal, d, bits, group)
            tau[e] = torch.kthvalue(v.abs().flatten(), zq).values
        return FL.Layer(experts, n_shared, top_k, renorm, wr, tau, False)

    stream = torch.cuda.Stream()
    for name, cfg, d, f, bits, group, n, n_shared, top_k, renorm, pct, Ts in (
            ("configs[2]", 3, 4096, 14336, 2, 64, 8, 0, 2, True, 90, (1, 4, 16, 64)),
            ("configs[4]", 5, 2048, 1408, 3, 32, 64, 2, 6, False, 85, (1, 8, 32, 128))):
        want = [c.split(":") for c in args.batch_cases.split(",") if c]
        if want:  # any batch size may be asked for, not only the ones of the default run
            Ts = sorted({int(t) for c, t in want if c == name[8]})
        if not Ts:
            continue
        L = make_layer(cfg, d, f, bits, group, n, n_shared, top_k, renorm, pct)
        for T in Ts:
            x = torch.from_numpy(S.tokens(SEED, cfg, T, d, layer=9)).to(dev)
            y = torch.empty((T, d), dtype=torch.float16, device=dev)
            slots = top_k + n_shared
            st = torch.zeros((T, slots, 4), dtype=torch.int32, device=dev)
            FL.floe_moe_layer_decode(L, x, y, st)
            torch.cuda.synchronize()
            rec = st.cpu().numpy().reshape(T * slots, 4)
            sp = {}
            ms = _graph_time(torch, stream, lambda i: FL.floe_moe_layer_decode(L, x, y), K, W, reps=5, spread=sp)
            # Algorithmic bytes of the call: the codes, scales and zeros of every expert that is used, once; per expert
            # the [gate | down] chunks of the UNION of the channels its tokens select, once (a row serves every token
            # whose mask holds it); router, x, y.  The unions come from this run's own routing (stats) and the masks
            # |v| > tau of the same tokens (dense v per expert from floe_up_gemv: harness work, not timed).
            codes_meta = d * f * bits // 8 + 4 * f * (d // group)
            by_expert = {}
            for q in range(T * slots):
                by_expert.setdefault(int(rec[q, 0]), []).append(q // slots)
            union_rows = 0
            for e, toks in by_expert.items():
                ex = L.experts[e]
                v = FL.floe_up_gemv(ex.up_codes, ex.up_scale, ex.up_zero, x[toks].contiguous(), d, bits, group)
                union_rows += int(((v.abs() > L.tau[e]).any(dim=0)).sum().item())
            used = len(by_expert)
            requested_rows = int(rec[:, 1].sum())
            fixed = used * codes_meta + n * d * 2 + T * d * 2 * 2
            nbytes = fixed + union_rows * 4 * d
            out.append({"config": name, "T": T, "us_per_layer_call": round(ms * 1e3, 2), "us_per_layer_token": round(ms * 1e3 / T, 2),
                        "us_per_layer_call_median_p10_p90": [round(sp[k] * 1e3, 2) for k in ("median", "p10", "p90")],
                        "experts_used": used, "rows_union": union_rows, "rows_requested": requested_rows,
                        "algorithmic_bytes": int(nbytes), "bytes_requested": int(fixed + requested_rows * 4 * d),
                        "GBps": round(nbytes / ms / 1e6, 1), "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)})
            log(f"[bench] {name} T={T}: {ms * 1e3:.1f} us per layer call, {ms * 1e3 / T:.2f} us per layer-token, "
                f"{out[-1]['GBps']} GB/s over {nbytes / 1e6:.0f} MB (union of selected rows per expert; "
                f"{(fixed + requested_rows * 4 * d) / 1e6:.0f} MB if every (token, slot) read its own rows)")
        del L
    print(json.dumps({"metric": "us per MoE layer-token for decode batches", "value": out[0]["us_per_layer_token"], "unit": "us",
                      "n_gpus": 1, "higher_is_better": False, "data": "synthetic",
                      "config": {"workload": "BASELINE configs[2] (T=1,4,16,64) and configs[4] (T=1,8,32,128), one layer replayed (weights may sit in the last-level cache), HIP-graph replay"},
                      "results": out}), flush=True)


if __name__ == "__main__":
    main()
