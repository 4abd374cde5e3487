#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic batch of the GPT-MoE-350M-shaped
configuration (d_model 1024, d_ff 4096, 8 experts, top-1, 8192 tokens, bf16, fp32 accumulation):
gate+top-k -> dispatch -> grouped expert FFN -> combine (bf16: index-only dispatch and
moe_expert_ffn_fused), and the affinity statistic (co-routing counts, loads, conditional
probabilities and the locality numerators of a placement: affinity_statistics, one pass) over the
configuration's 12-layer x 8192-token routing trace.
Inputs are resident in HBM before the timed region; no allocation happens inside it.

`--config N` times another of the five workload configurations the same way (the decode-shaped
one runs its 8 consecutive layers per step and reports the weight-streaming HBM roofline).

Prints ONE JSON line: tokens/s of the whole step (mean of the K timed steps, which follow a fixed
0.3 s of untimed steps and the caller's W; the median and minimum over per-step event pairs beside
it), the roofline of the dominant kernel (the grouped expert GEMM, measured with HIP events on the
launch stream; its HBM-side bytes come from the tracked profile summary), per-entry-point timings
(median / mean / minimum), the HBM-bound entry points at the larger shapes of the one-GPU-share
configuration (rotated over buffer sets larger than the 256 MB cache, and un-rotated), the expert
FFN of the three larger configurations, the copy, MFMA and vendor-GEMM rates of the box, the
placement search with the communication volumes of the paper's comparison table, and the CPU oracle
timed on all host threads and on one.

`--sections` runs a part of this (profiling runs use it so that every kernel appears at one shape
only); `--timeline` prints where the time of the grouped GEMM's workgroups goes instead.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

WARM_SECONDS = 0.3          # steps run before the caller's --warmup, so that the clocks are up whatever W is

# HBM-side bytes per moe_expert_ffn_fused call at the benchmark configuration come from a tracked
# rocprofv3 summary (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for
# the 1 GiB copy probe); the file records the commit it was taken at.  Missing or unreadable: null.
FFN_TRAFFIC_FILE = os.path.join(ROOT, "profiles", "ffn_config2_hbm_traffic.txt")


def ffn_traffic_from_profile():
    """(bytes per call, commit the profile was taken at) from the tracked summary, or (None, None)."""
    try:
        text = open(FFN_TRAFFIC_FILE).read()
    except OSError:
        return None, None
    val = head = None
    for line in text.splitlines():
        if line.startswith("traffic_bytes_per_call:"):
            val = int(float(line.split(":", 1)[1].split()[0]))
        if line.startswith("head:"):
            head = line.split(":", 1)[1].strip()
    return val, head


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _time_call(fn, iters, warmup=3):
    """Average milliseconds of `fn` (enqueued on the current stream) over `iters` launches."""
    import torch
    for _ in range(warmup):
        fn()
    a, b = _events(2)
    torch.cuda.synchronize()
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def _time_groups(fns, groups=12, inner=5, warmup=10):
    """Milliseconds per call of the calls in `fns`, cycled through in order (one buffer set per entry:
    several entries whose buffers together exceed the 256 MB Infinity Cache give the rotated figure, one
    entry the un-rotated one).  `groups` event pairs bracket `inner` calls each; returns mean, median
    and min over the groups."""
    import torch
    n = len(fns)
    for i in range(max(warmup, n)):
        fns[i % n]()
    ev = [_events(2) for _ in range(groups)]
    torch.cuda.synchronize()
    c = 0
    for g in range(groups):
        ev[g][0].record()
        for _ in range(inner):
            fns[c % n]()
            c += 1
        ev[g][1].record()
    torch.cuda.synchronize()
    t = np.array([a.elapsed_time(b) / inner for a, b in ev])
    return {"ms": float(t.mean()), "ms_median": float(np.median(t)), "ms_min": float(t.min())}


def _hbm_entry(make_fn, n_sets, nbytes, extra=None):
    """One HBM-bound call: rotated over `n_sets` buffer sets and un-rotated (set 0 only)."""
    rot = _time_groups([make_fn(i) for i in range(n_sets)])
    same = _time_groups([make_fn(0)])
    gbs = nbytes / (rot["ms_median"] * 1e-3) / 1e9
    out = {"ms": rot["ms_median"], "ms_mean": rot["ms"], "ms_min": rot["ms_min"], "GBps": gbs, "frac": gbs / PEAK_HBM_GBS, "bytes": nbytes,
           "unrotated_ms": same["ms_median"], "unrotated_ms_min": same["ms_min"],
           "unrotated_GBps": nbytes / (same["ms_median"] * 1e-3) / 1e9,
           "unrotated_frac": nbytes / (same["ms_median"] * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if extra:
        out.update(extra(rot["ms_median"]))
    return out


def _set_oracle_threads(n):
    """Thread count of the oracle's OpenMP loops (the GNU OpenMP runtime the oracle is linked with)."""
    import ctypes
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def cpu_baseline(cfg, x, wg, w1, w2, trace, placement, sample_rows_per_expert=None):
    """The CPU oracle as it stands, timed on this host: every step in full except the expert
    FFN, which runs on a sample of rows of every expert and is extrapolated linearly."""
    import oracle
    oracle.build()
    t = {}
    t0 = time.perf_counter()
    logits = oracle.gate_logits(x, wg)
    idx, w = oracle.topk(logits, cfg.k, cfg.renormalize)
    t["gate"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    disp = oracle.dispatch(idx, None, cfg.E, cfg.E_local)
    xs = oracle.gather_rows(x, disp["src_of_sorted"], cfg.k)
    t["dispatch"] = time.perf_counter() - t0
    rows = []
    for e in range(cfg.E_local):
        lo, hi = int(disp["offsets"][e]), int(disp["offsets"][e + 1])
        rows.extend(range(lo, hi if sample_rows_per_expert is None else min(hi, lo + sample_rows_per_expert)))
    rows = np.array(rows, dtype=np.int64)
    t0 = time.perf_counter()
    y = oracle.expert_ffn_rows(xs, disp["offsets"], w1, None, w2, None, 0, rows)
    t_ffn_sample = time.perf_counter() - t0
    t["ffn"] = t_ffn_sample * (disp["kept"] / max(len(rows), 1))
    y_full = np.zeros((disp["kept"], cfg.d))
    y_full[rows] = y
    t0 = time.perf_counter()
    oracle.combine(y_full, disp["sorted_of_src"], w)
    t["combine"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    counts, loads, _ = oracle.affinity_counts(trace, cfg.trace_E)
    oracle.cond_prob(counts)
    t["affinity"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.placement_locality(trace, placement)
    t["locality"] = time.perf_counter() - t0
    total = sum(t.values())
    return {
        "value": cfg.T / total,
        "unit": "tokens/s",
        "cores": oracle.threads(),
        "kind": "oracle",
        "sample": (f"one full step of the benchmark workload (all {disp['kept']} rows through the expert FFN, "
                   f"{t_ffn_sample:.2f} s of the total)") if len(rows) == disp["kept"] else
                  (f"expert FFN on {len(rows)} of {disp['kept']} rows (measured {t_ffn_sample:.2f} s, extrapolated linearly); "
                   f"gate, dispatch, combine, affinity, locality in full"),
        "seconds_per_step_extrapolated": total,
        "seconds": {k: round(v, 4) for k, v in t.items()},
    }


def cpu_baseline_single_thread(cfg, x, wg, w1, w2, rows_per_expert=4):
    """The same oracle on ONE thread, on a bounded sample: the gate in full, the expert FFN (which is
    all but a fraction of a percent of the step) on `rows_per_expert` rows of every expert,
    extrapolated linearly; the other steps are taken from the full run (they are single-threaded
    loops or negligible)."""
    import oracle
    _set_oracle_threads(1)
    try:
        t0 = time.perf_counter()
        logits = oracle.gate_logits(x, wg)
        idx, _ = oracle.topk(logits, cfg.k, cfg.renormalize)
        t_gate = time.perf_counter() - t0
        disp = oracle.dispatch(idx, None, cfg.E, cfg.E_local)
        xs = oracle.gather_rows(x, disp["src_of_sorted"], cfg.k)
        rows = []
        for e in range(cfg.E_local):
            lo, hi = int(disp["offsets"][e]), int(disp["offsets"][e + 1])
            rows.extend(range(lo, min(hi, lo + rows_per_expert)))
        rows = np.array(rows, dtype=np.int64)
        t0 = time.perf_counter()
        oracle.expert_ffn_rows(xs, disp["offsets"], w1, None, w2, None, 0, rows)
        t_ffn = time.perf_counter() - t0
    finally:
        _set_oracle_threads(oracle.threads())
    total = t_gate + t_ffn * disp["kept"] / max(len(rows), 1)
    return {"value": cfg.T / total, "unit": "tokens/s", "cores": 1,
            "sample": f"gate in full ({t_gate:.2f} s), expert FFN on {len(rows)} of {disp['kept']} rows ({t_ffn:.2f} s, extrapolated linearly)"}


def other_configs(syn, torch, MoELayerRun, dev):
    """Expert FFN (moe_expert_ffn_fused) and whole-layer time of the three larger configurations, each
    against the roofline that bounds it.  Expert weights are drawn on the device (same distribution as
    the host recipe, torch's generator); the decode-shaped configuration runs ONE layer's distinct
    weights repeatedly - 17 GB per pass, far beyond any cache, so the timing is that of distinct layers."""
    out = {}
    for index in (3, 4, 5):
        c = syn.CONFIGS[index]
        x = torch.from_numpy(syn.tokens(c)).to(torch.bfloat16).to(dev)
        wg = torch.from_numpy(syn.gate_weight(c)).to(torch.bfloat16).to(dev)
        w1, w2 = syn.device_expert_weights(c, 0, dev)
        kw = {}
        if index == 3:
            tr3, _ = syn.config_trace(c)
            kw["topk_idx"] = torch.from_numpy(tr3[0].reshape(-1, 1).copy()).to(dev)
        if index == 4:
            idx4_h, map4_h = syn.local_routing(c, syn.seed_for(4, 4, 1))
            kw["topk_idx"] = torch.from_numpy(idx4_h).to(dev)
            kw["expert_map"] = torch.from_numpy(map4_h).to(dev)
        run = MoELayerRun(x, wg, w1, w2, c.k, c.renormalize, fused=True, **kw)
        run.step()
        torch.cuda.synchronize()
        t_w = time.perf_counter()  # the same fixed warm-up as the benchmark step: clocks and caches settle
        while time.perf_counter() - t_w < WARM_SECONDS:
            for _ in range(4):
                run.step()
            torch.cuda.synchronize()
        ffn = _time_groups([run.ffn], groups=10, inner=4, warmup=4)
        layer = _time_groups([run.step], groups=10, inner=4, warmup=4)
        A = c.T * c.k
        flops = 4.0 * A * c.d * c.f
        entry = {"workload": c.name, "tokens": c.T, "d_model": c.d, "d_ff": c.f, "local_experts": c.E_local, "top_k": c.k,
                 "ffn_ms": ffn["ms_median"], "ffn_ms_min": ffn["ms_min"], "layer_ms": layer["ms_median"],
                 "layer_tokens_per_s": c.T / (layer["ms_median"] * 1e-3), "weights": "drawn on the device, N(0, 0.02)"}
        if index == 5:
            nbytes = 2.0 * c.E_local * c.d * c.f * 2 + 2.0 * A * c.d * 2
            gbs = nbytes / (ffn["ms_median"] * 1e-3) / 1e9
            entry.update({"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                          "bytes_per_call": nbytes, "layers": "one layer's weights, repeated (the 8 layers of a step alias it here)"})
        else:
            tf = flops / (ffn["ms_median"] * 1e-3) / 1e12
            entry.update({"bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS,
                          "flops_per_call": flops})
        out[f"config{index}"] = entry
        del run, x, wg, w1, w2
        torch.cuda.empty_cache()
    return out


def timeline_report(syn, torch, B, index, dev):
    """Where the time of the grouped GEMM's workgroups goes at one configuration (exf_probe_ffn_timeline):
    per launch the span from the first workgroup's start to the last one's end, per tile kind the phases
    of a workgroup (tile lookup, arrival of the first K tile, K loop, epilogue), the busy time of the
    compute units, and the gap between the two launches.  Plain text, one fact per line."""
    import ctypes
    c = syn.CONFIGS[index]
    lib = B.lib()
    x = torch.from_numpy(syn.tokens(c)).to(torch.bfloat16).to(dev)
    wg = torch.from_numpy(syn.gate_weight(c)).to(torch.bfloat16).to(dev)
    w1, w2 = syn.device_expert_weights(c, 0, dev)
    emap = None
    if index == 3:
        tr3, _ = syn.config_trace(c)
        idx = torch.from_numpy(tr3[0].reshape(-1, 1).copy()).to(dev)
        w = torch.rand((c.T, 1), device=dev)
    elif index == 4:
        i4, m4 = syn.local_routing(c, syn.seed_for(4, 4, 1))
        idx, emap = torch.from_numpy(i4).to(dev), torch.from_numpy(m4).to(dev)
        w = torch.rand((c.T, 1), device=dev)
    else:
        idx, w, _ = B.moe_gate_topk(x, wg, c.k, c.renormalize)
    disp = B.moe_dispatch(x, idx, c.E, E_local=c.E_local, expert_map=emap, gather=False)
    ws = torch.empty(lib.moe_expert_ffn_fused_workspace_bytes(c.T, c.k, c.d, c.f, c.E_local, B.EXF_BF16), dtype=torch.uint8, device=dev)
    out = torch.empty((c.T, c.d), dtype=torch.bfloat16, device=dev)
    cap = 16384
    tl = torch.zeros((2, cap, 8), dtype=torch.int64, device=dev)
    args = (x.data_ptr(), disp.src_of_sorted.data_ptr(), disp.sorted_of_src.data_ptr(), w.data_ptr(), disp.expert_offsets.data_ptr(),
            w1.data_ptr(), w2.data_ptr(), c.T, c.k, c.d, c.f, c.E_local, out.data_ptr(), ws.data_ptr(), ws.numel(), tl.data_ptr(), cap,
            B._stream())
    ms = _time_groups([lambda: B._check(lib.exf_probe_ffn_timeline(*args))], groups=6, inner=5, warmup=20)
    t = tl.cpu().numpy()
    us = 0.01  # the device clock of the records ticks at 100 MHz
    print(f"timeline of moe_expert_ffn_fused, {c.name}: T={c.T} d={c.d} f={c.f} E_local={c.E_local} k={c.k}; "
          f"rows per expert {disp.expert_counts.cpu().numpy().tolist()}")
    print(f"call: {ms['ms_median'] * 1e3:.1f} us median, {ms['ms_min'] * 1e3:.1f} us min (back to back, timeline recording on)")
    spans = []
    for which, name in ((0, "first contraction"), (1, "second contraction")):
        r = t[which]
        ran = (r[:, 4] > 0) & (r[:, 1] > 0)
        if not ran.any():
            print(f"{name}: no record")
            continue
        t0, t1 = r[ran, 0].min(), r[ran, 4].max()
        spans.append((t0, t1))
        print(f"{name}: {int(ran.sum())} workgroups ran a tile, first start to last end {(t1 - t0) * us:.1f} us")
        kind = r[:, 6] & 3
        for kd, kn in ((2, "tall"), (0, "full"), (1, "remainder")):
            m = ran & (kind == kd)
            if not m.any():
                continue
            nk = np.unique((r[m, 6] >> 48) & 0xffff).tolist()
            ph = {"row ranges": r[m, 7] - r[m, 0], "lookup": r[m, 1] - r[m, 0], "first K tile": r[m, 2] - r[m, 1], "K loop": r[m, 3] - r[m, 2], "epilogue": r[m, 4] - r[m, 3],
                  "total": r[m, 4] - r[m, 0]}
            print(f"  {kn} tiles: {int(m.sum())}, K tiles per work item {nk}, starts {(r[m, 0].min() - t0) * us:.1f}..{(r[m, 0].max() - t0) * us:.1f} us, "
                  f"ends {(r[m, 4].min() - t0) * us:.1f}..{(r[m, 4].max() - t0) * us:.1f} us")
            for pn, v in ph.items():
                v = v * us
                print(f"    {pn:13s} mean {v.mean():6.2f}  p10 {np.percentile(v, 10):6.2f}  median {np.median(v):6.2f}  p90 {np.percentile(v, 90):6.2f}  max {v.max():6.2f} us")
        hw = r[:, 5]
        cu = (hw >> 32) * 4096 + ((hw >> 13) & 7) * 256 + ((hw >> 8) & 15)  # XCD, shader engine, compute unit
        keys = np.unique(cu[ran])
        busy = np.array([((r[ran & (cu == k), 4] - r[ran & (cu == k), 0]).sum() * us, (r[ran & (cu == k), 4].max() - t0) * us) for k in keys])
        print(f"  compute units seen {len(keys)}; busy per unit mean {busy[:, 0].mean():.1f} max {busy[:, 0].max():.1f} us; "
              f"last end per unit min {busy[:, 1].min():.1f} mean {busy[:, 1].mean():.1f} max {busy[:, 1].max():.1f} us")
    if len(spans) == 2:
        print(f"gap between the launches (last end of the first to first start of the second): {(spans[1][0] - spans[0][1]) * us:.2f} us; "
              f"first start to last end of both: {(spans[1][1] - spans[0][0]) * us:.1f} us")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="workload configuration (default 2: the one the headline metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--timeline", action="store_true",
                    help="print the per-workgroup phase timeline of the grouped GEMM at --config (text) instead of the benchmark line")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-kernel and large-shape measurements")
    ap.add_argument("--sections", default="all",
                    help="comma list of what to run: step (the timed steps), per_call, box, hbm4 (the HBM-bound calls, the placement "
                         "search and the transfer counters at the shapes of the one-GPU-share configuration), other (the larger "
                         "configurations), search (placement search, transfer ratios, multi-hop statistic), cpu; default all.  "
                         "Profiling runs pick one so that every kernel appears at one shape only")
    ap.add_argument("--hbm4-calls", default="all",
                    help="comma list of the calls the hbm4 section times (dispatch, combine, gate, affinity_histogram, "
                         "placement_locality, affinity_statistics, routing_transfers); default all")
    ap.add_argument("--unfused", action="store_true",
                    help="sorted copies of the activations and a separate combine pass "
                         "(moe_expert_ffn + moe_combine) instead of moe_expert_ffn_fused")
    ap.add_argument("--two-pass-affinity", action="store_true",
                    help="affinity_histogram + placement_locality (two passes over the trace) instead of affinity_statistics")
    ap.add_argument("--overlap", action="store_true",
                    help="run the affinity statistic on a second stream beside the layer (forked and joined every step) "
                         "instead of on the layer's stream")
    args = ap.parse_args()
    sections = {"step", "per_call", "box", "hbm4", "search", "other", "cpu"} if args.sections == "all" else set(args.sections.split(","))
    want4 = (lambda name: True) if args.hbm4_calls == "all" else (lambda name: name in args.hbm4_calls.split(","))
    if args.no_extra:
        sections &= {"step", "cpu"}
    if args.no_cpu_baseline:
        sections.discard("cpu")
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported (no collectives, no sharding)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as syn
    from paper_2401_08383_amd import binding as B
    from paper_2401_08383_amd.pipeline import AffinityRun, MoELayerRun

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    lib = B.lib()
    if args.timeline:
        timeline_report(syn, torch, B, args.config, dev)
        return

    cfg = syn.CONFIGS[args.config]
    bf16 = cfg.dtype == "bf16"
    fused = not args.unfused

    def to_device(a):
        t = torch.from_numpy(a)
        return (t.to(torch.bfloat16) if bf16 else t).to(dev)

    # ---- the workload: one MoELayerRun per consecutive layer, plus the affinity part ------------
    layers = []
    host = None  # host copies of layer 0 for the CPU baseline (benchmark configuration only)
    for l in range(cfg.layers):
        x_h, wg_h = syn.tokens(cfg, l), syn.gate_weight(cfg, l)
        if cfg.index == 5:
            w1_d, w2_d = syn.device_expert_weights(cfg, l, dev)  # 17 GB per layer: drawn on the device
        else:
            w1_h, w2_h = syn.expert_weights(cfg, l)
            w1_d, w2_d = to_device(w1_h), to_device(w2_h)
            if l == 0 and cfg.index == 2:
                host = (x_h, wg_h, w1_h, w2_h)
        kwargs = {}
        if cfg.index == 3:  # trace-driven (Zipf) routing: layer-0 column of the trace
            tr3, _ = syn.config_trace(cfg)
            kwargs["topk_idx"] = torch.from_numpy(tr3[0].reshape(-1, 1).copy()).to(dev)
        if cfg.index == 4:  # this GPU's post-exchange share: 8 resident experts of 64
            idx4_h, map4_h = syn.local_routing(cfg, syn.seed_for(4, 4, 1))
            kwargs["topk_idx"] = torch.from_numpy(idx4_h).to(dev)
            kwargs["expert_map"] = torch.from_numpy(map4_h).to(dev)
        layers.append(MoELayerRun(to_device(x_h), to_device(wg_h), w1_d, w2_d, cfg.k, cfg.renormalize, fused=fused, **kwargs))
    layer = layers[0]
    aff = None
    if cfg.trace_L > 0:
        trace_h, _ = syn.config_trace(cfg)
        pl_h = syn.balanced_random_placement(cfg.trace_L, cfg.trace_E, cfg.G, syn.seed_for(cfg.index, 5))
        aff = AffinityRun(torch.from_numpy(trace_h).to(dev), torch.from_numpy(pl_h).to(dev), cfg.trace_E, cfg.G,
                          one_pass=not args.two_pass_affinity)

    # The affinity statistic reads a routing trace and nothing of the layer.  By default its two
    # launches go to the layer's stream; --overlap puts them on a second stream (default priority),
    # forked at the start of a step and joined at its end - measured slower at this configuration (the
    # two cross-stream waits cost more than the 10 us of statistic they hide).
    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream() if (aff is not None and args.overlap) else None

    def affinity_fork():
        if aff is None:
            return
        if side_stream is None:
            aff.step()
            return
        side_stream.wait_stream(main_stream)
        with torch.cuda.stream(side_stream):
            aff.step()

    def affinity_join():
        if side_stream is not None:
            main_stream.wait_stream(side_stream)

    def step():
        affinity_fork()
        for lay in layers:
            lay.step()
        affinity_join()

    ms_per_step, per_step, ffn_all, ffn_ms, n_internal = float("nan"), np.array([float("nan")]), np.array([float("nan")]), float("nan"), 0
    if "step" in sections:
        # fixed internal warm-up (clocks, caches, lazy module loads), then the caller's W steps
        step()
        torch.cuda.synchronize()
        t_w = time.perf_counter()
        n_internal = 1
        while time.perf_counter() - t_w < WARM_SECONDS:
            for _ in range(8):
                step()
            n_internal += 8
            torch.cuda.synchronize()
        for _ in range(args.warmup):
            step()
        ffn_ev = [[_events(2) for _ in layers] for _ in range(args.steps)]
        step_ev = _events(args.steps + 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_ev[i].record()
            affinity_fork()
            for j, lay in enumerate(layers):
                lay.gate()
                lay.dispatch()
                ffn_ev[i][j][0].record()
                lay.ffn()
                ffn_ev[i][j][1].record()
                lay.combine()
            affinity_join()
        step_ev[args.steps].record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ms_per_step = elapsed * 1e3 / args.steps
        per_step = np.array([step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(args.steps)])
        ffn_all = np.array([a.elapsed_time(b) for step_ev_ in ffn_ev for a, b in step_ev_])
        ffn_ms = float(ffn_all.mean())

    A = cfg.T * cfg.k
    ffn_flops = 4.0 * A * cfg.d * cfg.f
    elem = 2 if bf16 else 4
    achieved_tf = ffn_flops / (ffn_ms * 1e-3) / 1e12
    ffn_entry = "moe_expert_ffn_fused" if fused else "moe_expert_ffn"
    if cfg.index == 5:
        # weight-bandwidth bound: every expert that owns a row streams W1 and W2 once
        ffn_bytes = 2.0 * cfg.E_local * cfg.d * cfg.f * elem + 2.0 * A * cfg.d * elem
        achieved = ffn_bytes / (ffn_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": f"grouped_gemm_bf16_kernel ({ffn_entry}: both contractions)", "achieved": achieved,
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS, "traffic": None,
                    "ms_per_launch": ffn_ms, "bytes_per_launch": ffn_bytes}
    else:
        roofline = {"bound": "mfma", "kernel": f"grouped_gemm_bf16_kernel ({ffn_entry}: both contractions)"
                    if bf16 else f"grouped_gemm_f32_kernel ({ffn_entry}, fp32 vector ALU: latency-bound tiny case)",
                    "achieved": achieved_tf, "peak": PEAK_BF16_TFLOPS if bf16 else 157.3, "unit": "TFLOP/s",
                    "frac": achieved_tf / (PEAK_BF16_TFLOPS if bf16 else 157.3),
                    "traffic": None, "ms_per_launch": ffn_ms, "flops_per_launch": ffn_flops}
        if cfg.index == 2 and fused:
            roofline["traffic"], roofline["traffic_profile_head"] = ffn_traffic_from_profile()
    roofline["ms_per_launch_median"] = float(np.median(ffn_all))
    roofline["ms_per_launch_min"] = float(ffn_all.min())
    workloads = {
        1: "configs[0] tiny fp32: d_model=64 d_ff=256 E=8 top-1 T=512; 2-layer x 512-token trace",
        2: "configs[1] GPT-MoE-350M-shaped: d_model=1024 d_ff=4096 E=8 top-1 T=8192 bf16; affinity on a 12-layer x 8192-token "
           "trace, placement G=4",
        3: "configs[2] GPT-MoE-XL-shaped: d_model=2048 d_ff=8192 E=32 top-1 T=16384 bf16, Zipf(1.1) expert loads from the trace; "
           "12-layer x 16384-token trace, G=8",
        4: "configs[3] one GPU's share of E=64 (8 local experts): d_model=1024 d_ff=4096 T=32768 bf16; 24-layer x 1M-token trace, G=8",
        5: "configs[4] decode-shaped: d_model=4096 d_ff=16384 E=64 top-2 renormalised T=256 bf16, 8 consecutive layers with "
           "distinct weights (a step = all 8 layers)",
    }
    result = {
        "metric": "MoE-layer tokens/s (gate+dispatch+expert FFN+combine+affinity statistic per step)",
        "value": cfg.T * cfg.layers / (ms_per_step * 1e-3),  # token-layer passes per second (layers = 1 except for the decode shape)
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": float(np.median(per_step)),
        "ms_per_step_min": float(per_step.min()),
        "internal_warmup_steps": n_internal,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": workloads[cfg.index], "tokens": cfg.T, "d_model": cfg.d, "d_ff": cfg.f, "experts": cfg.E,
                   "local_experts": cfg.E_local, "top_k": cfg.k, "layers_per_step": cfg.layers, "trace_layers": cfg.trace_L,
                   "trace_tokens": cfg.trace_N, "ffn_entry": ffn_entry,
                   "affinity_entry": "affinity_histogram + placement_locality" if args.two_pass_affinity else "affinity_statistics"},
        "roofline": roofline,
    }
    achieved = achieved_tf

    if "per_call" in sections:
        # per-entry-point averages at the benchmark configuration
        per = {}
        calls = [("gate", layer.gate), ("dispatch", layer.dispatch), ("ffn", layer.ffn)]
        if not fused:
            calls.append(("combine", layer.combine))
        if aff is not None:
            calls += [("affinity_statistics", aff.statistics), ("affinity_histogram", aff.histogram), ("placement_locality", aff.locality)]
        for name, fn in calls:
            st = _time_groups([fn], groups=10, inner=5 if name == "ffn" else 10)
            per[name + "_ms"] = st["ms_median"]
            per[name + "_ms_mean"] = st["ms"]
            per[name + "_ms_min"] = st["ms_min"]
        layer_ms = per["gate_ms"] + per["dispatch_ms"] + per["ffn_ms"] + per.get("combine_ms", 0.0)
        per["layer_tokens_per_s"] = cfg.T / (layer_ms * 1e-3)
        result["per_call"] = per

    if "box" in sections:
        # achieved rates of this machine
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        ms = _time_call(lambda: lib.exf_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, B._stream()), 20)
        copy_gbs = 2 * nbytes / (ms * 1e-3) / 1e9
        del src, dst
        wgs, iters = 256 * 8, 2000
        sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
        ms = _time_call(lambda: lib.exf_probe_mfma(wgs, iters, sink.data_ptr(), B._stream()), 5)
        mfma_tflops = wgs * 4 * 4 * iters * 32768.0 / (ms * 1e-3) / 1e12
        # the bare GEMM K loop on all-zero and on random operands (the chip holds a power limit: what
        # the matrix cores sustain depends on the values they multiply), the latter also after a longer run
        loop_bytes = lib.exf_probe_gemm_loop_bytes()
        loop_sink = torch.empty(256 * 256, dtype=torch.float32, device=dev)
        loop_flops = 10 * 512 * 2.0 * 256 * 256 * 1024

        def loop_rate(buf, iters):
            ms = _time_call(lambda: lib.exf_probe_gemm_loop(buf.data_ptr(), loop_bytes, 10, loop_sink.data_ptr(), B._stream()), iters)
            return loop_flops / (ms * 1e-3) / 1e12

        zeros = torch.zeros(loop_bytes // 2, dtype=torch.bfloat16, device=dev)
        loop_zero = loop_rate(zeros, 3)
        del zeros
        rnd = torch.randn(loop_bytes // 2, dtype=torch.float32, device=dev).to(torch.bfloat16)
        torch.cuda.synchronize()
        time.sleep(0.2)
        loop_rand = loop_rate(rnd, 3)
        loop_rand_sustained = loop_rate(rnd, 40)
        del rnd
        # what the vendor GEMM library (through torch.matmul) sustains on this machine on random bf16 operands at
        # the two contraction shapes of the benchmark configuration, as dense GEMMs of the same flop count:
        # [8192,1024] x [4096,1024]^T (first contraction) and [8192,4096] x [1024,4096]^T (second)
        ref_gemm = {}
        if bf16:
            for name, (m_, n_, k_) in (("gemm1_8192x4096x1024", (8192, 4096, 1024)), ("gemm2_8192x1024x4096", (8192, 1024, 4096))):
                a_ = torch.randn((m_, k_), device=dev).to(torch.bfloat16)
                b_ = (torch.randn((n_, k_), device=dev) * 0.02).to(torch.bfloat16)
                c_ = torch.empty((m_, n_), dtype=torch.bfloat16, device=dev)
                st = _time_groups([lambda: torch.matmul(a_, b_.t(), out=c_)], groups=10, inner=10)
                ref_gemm[name + "_TFLOPs"] = 2.0 * m_ * n_ * k_ / (st["ms_median"] * 1e-3) / 1e12
                del a_, b_, c_
            # the same two contractions as batched GEMMs over 8 equal experts of 1024 rows (torch.bmm): eight weight
            # matrices as in the grouped GEMM, but no ragged groups, no GELU, no gather / scatter
            for name, (m_, n_, k_) in (("bmm1_8x1024x4096x1024", (1024, 4096, 1024)), ("bmm2_8x1024x1024x4096", (1024, 1024, 4096))):
                a_ = torch.randn((8, m_, k_), device=dev).to(torch.bfloat16)
                b_ = (torch.randn((8, n_, k_), device=dev) * 0.02).to(torch.bfloat16)
                c_ = torch.empty((8, m_, n_), dtype=torch.bfloat16, device=dev)
                st = _time_groups([lambda: torch.bmm(a_, b_.transpose(1, 2), out=c_)], groups=10, inner=10)
                ref_gemm[name + "_TFLOPs"] = 8 * 2.0 * m_ * n_ * k_ / (st["ms_median"] * 1e-3) / 1e12
                del a_, b_, c_
        result["box"] = {"torch_matmul_random_bf16": ref_gemm, "copy_GBps": copy_gbs, "mfma_loop_TFLOPs": mfma_tflops, "gemm_k_loop_zero_operands_TFLOPs": loop_zero,
                         "gemm_k_loop_random_operands_TFLOPs": loop_rand,
                         "gemm_k_loop_random_operands_sustained_TFLOPs": loop_rand_sustained}
        if roofline["bound"] == "mfma" and bf16:
            result["roofline"]["frac_of_measured_mfma_loop"] = achieved / mfma_tflops
            result["roofline"]["frac_of_measured_gemm_k_loop_random_operands"] = achieved / max(loop_rand, loop_rand_sustained)
            if ref_gemm and cfg.index == 2:  # the vendor library's two GEMMs of the same flop counts, random operands
                for key, names in (("frac_of_vendor_dense_gemms", ("gemm1_8192x4096x1024_TFLOPs", "gemm2_8192x1024x4096_TFLOPs")),
                                   ("frac_of_vendor_batched_gemms", ("bmm1_8x1024x4096x1024_TFLOPs", "bmm2_8x1024x1024x4096_TFLOPs"))):
                    t_ref = sum(ffn_flops / 2 / (ref_gemm[n] * 1e12) for n in names)
                    result["roofline"][key] = achieved / (ffn_flops / t_ref / 1e12)

    if ("hbm4" in sections or "search" in sections) and cfg.index == 2:
        # HBM-bound entry points at the shapes of the one-GPU-share configuration (rotating buffers)
        c4 = syn.CONFIGS[4]
        hbm = {}
        T4, d4 = c4.T, c4.d
        sets = 5  # 5 x (67 MB in + 67 MB out) > 256 MB
        xs4 = [torch.randn((T4, d4), device=dev).to(torch.bfloat16) for _ in range(sets)]
        idx4_h, map4_h = syn.local_routing(c4, syn.seed_for(4, 4, 1))
        idx4 = torch.from_numpy(idx4_h).to(dev)
        map4 = torch.from_numpy(map4_h).to(dev)
        outs = [B.moe_dispatch(xs4[i], idx4, c4.E, c4.E_local, map4) for i in range(sets)]
        ws = torch.empty(max(lib.moe_dispatch_workspace_bytes(T4, 1, c4.E_local), 256), dtype=torch.uint8, device=dev)
        stream = B._stream()
        # (the library is called directly with plain addresses: a call is ~20-30 us on the GPU, the
        # binding's argument checks would be a visible share of that on the host)

        def disp_fn(i):
            a = (xs4[i].data_ptr(), idx4.data_ptr(), map4.data_ptr(), T4, d4, 1, c4.E, c4.E_local, B.EXF_BF16, outs[i].x_sorted.data_ptr(),
                 outs[i].src_of_sorted.data_ptr(), outs[i].sorted_of_src.data_ptr(), outs[i].expert_counts.data_ptr(),
                 outs[i].expert_offsets.data_ptr(), ws.data_ptr(), ws.numel(), stream)
            return lambda: lib.moe_dispatch(*a)

        bytes_disp = T4 * d4 * 2 * 2 + T4 * 16
        if "hbm4" in sections and want4("dispatch"):
            hbm["dispatch"] = _hbm_entry(disp_fn, sets, bytes_disp)
        w4 = torch.rand((T4, 1), device=dev)
        couts = [torch.empty((T4, d4), dtype=torch.bfloat16, device=dev) for _ in range(sets)]

        def comb_fn(i):
            a = (outs[i].x_sorted.data_ptr(), outs[i].sorted_of_src.data_ptr(), w4.data_ptr(), T4, d4, 1, B.EXF_BF16, couts[i].data_ptr(), stream)
            return lambda: lib.moe_combine(*a)

        bytes_comb = T4 * d4 * 2 * 2 + T4 * 12
        if "hbm4" in sections and want4("combine"):
            hbm["combine"] = _hbm_entry(comb_fn, sets, bytes_comb)
        gw4 = torch.randn((c4.E, d4), device=dev).to(torch.bfloat16)
        gi = torch.empty((T4, 1), dtype=torch.int32, device=dev)
        gwt = torch.empty((T4, 1), dtype=torch.float32, device=dev)

        def gate_fn(i):
            a = (xs4[i].data_ptr(), gw4.data_ptr(), T4, d4, c4.E, 1, 0, B.EXF_BF16, None, gi.data_ptr(), gwt.data_ptr(), stream)
            return lambda: lib.moe_gate_topk(*a)

        bytes_gate = T4 * d4 * 2 + c4.E * d4 * 2 + T4 * 8
        if "hbm4" in sections and want4("gate"):
            hbm["gate"] = _hbm_entry(gate_fn, sets, bytes_gate)
        del xs4, outs, couts
        tr4_h, _ = syn.config_trace(c4)
        pl4 = torch.from_numpy(syn.balanced_random_placement(c4.trace_L, c4.trace_E, c4.G, syn.seed_for(4, 5))).to(dev)
        tr_sets = 3  # 3 x 100.7 MB > 256 MB
        base = torch.from_numpy(tr4_h).to(dev)
        traces = [base] + [base.roll(shifts=7 * (i + 1), dims=1).contiguous() for i in range(tr_sets - 1)]
        aff4 = AffinityRun(base, pl4, c4.trace_E, c4.G)
        bytes_tr = 4 * c4.trace_L * c4.trace_N
        tok = lambda ms: {"trace_tokens_per_s": c4.trace_N / (ms * 1e-3)}
        gh = torch.Generator(device="cpu")
        gh.manual_seed(syn.seed_for(4, 7))
        home4 = torch.randint(0, c4.G, (c4.trace_N,), generator=gh, dtype=torch.int32).to(dev)  # requests owned by uniformly drawn GPUs
        ws_rt = torch.empty(max(lib.routing_transfers_workspace_bytes(c4.trace_L, c4.trace_N), 256), dtype=torch.uint8, device=dev)
        if "hbm4" in sections:
            if want4("affinity_histogram"):
                hbm["affinity_histogram"] = _hbm_entry(lambda i: (lambda: aff4.histogram(traces[i])), tr_sets, bytes_tr, tok)
            if want4("placement_locality"):
                hbm["placement_locality"] = _hbm_entry(lambda i: (lambda: aff4.locality(traces[i])), tr_sets, bytes_tr, tok)
            if want4("affinity_statistics"):
                hbm["affinity_statistics"] = _hbm_entry(lambda i: (lambda: aff4.statistics(traces[i])), tr_sets, bytes_tr, tok)
            if want4("routing_transfers"):
                hbm["routing_transfers"] = _hbm_entry(lambda i: (lambda: B.routing_transfers(traces[i], pl4, home4, c4.G, workspace=ws_rt)),
                                                      tr_sets, bytes_tr + 4 * c4.trace_N, tok)
            result["hbm_bound_calls_config4_shapes"] = hbm

    if "search" in sections and cfg.index == 2:
        # placement search on the one-GPU-share trace (24 layers x 1M tokens, E=64, 8 GPUs on 2 nodes):
        # counts on the GPU, host solver, GPU batch scoring of {found, default, random} from the counts
        res4 = B.affinity_histogram(base, c4.trace_E)
        counts4_host = res4["counts"].cpu()
        t_s = time.perf_counter()
        found = B.placement_search(counts4_host, c4.G, nodes=2, restarts=2, seed=1)
        solver_s = time.perf_counter() - t_s
        cands = torch.stack([found, torch.from_numpy(syn.contiguous_placement(c4.trace_L, c4.trace_E, c4.G)),
                             torch.from_numpy(syn.balanced_random_placement(c4.trace_L, c4.trace_E, c4.G, 11))]).to(dev)
        many = cands[torch.arange(4096, device=dev) % 3].contiguous()  # a search-sized batch for the timing
        score_out = torch.empty((4096, c4.trace_L - 1), dtype=torch.int64, device=dev)
        ms = _time_call(lambda: B.placement_locality_from_counts(res4["counts"], many, out=score_out), 20)
        sc = B.placement_locality_from_counts(res4["counts"], cands).sum(dim=1).cpu().numpy()
        total = float(c4.trace_N) * (c4.trace_L - 1)
        node_sc = B.placement_locality_from_counts(res4["counts"], (cands // (c4.G // 2)).to(torch.int32).contiguous()).sum(dim=1).cpu().numpy()
        # cross-GPU transfers of the trace: ratio of token-layer visits that take part in an Alltoall, vanilla (out
        # and back) against coherent contexts
        ratios = {}
        # p and p* of the trace and the forward communication volumes of the paper's comparison table for it
        # (G GPUs holding trace_N / G tokens each, L MoE layers; the top-2 columns use the same ratios)
        for name, pl_t in (("found", cands[0]), ("contiguous", cands[1])):
            loc_t, away_t = B.routing_transfers(base, pl_t.contiguous(), home4, c4.G, workspace=ws_rt)
            p_van, p_star = B.transfer_ratios(away_t.cpu(), loc_t.cpu(), c4.trace_N)
            vol = B.comm_volume(c4.G, c4.trace_N // c4.G, c4.trace_L, p_van, p_star)
            ratios[name] = {"vanilla_p": p_van, "coherent_p_star": p_star, "volume_tokens": vol,
                            "coherent_over_vanilla_top1": vol["coherent_top1"] / vol["vanilla_top1"]}
        result["alltoall_token_ratio"] = ratios
        # affinity across several layers: all 276 ordered layer pairs of the same trace
        ws_mh = torch.empty(max(lib.affinity_multihop_workspace_bytes(c4.trace_L, c4.trace_N, c4.trace_E), 256), dtype=torch.uint8,
                            device=dev)
        ms_mh = _time_groups([(lambda i: (lambda: B.affinity_multihop(traces[i], c4.trace_E, want_prob=True, workspace=ws_mh)))(i)
                              for i in range(tr_sets)], groups=4, inner=3, warmup=3)["ms_median"]
        n_pairs = c4.trace_L * (c4.trace_L - 1) // 2
        result["affinity_multihop"] = {"ms": ms_mh, "layer_pairs": n_pairs, "pair_transitions_per_s": n_pairs * c4.trace_N / (ms_mh * 1e-3),
                                       "trace_bytes": bytes_tr, "workspace_bytes": ws_mh.numel()}
        del ws_mh
        result["placement_search"] = {
            "trace": "24 layers x 1048576 tokens, E=64, planted affinity rho=0.7", "gpus": c4.G, "nodes": 2,
            "host_solver_s": solver_s, "gpu_score_4096_maps_ms": ms, "maps_per_s": 4096 / (ms * 1e-3),
            "gpu_locality": {"found": sc[0] / total, "contiguous": sc[1] / total, "random": sc[2] / total},
            "node_locality": {"found": node_sc[0] / total, "contiguous": node_sc[1] / total, "random": node_sc[2] / total}}

    if "other" in sections and cfg.index == 2 and fused:
        result["other_configs"] = other_configs(syn, torch, MoELayerRun, dev)

    if "cpu" in sections and host is not None:
        result["cpu_baseline"] = cpu_baseline(cfg, host[0], host[1], host[2], host[3], trace_h, pl_h)
        result["cpu_baseline"]["single_thread"] = cpu_baseline_single_thread(cfg, host[0], host[1], host[2], host[3])
    else:
        result["cpu_baseline"] = None

    print(json.dumps(result))


if __name__ == "__main__":
    main()
