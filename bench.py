#!/usr/bin/env python3
"""Benchmark of the LSP per-step hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input:
lsp_attn_step_layers (the attention of every layer of the workload, one launch),
lsp_confidence over the logits, lsp_commit (boundary search + snap + token
commit + KV append for every layer).  Inputs are resident in HBM before the
timed region.  To keep the Infinity Cache from serving re-reads, steps rotate
over several independent input sets whose total size exceeds 256 MB, and every
step gets fresh (prefix_len, suffix_len) arrays so that no restore kernel sits
in the timed region.

Default run (no flags): the headline is configuration 4 (LLaDA-8B shape, long
context, all 32 layers, batch 8): per-step latency and committed tokens/s over
exactly --steps steps; next to it, under "c5_loop", the whole decode loop of
configuration 5 (batch 16, 1024 generated positions, run to termination) with
its own steps / flips / roofline / cpu_baseline, and under "side" the small
configurations 2 and 3.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MALL_BYTES = 256 << 20
MIN_TIMED_MS = 50.0            # a timed region shorter than this is repeated (clocks ramp for ~10 ms after idle)
METRIC = "committed tokens/sec + per-step latency (ms), LLaDA-8B shape, 1 MI355X"
TRAFFIC_FILE = os.path.join("profiles", "lsp_step_hbm_traffic_counters.txt")

# kernels behind each entry point, by name prefix (as rocprofv3 prints them)
KERNELS_OF = {"lsp_attn_step": ("attn_",), "lsp_confidence": ("confidence_",), "lsp_commit": ("append_kernel", "boundary_kernel")}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "scatter", "lmhead"],
                    help="c1..c4: one step; c5: the decode loop; scatter: prefix-first against Scattered-Margin commits; "
                         "lmhead: output head fused with the confidence reduction against library GEMM + lsp_confidence")
    ap.add_argument("--sizing", default="tau", choices=["tau", "adaptive", "full"],
                    help="c5: fixed threshold (default), adaptive threshold (Eq. 2, [0.25, 0.5]) or the Full baseline (1 position per step)")
    ap.add_argument("--loop-steps", type=int, default=0, help="c5: stop the decode loop after this many steps (0 = run to the end)")
    ap.add_argument("--layers", type=int, default=0, help="override the workload's layer count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--also", default="auto",
                    help="comma list of further workloads reported next to the headline; auto = c5,c2,c3 for the default "
                         "headline (c4), none otherwise; \"\" = none")
    ap.add_argument("--calibrate-copy", action="store_true", help="only run the 1 GiB copy used to scale HBM counters")
    ap.add_argument("--calibrate-read", action="store_true",
                    help="only run a bare streaming read of configuration 2's logits bytes (what bounds lsp_confidence there)")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="only run the power-limit probe: bare matrix loop and attention on constant vs N(0,1) operands")
    ap.add_argument("--graph", type=int, default=1, help="replay the step from a HIP graph (1) or launch eagerly (0)")
    ap.add_argument("--loop-graph", type=int, default=0,
                    help="c5: replay every step after the first from one captured HIP graph")
    ap.add_argument("--flip-trace", type=int, default=0, help="c5: 1 = add the per-step flip trace to the output")
    return ap.parse_args()


# --------------------------------------------------------------------------- #
# HBM traffic per launch, from the committed rocprofv3 counter summary
# --------------------------------------------------------------------------- #
def parse_traffic(path=os.path.join(ROOT, TRAFFIC_FILE)):
    """{workload: {kernel name: {counter: units per dispatch}}} and the KiB-per-unit scale of
    each counter (from the 1 GiB copy in the same file).  Empty when the file is missing.
    table[workload]["layers"] = layer count of the profiled run ("-- workload c4 layers=2")."""
    table, scale = {}, {}
    try:
        text = open(path).read()
    except OSError:
        return table, scale
    sect = "calibration"
    for line in text.splitlines():
        m = re.match(r"-- workload (\w+)(?: layers=(\d+))?", line)
        if m:
            sect = m.group(1)
            table.setdefault(sect, {})["layers"] = int(m.group(2) or 1)
            continue
        m = re.match(r"(\S.*?)\s+(FETCH_SIZE|WRITE_SIZE)\s+dispatches=\s*(\d+)\s+avg_per_dispatch=\s*([0-9.]+)", line)
        if not m:
            continue
        kern, ctr, val = m.group(1).strip(), m.group(2), float(m.group(4))
        table.setdefault(sect, {}).setdefault(kern, {})[ctr] = val
    cal = table.get("calibration", {}).get("__amd_rocclr_copyBuffer")
    if cal and "FETCH_SIZE" in cal and "WRITE_SIZE" in cal:
        gib_kib = float(1 << 20)
        scale = {"FETCH_SIZE": gib_kib / cal["FETCH_SIZE"], "WRITE_SIZE": gib_kib / cal["WRITE_SIZE"]}
    return table, scale


def traffic_for(workload, call, layers=1):
    """Measured HBM bytes per launch of `call` at `workload` with `layers` layers (read + written), or
    None when the committed summary has no line for every kernel of that call.  The attention and
    append kernels move bytes in proportion to the layer count of a launch: their counters are taken
    per layer of the profiled run and multiplied by `layers`."""
    table, scale = parse_traffic()
    sec = table.get(workload)
    if not sec or not scale:
        return None
    total, found = 0.0, 0
    for kern, ctrs in sec.items():
        if kern == "layers" or not kern.startswith(KERNELS_OF[call]) or "FETCH_SIZE" not in ctrs or "WRITE_SIZE" not in ctrs:
            continue
        per_layer = kern.startswith(("attn_", "append_kernel"))
        f = layers / sec["layers"] if per_layer else 1.0
        total += (ctrs["FETCH_SIZE"] * scale["FETCH_SIZE"] + ctrs["WRITE_SIZE"] * scale["WRITE_SIZE"]) * 1024 * f
        found += 1
    return round(total) if found >= len(KERNELS_OF[call]) else None


def attn_roofline_entry(w, W, flops, seconds, bytes_moved):
    """The attention is bound by the matrix cores only above the machine balance (2.5 PFLOP/s
    over 8 TB/s = 312 flop per byte); below it (a short suffix over a short prefix) by HBM."""
    peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 157.3
    if flops / bytes_moved >= peak * 1e12 / (HBM_PEAK_GBS * 1e9):
        return {"s": seconds, "bound": "mfma", "achieved": flops / seconds / 1e12, "peak": peak, "unit": "TFLOP/s"}
    return {"s": seconds, "bound": "hbm", "achieved": bytes_moved / seconds / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}


# --------------------------------------------------------------------------- #
# one step (configurations 1-4)
# --------------------------------------------------------------------------- #
def run_workload(name, K, Wm, layers=0, use_graph=True, cpu_baseline=True, cpu_budget_s=10.0):
    """Time K steps of one workload; returns (value, ms_per_step, config, roofline, cpu_baseline)."""
    import torch
    import paper_2603_05454_amd as lsp
    import workloads as W

    dev = torch.device("cuda:0")
    w = {"c1": W.C1, "c2": W.C2, "c3": W.C3, "c4": W.C4}[name]
    if layers:
        w = W.scaled(w, layers=layers)
    es = W.elem_bytes(w)

    # ---- input sets ------------------------------------------------------------
    kv_bytes_layer = (w.B * w.S * (w.Hq + 2 * w.Hkv) * w.D + 2 * w.B * w.C * w.Hkv * w.D) * es
    set_bytes = w.B * w.S * w.V * es + w.layers * kv_bytes_layer
    R = max(1, min(8, -(-3 * MALL_BYTES // set_bytes)))       # >= 768 MB in rotation when sets are small
    sets = []
    _, bitmap = W.make_delimiters(w)
    bitmap = bitmap.to(dev)
    for r in range(R):
        wr = W.scaled(w, seed=w.seed + 101 * r)
        z, _ = W.make_logits(wr, device=dev)
        lay = [W.make_layer_kv(wr, l, device=dev) for l in range(w.layers)]
        table = lsp.LayerTable([L["k_suf"] for L in lay], [L["v_suf"] for L in lay],
                               [L["k_cache"] for L in lay], [L["v_cache"] for L in lay])
        attn = lsp.AttnLayerTable(*[[L[k] for L in lay] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")],
                                  [torch.empty_like(L["q"]) for L in lay])        # one output per layer
        sets.append(dict(z=z, layers=lay, table=table, attn=attn, tokens=W.make_tokens(wr, w.C).to(dev), w=wr))
    pl0, sl0 = W.make_lengths(w, device=dev)
    n_state = K + Wm
    PL = pl0.repeat(n_state + 1, 1).contiguous()
    SL = sl0.repeat(n_state + 1, 1).contiguous()
    conf_out = (torch.empty((w.B, w.S), dtype=torch.int32, device=dev),
                torch.empty((w.B, w.S), dtype=torch.float32, device=dev),
                torch.empty((w.B, w.S), dtype=torch.float32, device=dev))
    commit_out = []
    for _ in range(n_state + 1):
        o = {"stable_mask": torch.empty((w.B, w.S), dtype=torch.uint8, device=dev)}
        for k in ("raw_boundary", "snapped_boundary", "commit_len", "status_flags"):
            o[k] = torch.zeros(w.B, dtype=torch.int32, device=dev)
        commit_out.append(o)
    ws_bytes = max(lsp.confidence_workspace_bytes(w.B, w.S, w.V), 256)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def attn(s, pl, sl):
        lsp.attn_step_layers(s["attn"], pl, sl)

    def conf(s, sl):
        lsp.confidence(s["z"], sl, out=conf_out, workspace=workspace)

    def commit(s, pl, sl, out):
        lsp.commit(conf_out[2], conf_out[0], bitmap, w.V, w.tau, w.window, w.min_commit, 1, pl, sl,
                   tokens=s["tokens"], layers=s["table"], out=out)

    def step(i):
        s = sets[i % R]
        attn(s, PL[i], SL[i])
        conf(s, SL[i])
        commit(s, PL[i], SL[i], commit_out[i])

    # ---- whole-step timing --------------------------------------------------------
    for i in range(Wm):
        step(i)
    torch.cuda.synchronize()
    graph = None
    if use_graph:
        # capture the K timed steps once (each has its own state arrays), replay inside the timed region
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(Wm, Wm + K):
                step(i)
        torch.cuda.synchronize()
        # capture does not execute: the state arrays of the timed steps are still untouched

    def timed_round():
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        if graph is not None:
            graph.replay()
        else:
            for i in range(Wm, Wm + K):
                step(i)
        ev1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1) * 1e-3

    # EXACTLY K steps per round.  A round shorter than MIN_TIMED_MS is repeated (state arrays
    # restored outside the timed region; an append then rewrites the same rows with the same
    # data) until the rounds add up to that, and the mean round is reported.
    walls, evs = [], []
    while True:
        wall, ev = timed_round()
        walls.append(wall)
        evs.append(ev)
        if sum(walls) * 1e3 >= MIN_TIMED_MS or len(walls) >= 500:
            break
        PL[Wm:Wm + K] = pl0
        SL[Wm:Wm + K] = sl0
    wall = sum(walls) / len(walls)
    ms_per_step = wall * 1e3 / K
    committed = int(sum(int(commit_out[i]["commit_len"].sum().item()) for i in range(Wm, Wm + K)))
    value = committed / wall

    # ---- per-call timing (HIP events on the launch stream, calls back to back) ------
    # Launched the way the timed step is: replayed from a captured graph of `reps` calls when the
    # step runs from a graph (eager launches of microsecond kernels would mostly time the host).
    def time_call(fn, reps):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        g = None
        if graph is not None:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for i in range(reps):
                    fn(i)
            g.replay()
            torch.cuda.synchronize()
        total, n = 0.0, 0
        while total * 1e3 < MIN_TIMED_MS and n < 200:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            if g is not None:
                g.replay()
            else:
                for i in range(reps):
                    fn(i)
            b.record()
            torch.cuda.synchronize()
            total += a.elapsed_time(b) * 1e-3
            n += 1
        return total / (n * reps)

    reps = max(4, min(K, 200))
    scratch_pl, scratch_sl = PL[n_state], SL[n_state]

    def reset_state():
        scratch_pl.copy_(pl0)
        scratch_sl.copy_(sl0)

    t_attn = time_call(lambda i: attn(sets[i % R], pl0, sl0), reps)        # all layers, one launch
    t_conf = time_call(lambda i: conf(sets[i % R], sl0), reps)
    # the commit mutates its state arrays: time it on scratch copies, restoring between calls
    # (the two tiny copies are timed separately and subtracted)
    t_copy = time_call(lambda i: reset_state(), reps)
    conf(sets[0], sl0)

    def commit_once(i):
        reset_state()
        commit(sets[0], scratch_pl, scratch_sl, commit_out[n_state])

    t_commit = max(time_call(commit_once, reps) - t_copy, 0.0)

    L0 = commit_out[n_state]["commit_len"].sum().item()
    conf_bytes = w.B * w.S * (w.V * es + 12)
    flops_all = W.attn_flops(w) * w.layers
    append_bytes = 2 * L0 * w.Hkv * w.D * es * 2 * w.layers
    attn_bytes = (2 * w.B * (w.P + w.S) * w.Hkv * w.D + 2 * w.B * w.S * w.Hq * w.D) * es * w.layers
    kernels = {
        "lsp_attn_step": attn_roofline_entry(w, W, flops_all, t_attn, attn_bytes),
        "lsp_confidence": {"s": t_conf, "bound": "hbm", "achieved": conf_bytes / t_conf / 1e9,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s"},
        "lsp_commit": {"s": t_commit, "bound": "hbm", "achieved": append_bytes / max(t_commit, 1e-9) / 1e9,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s"},
    }
    # an append of a few megabytes is two dependent launches, not an HBM stream: no roofline fraction for it
    commit_is_stream = append_bytes >= 64 << 20
    if not commit_is_stream:
        kernels["lsp_commit"]["bound"] = "latency"
    share = {k: v["s"] for k, v in kernels.items()}
    dom = max(share, key=share.get)
    kd = kernels[dom]
    traffic = traffic_for(name, dom, w.layers)
    path_bytes = conf_bytes + append_bytes
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": round(kd["achieved"], 2), "peak": kd["peak"],
                "unit": kd["unit"], "frac": round(kd["achieved"] / kd["peak"], 4),
                "traffic": traffic,
                "traffic_unit": f"HBM bytes per launch, read + written: rocprofv3 FETCH_SIZE / WRITE_SIZE in {TRAFFIC_FILE}"
                                + (f", per-layer figure of the profiled run x {w.layers} layers" if dom == "lsp_attn_step" and w.layers > 1 else ""),
                "avg_launch_us": round(kd["s"] * 1e6, 2),
                "launch": (f"one launch = all {w.layers} layers" if dom == "lsp_attn_step" else "one launch per step"),
                "all": {k: {"avg_us": round(v["s"] * 1e6, 2), "bound": v["bound"], "achieved": round(v["achieved"], 2),
                            "unit": v["unit"], "frac": (round(v["achieved"] / v["peak"], 4) if v["bound"] != "latency" else None)}
                        for k, v in kernels.items()},
                "reduction_plus_commit_path": {"bytes": path_bytes, "us": round((t_conf + t_commit) * 1e6, 2),
                                               "frac_of_hbm_peak": round(path_bytes / (t_conf + t_commit) / 1e9 / HBM_PEAK_GBS, 4)}}

    cpu = cpu_baseline_step(w, sets[0], bitmap, pl0, sl0, cpu_budget_s) if cpu_baseline else None

    config = {"workload": w.name, "B": w.B, "layers": w.layers, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
              "P": w.P, "S": w.S, "C": w.C, "V": w.V, "tau": w.tau, "window": w.window,
              "input_sets_rotated": R, "committed_tokens_per_step": round(committed / K, 2),
              "launch": ("hip_graph" if graph is not None else "eager") + ", 3 library calls per step",
              "timed_rounds_of_K_steps": len(walls), "min_round_ms_per_step": round(min(walls) * 1e3 / K, 5),
              "median_round_ms_per_step": round(sorted(walls)[len(walls) // 2] * 1e3 / K, 5),
              "event_ms_per_step": round(sum(evs) / len(evs) * 1e3 / K, 5), "dtype": w.dtype}
    return value, ms_per_step, config, roofline, cpu


def _attention_sample(w, gen_seed, rows_per_seq_head):
    """(layers, rows) of the oracle's attention sample: first / middle / last layer, heads
    0, 13 and the last (taken modulo the head count), seeded query rows of every sequence."""
    import torch
    lay = sorted({0, (w.layers - 1) // 2, w.layers - 1})
    heads = sorted({0, 13 % w.Hq, w.Hq - 1})
    g = torch.Generator().manual_seed(gen_seed)
    rows = torch.tensor([[b, i, h] for b in range(w.B) for h in heads
                         for i in torch.randint(0, w.S, (rows_per_seq_head,), generator=g).tolist()], dtype=torch.int32)
    return lay, heads, rows


def cpu_baseline_step(w, s, bitmap, pl0, sl0, budget_s=10.0):
    """The oracle, as it stands, on the host cores over one step of input set 0.  Nothing here
    comes from the HIP path: confidence in full (all rows), commit on the oracle's own ids and
    margins with the append over the sampled layers, attention on a stated row sample; sampled
    parts are scaled to the whole step.  Small workloads are also timed on one thread."""
    import torch
    import oracle
    import workloads as W

    total_rows = w.B * w.S * w.Hq
    full_attention = W.attn_flops(w) * w.layers < 8e9
    lay, heads, rows = _attention_sample(w, 1, 32 if w.S >= 512 else 8)
    if full_attention:
        lay, rows = list(range(w.layers)), None
    hz = s["z"].cpu()
    hl = {l: {k: v.cpu() for k, v in s["layers"][l].items()} for l in lay}
    bm = bitmap.cpu()
    threads = oracle.num_threads()

    def one_pass():
        pl, sl, tok = pl0.cpu().clone(), sl0.cpu().clone(), s["tokens"].cpu().clone()
        caches = {l: (hl[l]["k_cache"].clone(), hl[l]["v_cache"].clone()) for l in lay}
        c0 = time.perf_counter()
        for l in lay:
            L = hl[l]
            oracle.attention(L["q"], L["k_suf"], L["v_suf"], L["k_cache"], L["v_cache"], pl, sl, rows=rows)
        c1 = time.perf_counter()
        ids, _, mar = oracle.confidence(hz, sl)
        c2 = time.perf_counter()
        oc = oracle.commit(mar, ids, bm, w.V, w.tau, w.window, w.min_commit, 1, pl, sl, tokens=tok,
                           k_suf=[hl[l]["k_suf"] for l in lay], v_suf=[hl[l]["v_suf"] for l in lay],
                           k_cache=[caches[l][0] for l in lay], v_cache=[caches[l][1] for l in lay])
        c3 = time.perf_counter()
        return c1 - c0, c2 - c1, c3 - c2, int(oc["commit_len"].sum())

    ta = tc = tm = 0.0
    passes = 0
    begin = time.perf_counter()
    while passes < 40 and (passes == 0 or time.perf_counter() - begin < budget_s):
        a, c, m, committed = one_pass()
        ta, tc, tm, passes = ta + a, tc + c, tm + m, passes + 1
    spent = time.perf_counter() - begin
    attn_scale = (w.layers / len(lay)) * (1.0 if rows is None else total_rows / rows.shape[0])
    t_full = (ta * attn_scale + tc + tm * (w.layers / len(lay))) / passes
    cpu = {"value": round(committed / t_full, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
           "sample": (f"{passes} pass(es) over one step of input set 0: attention on "
                      + ("every row of every layer" if rows is None else
                         f"layers {lay} x heads {heads} x {rows.shape[0] // (w.B * len(heads))} seeded query rows per sequence "
                         f"(all keys), scaled x{attn_scale:.0f}")
                      + f"; confidence over all {w.B * w.S} rows; commit in full with the append over "
                      + (f"{len(lay)} of {w.layers} layers, scaled" if len(lay) < w.layers else "every layer")),
           "ms_per_step": round(t_full * 1e3, 2),
           "ms_parts_scaled": {"attention": round(ta * attn_scale / passes * 1e3, 2), "confidence": round(tc / passes * 1e3, 2),
                               "commit": round(tm * (w.layers / len(lay)) / passes * 1e3, 2)},
           "cpu_seconds_spent": round(spent, 2)}
    if full_attention and threads > 1:      # the small configurations: also on one thread
        oracle.set_num_threads(1)
        try:
            a, c, m, _ = one_pass()
        finally:
            oracle.set_num_threads(threads)
        cpu["single_thread_ms_per_step"] = round((a + c + m) * 1e3, 2)
    return cpu


# --------------------------------------------------------------------------- #
# configuration 5: the decode loop
# --------------------------------------------------------------------------- #
def run_loop_workload(max_steps=0, sizing="tau", use_graph=False, cpu_baseline=True, flip_trace=False):
    """Config 5: the whole decode loop (Algorithm 1 lines 3-11) at LLaDA-8B shape, batch 16,
    prompt 512, 1024 generated positions, all 32 layers' attention and KV append every step.
    The step's logits come from the seeded synthetic process (workloads.make_process_logits),
    which stands in for the denoiser and is NOT part of the timed path: every step's library
    calls are bracketed by HIP events and the sum is the loop time."""
    import torch
    import paper_2603_05454_amd as lsp
    from paper_2603_05454_amd.loop import decode_loop
    import workloads as W

    dev = torch.device("cuda:0")
    w = W.C5
    _, bitmap = W.make_delimiters(w)
    layers = [W.make_layer_kv(w, l, device=dev) for l in range(w.layers)]
    pl, sl = W.make_lengths(w, device=dev)
    tokens = W.make_tokens(w, w.C).to(dev)
    fn = lambda step, p: W.make_process_logits(w, dev, step, p)[0]
    # sizing: "tau" = fixed margin threshold (the configuration BASELINE.json names); "adaptive" = the
    # threshold chosen per step so that L' lies in [N/4, N/2] (Eq. 2 with Section 4.1's interval);
    # "full" = the paper's Full baseline, one position per step (T_max = generation length)
    tau, kw = w.tau, {}
    if sizing == "adaptive":
        kw = dict(adaptive=True, alpha=0.25, beta=0.5)
    elif sizing == "full":
        tau = float("inf")

    # roofline of the dominant kernel: the attention launch (all layers) at the loop's first step
    table = lsp.AttnLayerTable(*[[L[k] for L in layers] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")],
                               [torch.empty_like(L["q"]) for L in layers])
    for _ in range(2):
        lsp.attn_step_layers(table, pl, sl)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(3):
        lsp.attn_step_layers(table, pl, sl)
    b.record()
    torch.cuda.synchronize()
    t0_attn = a.elapsed_time(b) * 1e-3 / 3
    fl0 = W.attn_flops(w) * w.layers
    es = W.elem_bytes(w)
    by0 = (2 * w.B * (w.P + w.S) * w.Hkv * w.D + 2 * w.B * w.S * w.Hq * w.D) * es * w.layers
    e = attn_roofline_entry(w, W, fl0, t0_attn, by0)
    roofline = {"kernel": "lsp_attn_step", "bound": e["bound"], "achieved": round(e["achieved"], 2), "peak": e["peak"],
                "unit": e["unit"], "frac": round(e["achieved"] / e["peak"], 4), "traffic": None,
                "avg_launch_us": round(t0_attn * 1e6, 2),
                "launch": f"one launch = all {w.layers} layers, at the loop's first step (P_b = {w.P}, N_b = {w.S})"}
    del table
    torch.cuda.empty_cache()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    r = decode_loop(fn, bitmap.to(dev), w.V, tau, w.window, w.min_commit, 1, pl, sl, tokens,
                    kv_layers=layers, gen_len=w.gen_len, run_attention=True, timed=True,
                    stop_after=max_steps or None, commit_kw=kw, graph=use_graph, flip_trace=True)
    wall = time.perf_counter() - t0
    lsp_s = r["lsp_ms"] * 1e-3
    ms = r["lsp_ms_steps"]
    n = r["steps"]
    tr = r["flip_trace"].sum(1)                       # [steps, 2]: flips, positions compared, over the batch
    tail = ms[-max(1, n // 10):]
    config = {"workload": w.name, "B": w.B, "layers": w.layers, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
              "P": w.P, "gen_len": w.gen_len, "C": w.C, "V": w.V, "tau": tau, "window": w.window, "sizing": sizing,
              "loop_steps": n, "committed_tokens": r["committed"], "flips": r["flips"],
              "flip_rate": round(r["flips"] / max(1, r["flip_denominator"]), 5),
              "flip_rate_25_75": round(r["window_flips"] / max(1, r["window_denominator"]), 5),
              "flip_window": "sequences with 256..768 of their 1024 positions committed (Section 4.3.4's mid-stage)",
              "ms_at_steps": {str(i): round(ms[i], 3) for i in sorted({0, 1, n // 4, n // 2, 3 * n // 4, n - 1})},
              "ms_last_tenth_of_steps_mean": round(sum(tail) / len(tail), 3),
              "flip_rate_at_steps": {str(i): round(int(tr[i, 0]) / max(1, int(tr[i, 1])), 4)
                                     for i in sorted({1, n // 4, n // 2, 3 * n // 4, n - 1}) if i < n},
              "lsp_seconds": round(lsp_s, 4), "wall_seconds_with_logit_generator": round(wall, 2),
              "launch": ("first step eager, then one HIP graph replayed per step" if use_graph else "eager, 4 launches per step") +
                        ", one termination poll per step", "dtype": w.dtype}
    if flip_trace:
        config["flip_trace_per_step"] = [[int(f), int(c)] for f, c in tr.tolist()]
    cpu = cpu_baseline_loop(w, tau, kw, layers) if cpu_baseline else None
    return r["committed"] / lsp_s, r["lsp_ms"] / max(1, n), config, roofline, cpu


def cpu_baseline_loop(w, tau, kw, layers_dev, budget_s=12.0):
    """The oracle loop on the host cores over a bounded sample of configuration 5: ONE sequence
    of the same seeded process (K/V operands: sequence 0's), from the loop's start, for as many
    steps as fit the time budget (state from the oracle's own loop).  Per step: confidence and commit
    in full (append over layers 0/15/31, scaled to 32), attention on a row sample of those
    layers every 8th step (scaled to every row, layer and step).  Reported as committed
    tokens of that sequence per second of scaled oracle time - the batch's other sequences
    would multiply tokens and time alike."""
    import torch
    import oracle
    import workloads as W

    dev = "cuda:0"
    w1 = W.scaled(w, B=1)
    lay = sorted({0, (w.layers - 1) // 2, w.layers - 1})
    heads = sorted({0, 13 % w.Hq, w.Hq - 1})
    hl = [{k: v[:1].cpu().contiguous() for k, v in layers_dev[l].items()} for l in lay]
    # the timed run has appended to these caches: only the seeded prompt rows [0, P) are kept
    for L in hl:
        L["k_cache"][:, w.P:] = W.POISON_F32
        L["v_cache"][:, w.P:] = W.POISON_F32
    _, bm = W.make_delimiters(w1)
    pl, sl = W.make_lengths(w1)
    tokens = W.make_tokens(w1, w.C)
    g = torch.Generator().manual_seed(2)
    t_conf = t_commit = t_attn_scaled = 0.0
    steps = committed = 0
    begin = time.perf_counter()
    attn_rate = None            # seconds per (row, key) of the oracle's attention, refreshed every 8th step
    while int(sl.max()) > 0 and time.perf_counter() - begin < budget_s:
        z = W.make_process_logits(w1, dev, steps, pl)[0].cpu()
        N, P = int(sl[0]), int(pl[0])
        if steps % 8 == 0:
            rows = torch.tensor([[0, i, h] for h in heads for i in torch.randint(0, N, (8,), generator=g).tolist()], dtype=torch.int32)
            c0 = time.perf_counter()
            for L in hl:
                oracle.attention(L["q"], L["k_suf"], L["v_suf"], L["k_cache"], L["v_cache"], pl, sl, rows=rows)
            attn_rate = (time.perf_counter() - c0) / (len(hl) * rows.shape[0] * (P + N))
        t_attn_scaled += attn_rate * (w.layers * N * w.Hq * (P + N))
        c1 = time.perf_counter()
        ids, _, mar = oracle.confidence(z, sl)
        c2 = time.perf_counter()
        out = oracle.commit(mar, ids, bm, w.V, tau, w.window, w.min_commit, 1, pl, sl, tokens=tokens,
                            k_suf=[L["k_suf"] for L in hl], v_suf=[L["v_suf"] for L in hl],
                            k_cache=[L["k_cache"] for L in hl], v_cache=[L["v_cache"] for L in hl], **kw)
        c3 = time.perf_counter()
        t_conf += c2 - c1
        t_commit += (c3 - c2) * (w.layers / len(hl))
        committed += int(out["commit_len"].sum())
        steps += 1
    spent = time.perf_counter() - begin
    t_scaled = t_attn_scaled + t_conf + t_commit
    return {"value": round(committed / t_scaled, 4), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": (f"one sequence of {w.B}, first {steps} steps of its loop ({committed} of {w.gen_len} positions committed): "
                       f"confidence and commit in full, append over layers {lay} scaled to {w.layers}, attention on "
                       f"layers {lay} x heads {heads} x 8 seeded rows every 8th step, scaled to every row, layer and step"),
            "scaled_seconds": round(t_scaled, 2),
            "seconds_parts_scaled": {"attention": round(t_attn_scaled, 2), "confidence": round(t_conf, 3), "commit": round(t_commit, 3)},
            "cpu_seconds_spent": round(spent, 2)}


def run_scatter_comparison(layers=32):
    """Prefix-first against Scattered-Margin on the config-4 shapes (Section 4.3.3's systems
    claim, measured): the same number of rows per sequence is committed either as LSP's
    contiguous block or at the highest-margin positions anywhere; the cache is then either
    contiguous or addressed through a row index (a random permutation: full fragmentation)."""
    import torch
    import paper_2603_05454_amd as lsp
    import workloads as W

    dev = torch.device("cuda:0")
    w = W.scaled(W.C4, layers=layers)
    es = W.elem_bytes(w)
    _, bitmap = W.make_delimiters(w)
    bitmap = bitmap.to(dev)
    z, _ = W.make_logits(w, device=dev)
    kv = [W.make_layer_kv(w, l, device=dev) for l in range(w.layers)]
    table = lsp.LayerTable([L["k_suf"] for L in kv], [L["v_suf"] for L in kv], [L["k_cache"] for L in kv], [L["v_cache"] for L in kv])
    pl0, sl0 = W.make_lengths(w, device=dev)
    ids, prob, margin = lsp.confidence(z)
    pl, sl = pl0.clone(), sl0.clone()
    out = lsp.commit(margin, ids, bitmap, w.V, w.tau, w.window, w.min_commit, 1, pl, sl, C=w.C)   # sizes only
    count = out["commit_len"].clone()
    rows_total = int(count.sum().item())
    sel = lsp.select_scattered(margin, sl0, count)
    appended = torch.empty(w.B, dtype=torch.int32, device=dev)
    g = torch.Generator(device="cpu").manual_seed(5)
    perm = torch.stack([torch.randperm(w.C, generator=g) for _ in range(w.B)]).to(torch.int32).to(dev)
    attn_out = torch.empty_like(kv[0]["q"])

    def timed(fn, reps=30):
        for _ in range(15):      # clocks ramp for some milliseconds after idle
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    def reset():
        pl.copy_(pl0)
        sl.copy_(sl0)

    def contiguous_commit():
        reset()
        lsp.commit(margin, ids, bitmap, w.V, w.tau, w.window, w.min_commit, 1, pl, sl, layers=table, out=out)

    def scattered_commit():
        reset()
        lsp.select_scattered(margin, sl, count, out=sel)
        lsp.kv_gather_append(sel[0], count, pl, table, appended=appended)

    L0 = kv[0]
    t_reset = timed(reset)
    t_cont = timed(contiguous_commit) - t_reset
    t_scat = timed(scattered_commit) - t_reset
    t_sel = timed(lambda: lsp.select_scattered(margin, sl0, count, out=sel))
    t_attn = timed(lambda: lsp.attn_step(L0["q"], L0["k_suf"], L0["v_suf"], L0["k_cache"], L0["v_cache"], pl0, sl0, out=attn_out))
    t_attn_g = timed(lambda: lsp.attn_step(L0["q"], L0["k_suf"], L0["v_suf"], L0["k_cache"], L0["v_cache"], pl0, sl0,
                                           out=attn_out, cache_row_index=perm))
    moved = 2 * rows_total * w.Hkv * w.D * es * 2 * w.layers
    fl = W.attn_flops(w)
    return {"workload": "c4 shapes, %d layers" % w.layers, "rows_committed_per_step": rows_total,
            "commit_prefix_first_us": round(t_cont * 1e6, 1), "commit_scattered_us": round(t_scat * 1e6, 1),
            "of_which_selection_us": round(t_sel * 1e6, 1),
            "append_prefix_first_GBs": round(moved / t_cont / 1e9, 1), "append_scattered_GBs": round(moved / t_scat / 1e9, 1),
            "attention_contiguous_us": round(t_attn * 1e6, 1), "attention_indexed_us": round(t_attn_g * 1e6, 1),
            "attention_contiguous_TFLOPs": round(fl / t_attn / 1e12, 1), "attention_indexed_TFLOPs": round(fl / t_attn_g / 1e12, 1),
            "commit_ratio_scattered_over_prefix": round(t_scat / t_cont, 3),
            "attention_ratio_indexed_over_contiguous": round(t_attn_g / t_attn, 3)}


def run_lm_head_comparison(K=4096):
    """Output head fused with the confidence reduction (logits never stored) against the
    unfused path: the library's bf16 GEMM writing [rows, V] bf16 logits, then lsp_confidence.
    Config-2 and config-4 rows and vocabulary, hidden size 4096 (LLaDA-8B), random weights."""
    import torch
    import paper_2603_05454_amd as lsp
    import workloads as W

    dev = torch.device("cuda:0")
    res = {}
    for w in (W.C2, W.C4):
        hidden, weight, _ = W.make_lm_head(w, K, device=dev)
        rows = w.B * w.S
        out = lsp.lm_head_confidence(hidden, weight)
        ws = torch.empty(lsp.lib().lsp_lm_head_confidence_workspace_bytes(w.B, w.S, w.V), dtype=torch.uint8, device=dev)
        z = torch.empty((w.B, w.S, w.V), dtype=torch.bfloat16, device=dev)
        cws = torch.empty(max(16, lsp.confidence_workspace_bytes(w.B, w.S, w.V)), dtype=torch.uint8, device=dev)
        out2 = tuple(torch.empty_like(t) for t in out)

        def timed(fn, reps):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e-3 / reps

        reps = 20 if rows > 1024 else 100
        t_fused = timed(lambda: lsp.lm_head_confidence(hidden, weight, out=out, workspace=ws), reps)
        t_gemm = timed(lambda: torch.matmul(hidden, weight.t(), out=z), reps)
        t_conf = timed(lambda: lsp.confidence(z, out=out2, workspace=cws), reps)
        flop = 2.0 * rows * w.V * K
        agree = float((out[0] == out2[0]).float().mean().item())   # bf16-rounded logits can flip near-ties
        res[w.name] = {"rows": rows, "V": w.V, "K": K, "flop": flop,
                       "fused_us": round(t_fused * 1e6, 1), "fused_TFLOPs": round(flop / t_fused / 1e12, 1),
                       "fused_frac_of_2.5PFLOPs": round(flop / t_fused / 2.5e15, 3),
                       "library_gemm_us": round(t_gemm * 1e6, 1), "library_gemm_TFLOPs": round(flop / t_gemm / 1e12, 1),
                       "lsp_confidence_us": round(t_conf * 1e6, 1),
                       "unfused_total_us": round((t_gemm + t_conf) * 1e6, 1),
                       "fused_over_unfused_time": round(t_fused / (t_gemm + t_conf), 3),
                       "logits_bytes_not_written_or_read": 2 * rows * w.V * 2,
                       "top1_id_agreement_with_unfused": round(agree, 5)}
        del hidden, weight, z
        torch.cuda.empty_cache()
    return res


def calibrate_copy():
    """A plain device-to-device copy of known size (1 GiB read + 1 GiB written per
    launch, 5 launches): what rocprofv3's FETCH_SIZE / WRITE_SIZE counters read
    for it gives the factor that scales the counters of the other kernels."""
    import torch
    n = 1 << 30
    src = torch.full((n,), 1, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy_bytes_per_launch": n, "launches": 5}))


def calibrate_read():
    """What a bare streaming read of configuration 2's logits (256 rows x 126 464 bf16 = 64.7 MB,
    cold: rotated over 12 buffers, one workgroup of 512 threads per row like lsp_confidence there)
    costs end to end on this chip, and the streaming rate of a 2 GiB read.  lsp_bench_read does
    nothing but load and XOR: this bounds lsp_confidence at that size from below.  Launched the
    way the timed step is (replayed from a captured graph), HIP events around the replays."""
    import torch
    import paper_2603_05454_amd as lsp
    n = 256 * 126464 * 2
    bufs = [torch.randint(0, 100, (n // 4,), dtype=torch.int32, device="cuda:0") for _ in range(12)]
    big = torch.randint(0, 100, (512 << 20,), dtype=torch.int32, device="cuda:0")
    out = torch.zeros(8192, dtype=torch.int32, device="cuda:0")
    res = {}
    for name, fn, reps, nbytes in (("read_64.7MB_256_workgroups", lambda i: lsp.bench_read(bufs[i % 12], 256, out), 120, n),
                                   ("read_64.7MB_2048_workgroups", lambda i: lsp.bench_read(bufs[i % 12], 2048, out), 120, n),
                                   ("read_2GiB_8192_workgroups", lambda i: lsp.bench_read(big, 8192, out), 10, big.numel() * 4)):
        for i in range(12):
            fn(i)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(reps):
                fn(i)
        g.replay()
        torch.cuda.synchronize()
        total, k = 0.0, 0
        while total < MIN_TIMED_MS and k < 50:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            g.replay()
            b.record()
            torch.cuda.synchronize()
            total += a.elapsed_time(b)
            k += 1
        t = total * 1e-3 / (k * reps)
        res[name] = {"bytes": nbytes, "us": round(t * 1e6, 2), "GBs": round(nbytes / t / 1e9, 1)}
    print(json.dumps({"calibrate_read": res}))


class BoardPower:
    """Mean board power while a block of work runs: a host thread reads the GPU's hwmon sensor
    (power1_average, else power1_input; microwatts) every 20 ms.  `watts` stays None when no
    sensor is readable; `cap_watts` is the limit the driver enforces (power1_cap)."""

    def __init__(self):
        import glob
        import torch
        self.path = self.cap_watts = self.watts = None
        want = None
        try:
            pr = torch.cuda.get_device_properties(0)
            want = f"{pr.pci_domain_id:04x}:{pr.pci_bus_id:02x}:{pr.pci_device_id:02x}"
        except Exception:
            pass
        cands = []
        for d in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
            for name in ("power1_average", "power1_input"):
                if os.path.exists(os.path.join(d, name)):
                    cands.append((d, name))
                    break
        if want is not None and len(cands) > 1:
            cands = [c for c in cands if want in os.path.realpath(c[0])] or cands
        if cands:
            self.path = os.path.join(*cands[0])
            try:
                self.cap_watts = int(open(os.path.join(cands[0][0], "power1_cap")).read()) / 1e6
            except Exception:
                pass

    def __enter__(self):
        import threading
        self._stop = False
        self._samples = []

        def loop():
            while not self._stop:
                try:
                    self._samples.append(int(open(self.path).read()))
                except Exception:
                    return
                time.sleep(0.02)
        self._thread = threading.Thread(target=loop, daemon=True) if self.path else None
        if self._thread:
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        if self._thread:
            self._thread.join()
        if self._samples:
            self.watts = round(sum(self._samples) / len(self._samples) / 1e6, 1)
        return False


def power_limit_probe(attention=True):
    """Why the matrix-bound kernel is priced against a peak it cannot be given: the chip lowers its
    clock under the power that toggling operands draw.  (1) A bare loop of the matrix instruction
    the attention uses (lsp_bench_mfma: no memory traffic) on operands that are all 0.5 and on
    N(0,1) operands; (2) the shipped attention kernel on two configuration-4 layers whose Q/K/V are
    all 0.5 and on two layers of the workload's N(0,1) data.  Same instructions, same launches:
    only the values differ."""
    import torch
    import paper_2603_05454_amd as lsp
    import workloads as W
    dev = torch.device("cuda:0")

    def timed(fn, min_ms=300.0, burst=4):
        """Launches go out in bursts of `burst` with no host wait between them (a GPU that idles
        between launches drops its clock), after ~300 ms of the same work as warm-up (the power
        controller averages over a window of that order: shorter runs read high or low depending
        on what ran before)."""
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(burst):
            fn()
        b.record()
        torch.cuda.synchronize()
        for _ in range(int(min_ms / max(a.elapsed_time(b), 1e-3))):
            for _ in range(burst):
                fn()
            torch.cuda.synchronize()
        total, n = 0.0, 0
        with BoardPower() as meter:
            while total < min_ms and n < 100:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(burst):
                    fn()
                b.record()
                torch.cuda.synchronize()
                total += a.elapsed_time(b)
                n += 1
        power[0], power[1] = meter.watts, meter.cap_watts
        return total * 1e-3 / (n * burst)

    res = {}
    power = [None, None]      # board power of the last timed() call, and the driver's limit
    n16 = lsp.MFMA_BENCH_OPERAND_BYTES // 2
    g = torch.Generator().manual_seed(5)
    iters, wgs = 100000, 256
    out = torch.empty(wgs * 512, dtype=torch.float32, device=dev)
    flop = wgs * iters * lsp.MFMA_BENCH_FLOP_PER_WG_ITER
    for name, ops in (("constant_0.5", torch.full((n16,), 0.5, dtype=torch.bfloat16)),
                      ("normal_0_1", torch.randn(n16, generator=g).to(torch.bfloat16))):
        ops = ops.to(dev)
        t = timed(lambda: lsp.bench_mfma(ops, iters, wgs, out))
        res["bare_mfma_loop_TFLOPs_" + name] = round(flop / t / 1e12, 1)
        res["bare_mfma_loop_board_W_" + name] = power[0]
    if attention:
        w = W.scaled(W.C4, layers=2)
        pl, sl = W.make_lengths(w, device=dev)
        fl = W.attn_flops(w) * 2
        for name in ("normal_0_1", "constant_0.5"):
            lay = [W.make_layer_kv(w, l, device=dev) for l in range(2)]
            if name == "constant_0.5":
                for L in lay:
                    for k in L:
                        L[k].fill_(0.5)
            tab = lsp.AttnLayerTable(*[[L[k] for L in lay] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")],
                                     [torch.empty_like(L["q"]) for L in lay])
            t = timed(lambda: lsp.attn_step_layers(tab, pl, sl))
            res["attention_c4_us_per_layer_" + name] = round(t * 1e6 / 2, 1)
            res["attention_c4_TFLOPs_" + name] = round(fl / t / 1e12, 1)
            res["attention_c4_board_W_" + name] = power[0]
            del tab, lay
            torch.cuda.empty_cache()
    if attention:
        for name in ("normal_0_1", "constant_0.5"):
            res["attention_over_bare_loop_" + name] = round(res["attention_c4_TFLOPs_" + name]
                                                            / res["bare_mfma_loop_TFLOPs_" + name], 3)
    res["board_power_limit_W"] = power[1]
    res["note"] = ("identical instruction streams; only the operand values differ: with N(0,1) operands the chip runs the "
                   "matrix pipes at a lower clock to stay inside its power limit, so the bare loop on N(0,1) operands is "
                   "the matrix ceiling this data allows (roofline.frac still uses the published 2500 TFLOP/s); board_W = mean of the "
                   "GPU's hwmon power sensor over the timed launches, board_power_limit_W = the limit the driver enforces")
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {args.gpus} is not supported "
              "(every box has one MI355X and the path has no multi-GPU leg)", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        calibrate_copy()
        return
    if args.calibrate_read:
        calibrate_read()
        return
    if args.calibrate_mfma:
        print(json.dumps({"power_limit_probe": power_limit_probe()}))
        return
    K, Wm = args.steps, args.warmup
    if args.workload == "scatter":
        print(json.dumps({"comparison": "prefix-first vs Scattered-Margin (Section 4.3.3)", "n_gpus": 1, "dtype": "bf16",
                          "data": "synthetic", **run_scatter_comparison(args.layers or 32)}))
        return
    if args.workload == "lmhead":
        print(json.dumps({"comparison": "output head fused with Eq. 1 vs library GEMM + lsp_confidence (Algorithm 1 lines 4-5)",
                          "n_gpus": 1, "dtype": "bf16", "data": "synthetic", **run_lm_head_comparison()}))
        return
    cpu_on = not args.no_cpu_baseline

    def loop_entry():
        value, ms, config, roofline, cpu = run_loop_workload(args.loop_steps, args.sizing, use_graph=bool(args.loop_graph),
                                                             cpu_baseline=cpu_on, flip_trace=bool(args.flip_trace))
        return {"metric": METRIC, "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": config["loop_steps"],
                "warmup": 0, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": config.pop("dtype"), "data": "synthetic", "config": config,
                "roofline": roofline, "cpu_baseline": cpu}

    if args.workload == "c5":
        print(json.dumps(loop_entry()))
        return
    value, ms_per_step, config, roofline, cpu = run_workload(
        args.workload, K, Wm, layers=args.layers, use_graph=bool(args.graph), cpu_baseline=cpu_on)
    line = {
        "metric": METRIC,
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": config.pop("dtype"), "data": "synthetic",
        "config": config, "roofline": roofline, "cpu_baseline": cpu,
    }
    if args.workload == "c4" and not args.layers and args.also == "auto":
        torch.cuda.empty_cache()
        line["roofline"]["power_limit_probe"] = power_limit_probe()
    also = args.also
    if also == "auto":
        also = "c5,c2,c3" if args.workload == "c4" and not args.layers else ""
    side = {}
    for extra in [e for e in also.split(",") if e and e != args.workload]:
        torch.cuda.empty_cache()
        if extra == "c5":
            e = loop_entry()
            line["c5_loop"] = {k: e[k] for k in ("value", "unit", "steps", "ms_per_step", "config", "roofline", "cpu_baseline")}
            continue
        # the small configurations: launch-bound steps, reported next to the headline
        v, ms, cfg, rf, c = run_workload(extra, 100, 10, use_graph=bool(args.graph), cpu_baseline=cpu_on, cpu_budget_s=5.0)
        side[cfg["workload"]] = {"value": round(v, 1), "unit": "tokens/s", "ms_per_step": round(ms, 5), "layers": cfg["layers"],
                                 "committed_tokens_per_step": cfg["committed_tokens_per_step"],
                                 "kernels": rf["all"], "reduction_plus_commit_path": rf["reduction_plus_commit_path"],
                                 "cpu_baseline": c}
    if side:
        line["side"] = side
    print(json.dumps(line))


if __name__ == "__main__":
    main()
