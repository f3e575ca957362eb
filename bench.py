#!/usr/bin/env python3
"""Benchmark of the LSP per-step hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input:
lsp_attn_step for every layer of the workload, lsp_confidence over the logits,
lsp_commit (boundary search + snap + token commit + KV append for every layer).
Inputs are resident in HBM before the timed region.  To keep the Infinity Cache
from serving re-reads, steps rotate over several independent input sets whose
total size exceeds 256 MB, and every step gets fresh (prefix_len, suffix_len)
arrays so that no restore kernel sits in the timed region.

Prints ONE JSON line (see the field list at the bottom of this file).
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MALL_BYTES = 256 << 20

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (one counter per run,
# FETCH scaled x2 KiB and WRITE x1 KiB by the 1 GiB copy calibration; summary under profiles/):
# (workload, call) -> read + written bytes.  None where no counter run has been made.
_KIB = 1024
MEASURED_TRAFFIC = {
    ("c2", "lsp_confidence"): (31693.7 * 2 + 24.0) * _KIB,
    ("c2", "lsp_attn_step"): (7262.1 * 2 + 2048.0) * _KIB,
    ("c2", "lsp_commit"): ((912.5 + 13.1) * 2 + 1796.0 + 0.9) * _KIB,
    ("c3", "lsp_confidence"): (304247.0 * 2 + 192.3) * _KIB,
    ("c3", "lsp_attn_step"): (13467.1 * 2 + 14416.2) * _KIB,
    ("c4", "lsp_confidence"): (1011977.1 * 2 + 770.1) * _KIB,
    ("c4", "lsp_attn_step"): (360623.2 * 2 + 65554.4) * _KIB,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "scatter", "lmhead"],
                    help="c1..c4: one step; c5: the decode loop; scatter: prefix-first against Scattered-Margin commits; "
                         "lmhead: output head fused with the confidence reduction against library GEMM + lsp_confidence")
    ap.add_argument("--sizing", default="tau", choices=["tau", "adaptive", "full"],
                    help="c5: fixed threshold (default), adaptive threshold (Eq. 2, [0.25, 0.5]) or the Full baseline (1 position per step)")
    ap.add_argument("--loop-steps", type=int, default=0, help="c5: stop the decode loop after this many steps (0 = run to the end)")
    ap.add_argument("--layers", type=int, default=0, help="override the workload's layer count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--also", default="c3,c4", help="comma list of further workloads timed briefly (\"\" = none)")
    ap.add_argument("--calibrate-copy", action="store_true", help="only run the 1 GiB copy used to scale HBM counters")
    ap.add_argument("--overlap", type=int, default=0,
                    help="1: run lsp_attn_step on a second stream beside lsp_confidence (measured: the two "
                         "cross-stream joins per step cost more than the overlap gains at c2, and gain <1%% at c4)")
    ap.add_argument("--graph", type=int, default=1, help="replay the step from a HIP graph (1) or launch eagerly (0)")
    ap.add_argument("--loop-graph", type=int, default=0,
                    help="c5: replay every step after the first from one captured HIP graph (measured: no faster than "
                         "eager launches, the loop is bound by the attention kernels)")
    return ap.parse_args()


def run_workload(name, K, Wm, layers=0, use_graph=True, cpu_baseline=True, overlap=False):
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
        layers = [W.make_layer_kv(wr, l, device=dev) for l in range(w.layers)]
        table = lsp.LayerTable([L["k_suf"] for L in layers], [L["v_suf"] for L in layers],
                               [L["k_cache"] for L in layers], [L["v_cache"] for L in layers])
        sets.append(dict(z=z, layers=layers, table=table, tokens=W.make_tokens(wr, w.C).to(dev),
                         attn_out=torch.empty_like(layers[0]["q"])))
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
    ws_bytes = max(lsp.confidence_workspace_bytes(w.B, w.S, w.V),
                   lsp.attn_workspace_bytes(lsp.LSP_BF16 if w.dtype == "bf16" else lsp.LSP_F32, w.B, w.S, w.Hq, w.Hkv, w.D, w.C), 256)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    workspace_attn = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)   # the two calls may run side by side
    side = torch.cuda.Stream() if overlap else None                        # default priority

    def attn(s, pl, sl):
        for L in s["layers"]:
            lsp.attn_step(L["q"], L["k_suf"], L["v_suf"], L["k_cache"], L["v_cache"], pl, sl,
                          out=s["attn_out"], workspace=workspace_attn)

    def conf(s, sl):
        lsp.confidence(s["z"], sl, out=conf_out, workspace=workspace)

    def commit(s, pl, sl, out):
        lsp.commit(conf_out[2], conf_out[0], bitmap, w.V, w.tau, w.window, w.min_commit, 1, pl, sl,
                   tokens=s["tokens"], layers=s["table"], out=out)

    def step(i):
        s = sets[i % R]
        if side is None:
            attn(s, PL[i], SL[i])
            conf(s, SL[i])
        else:
            # attention (K/V, lengths) and confidence (logits, lengths) share no data: the attention of
            # every layer goes to a second stream and joins before the commit, which writes the caches
            main = torch.cuda.current_stream()
            side.wait_stream(main)
            with torch.cuda.stream(side):
                attn(s, PL[i], SL[i])
            conf(s, SL[i])
            main.wait_stream(side)
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
    wall = time.perf_counter() - t0
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
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        if g is not None:
            g.replay()
        else:
            for i in range(reps):
                fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    reps = max(20, min(K, 200))
    scratch_pl, scratch_sl = PL[n_state], SL[n_state]

    def reset_state():
        scratch_pl.copy_(pl0)
        scratch_sl.copy_(sl0)

    t_attn = time_call(lambda i: attn(sets[i % R], pl0, sl0), reps) / max(1, w.layers)
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
    flops_layer = W.attn_flops(w)
    append_bytes = 2 * L0 * w.Hkv * w.D * es * 2 * w.layers
    # the attention is bound by the matrix cores only above the machine balance (2.5 PFLOP/s over
    # 8 TB/s = 312 flop per byte); below it - a short suffix over a short prefix - by HBM
    attn_bytes = (2 * w.B * (w.P + w.S) * w.Hkv * w.D + 2 * w.B * w.S * w.Hq * w.D) * es
    attn_peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 157.3
    if flops_layer / attn_bytes >= attn_peak * 1e12 / (HBM_PEAK_GBS * 1e9):
        attn_entry = {"s": t_attn, "bound": "mfma", "achieved": flops_layer / t_attn / 1e12, "peak": attn_peak, "unit": "TFLOP/s"}
    else:
        attn_entry = {"s": t_attn, "bound": "hbm", "achieved": attn_bytes / t_attn / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    kernels = {
        "lsp_attn_step": attn_entry,
        "lsp_confidence": {"s": t_conf, "bound": "hbm", "achieved": conf_bytes / t_conf / 1e9,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s"},
        "lsp_commit": {"s": t_commit, "bound": "hbm", "achieved": append_bytes / max(t_commit, 1e-9) / 1e9,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s"},
    }
    share = {"lsp_attn_step": t_attn * w.layers, "lsp_confidence": t_conf, "lsp_commit": t_commit}
    dom = max(share, key=share.get)
    kd = kernels[dom]
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": round(kd["achieved"], 2), "peak": kd["peak"],
                "unit": kd["unit"], "frac": round(kd["achieved"] / kd["peak"], 4),
                "traffic": MEASURED_TRAFFIC.get((name, dom)), "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, profiles/)",
                "avg_launch_us": round(kd["s"] * 1e6, 2),
                "all": {k: {"avg_us": round(v["s"] * 1e6, 2), "bound": v["bound"], "achieved": round(v["achieved"], 2),
                            "unit": v["unit"], "frac": round(v["achieved"] / v["peak"], 4)} for k, v in kernels.items()}}

    # ---- oracle on the host cores ---------------------------------------------------
    cpu = None
    if cpu_baseline:
        import oracle
        s = sets[0]
        nl = min(w.layers, 1)
        hz = s["z"].cpu()
        hl = [{k: v.cpu() for k, v in L.items()} for L in s["layers"][:nl]]
        bm = bitmap.cpu()
        pl, sl, tok = pl0.cpu().clone(), sl0.cpu().clone(), s["tokens"].cpu().clone()
        # attention rows: every row when the layer is small, else a seeded sample scaled up
        total_rows = w.B * w.S * w.Hq
        n_rows = total_rows if W.attn_flops(w) < 8e9 else 4096
        g = torch.Generator().manual_seed(1)
        rows = None
        if n_rows < total_rows:
            rows = torch.stack([torch.randint(0, w.B, (n_rows,), generator=g), torch.randint(0, w.S, (n_rows,), generator=g),
                                torch.randint(0, w.Hq, (n_rows,), generator=g)], 1).to(torch.int32)
        # confidence rows: all when < 64M logits, else the first rows up to that
        zr = hz if hz.numel() <= (64 << 20) else hz[:, : max(1, (64 << 20) // (w.B * w.V))].contiguous()
        # repeat the step (state restored each time) until about 10 s of CPU work are spent
        t_attn_c = t_conf_c = t_commit_c = 0.0
        passes = 0
        begin = time.perf_counter()
        while passes < 40 and (passes == 0 or time.perf_counter() - begin < 10.0):
            pl, sl, tok = pl0.cpu().clone(), sl0.cpu().clone(), s["tokens"].cpu().clone()
            caches = [(L["k_cache"].clone(), L["v_cache"].clone()) for L in hl]
            c0 = time.perf_counter()
            for L in hl:
                oracle.attention(L["q"], L["k_suf"], L["v_suf"], L["k_cache"], L["v_cache"], pl, sl, rows=rows)
            c1 = time.perf_counter()
            ids_r, p_r, m_r = oracle.confidence(zr)
            c2 = time.perf_counter()
            if zr.shape[1] != w.S:      # commit needs all rows: fill the rest from the GPU result
                ids_f, m_f = conf_out[0].cpu(), conf_out[2].cpu()
                ids_f[:, : zr.shape[1]] = ids_r
                m_f[:, : zr.shape[1]] = m_r
                ids_r, m_r = ids_f, m_f
            c3 = time.perf_counter()
            oc = oracle.commit(m_r, ids_r, bm, w.V, w.tau, w.window, w.min_commit, 1, pl, sl, tokens=tok,
                               k_suf=[L["k_suf"] for L in hl], v_suf=[L["v_suf"] for L in hl],
                               k_cache=[c[0] for c in caches], v_cache=[c[1] for c in caches])
            c4 = time.perf_counter()
            t_attn_c += c1 - c0
            t_conf_c += c2 - c1
            t_commit_c += c4 - c3
            passes += 1
        spent = time.perf_counter() - begin
        t_full = (t_attn_c * (total_rows / n_rows) * (w.layers / max(nl, 1)) + t_conf_c * (w.S / zr.shape[1])
                  + t_commit_c * (w.layers / max(nl, 1))) / passes
        cpu = {"value": round(float(oc["commit_len"].sum()) / t_full, 2), "unit": "tokens/s",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": (f"{passes} pass(es) over one step of input set 0: attention {n_rows}/{total_rows} (b,i,h) rows x {nl}/{w.layers} layers, "
                          f"confidence {zr.shape[1]}/{w.S} rows per sequence, commit in full; "
                          "sampled parts scaled to the whole step"),
               "ms_per_step": round(t_full * 1e3, 2), "cpu_seconds_spent": round(spent, 2)}

    config = {"workload": w.name, "B": w.B, "layers": w.layers, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
              "P": w.P, "S": w.S, "C": w.C, "V": w.V, "tau": w.tau, "window": w.window,
              "input_sets_rotated": R, "committed_tokens_per_step": round(committed / K, 2),
              "launch": ("hip_graph" if graph is not None else "eager") + (", attention on a second stream beside confidence" if overlap else ""),
              "event_ms_per_step": round(ev0.elapsed_time(ev1) / K, 5), "dtype": w.dtype}
    return value, ms_per_step, config, roofline, cpu


def run_loop_workload(max_steps=0, sizing="tau", use_graph=True):
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
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    r = decode_loop(fn, bitmap.to(dev), w.V, tau, w.window, w.min_commit, 1, pl, sl, tokens,
                    kv_layers=layers, gen_len=w.gen_len, run_attention=True, timed=True,
                    stop_after=max_steps or None, commit_kw=kw, graph=use_graph)
    wall = time.perf_counter() - t0
    lsp_s = r["lsp_ms"] * 1e-3
    config = {"workload": w.name, "B": w.B, "layers": w.layers, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
              "P": w.P, "gen_len": w.gen_len, "C": w.C, "V": w.V, "tau": tau, "window": w.window, "sizing": sizing,
              "loop_steps": r["steps"], "committed_tokens": r["committed"], "flips": r["flips"],
              "flip_rate": round(r["flips"] / max(1, r["flip_denominator"]), 5),
              "ms_at_steps": {str(i): round(r["lsp_ms_steps"][i], 3)
                              for i in sorted({0, 1, r["steps"] // 4, r["steps"] // 2, 3 * r["steps"] // 4, r["steps"] - 1})},
              "lsp_seconds": round(lsp_s, 4), "wall_seconds_with_logit_generator": round(wall, 2),
              "launch": ("first step eager, then one HIP graph replayed per step" if use_graph else "eager") +
                        ", one termination poll per step", "dtype": w.dtype}
    return r["committed"] / lsp_s, r["lsp_ms"] / max(1, r["steps"]), config


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
    K, Wm = args.steps, args.warmup
    if args.workload == "scatter":
        print(json.dumps({"comparison": "prefix-first vs Scattered-Margin (Section 4.3.3)", "n_gpus": 1, "dtype": "bf16",
                          "data": "synthetic", **run_scatter_comparison(args.layers or 32)}))
        return
    if args.workload == "lmhead":
        print(json.dumps({"comparison": "output head fused with Eq. 1 vs library GEMM + lsp_confidence (Algorithm 1 lines 4-5)",
                          "n_gpus": 1, "dtype": "bf16", "data": "synthetic", **run_lm_head_comparison()}))
        return
    if args.workload == "c5":
        value, ms, config = run_loop_workload(args.loop_steps, args.sizing, use_graph=bool(args.loop_graph))
        print(json.dumps({"metric": "committed tokens/sec + per-step latency (ms), LLaDA-8B shape, 1 MI355X",
                          "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": config["loop_steps"],
                          "warmup": 0, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": config.pop("dtype"), "data": "synthetic", "config": config,
                          "roofline": None, "cpu_baseline": None}))
        return
    value, ms_per_step, config, roofline, cpu = run_workload(
        args.workload, K, Wm, layers=args.layers, use_graph=bool(args.graph),
        cpu_baseline=not args.no_cpu_baseline, overlap=bool(args.overlap))
    # the same path at the larger shapes, where the kernels are bandwidth / matrix-core bound
    # rather than launch bound (fewer steps; reported next to the headline workload)
    at_scale = {}
    for extra in [e for e in args.also.split(",") if e and e != args.workload]:
        torch.cuda.empty_cache()
        v, ms, cfg, rf, _ = run_workload(extra, 10, 5, use_graph=bool(args.graph), cpu_baseline=False, overlap=bool(args.overlap))
        at_scale[cfg["workload"]] = {"value": round(v, 1), "ms_per_step": round(ms, 5), "layers": cfg["layers"],
                                     "committed_tokens_per_step": cfg["committed_tokens_per_step"],
                                     "kernels": rf["all"]}
    line = {
        "metric": "committed tokens/sec + per-step latency (ms), LLaDA-8B shape, 1 MI355X",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": config.pop("dtype"), "data": "synthetic",
        "config": config, "roofline": roofline, "cpu_baseline": cpu, "at_scale": at_scale,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
