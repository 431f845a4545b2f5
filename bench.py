#!/usr/bin/env python3
"""Benchmark of the Block-attention prefill hot path on one MI355X.

Headline (the metric's configuration): long-context final-block prefill, Llama-3-8B head
shape (32 query / 8 KV heads, head_dim 128, bf16), 31 cached and re-encoded passage blocks
of 1024 tokens plus a 256-token final block, 32 layers with distinct Q/K/V buffers.  One
"step" is the 32-layer loop of ba_final_block_attention calls (RoPE of the final block's
q/k, the MFMA attention core over all 32,000 keys, the split-KV merge), inputs resident in
HBM.  value = algorithmic TFLOP/s = 4 * D * visible (query, key, head) triples / time.

The same run also reports, outside the timed steps:
  * roofline: the attention core's own average launch time from HIP events recorded by the
    library on the launch stream (a second, event-instrumented pass over the same steps);
  * rows: ba_reencode_positions at config 4 (GB/s against HBM), ba_encode_blocks on the
    same 32,000 tokens as a single block (full-attention mode) and on config 3's ragged
    blocks;
  * cpu_baseline: the CPU oracle, as it stands, on a bounded sample of the headline
    workload's rows.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
HBM_PEAK_GBS = 8000.0


NOMINAL_CLOCK_GHZ = 2.4         # the clock the published peaks are quoted at


def visible_pairs_final(t_ctx: int, l_q: int) -> int:
    return l_q * t_ctx + l_q * (l_q + 1) // 2


def kernel_sources_sha16() -> str:
    """Fingerprint of the HIP sources the library is built from: counter readings stored under
    profiles/ are only quoted while it matches the sources they were collected with."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2409_15355_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def stored_counters():
    """profiles/counters.json (rocprofv3 --pmc readings of this benchmark's kernels), or None when it
    is missing or was collected with other kernel sources."""
    path = os.path.join(ROOT, "profiles", "counters.json")
    try:
        c = json.load(open(path))
    except (OSError, ValueError):
        return None
    return c if c.get("csrc_sha16") == kernel_sources_sha16() else None


def parity_figures(got: np.ndarray, ref: np.ndarray) -> dict:
    err = np.abs(got - ref)
    return {"max_abs": float(err.max()), "mean_abs": float(err.mean())}


def phase_budget(args, torch, ba, dev, randn_bf16) -> int:
    """Per-phase budget of the headline kernel by differences: the same geometry (256 query tokens,
    32/8 heads of 128, one workgroup per compute unit) over contexts of 8K to 62K tokens.  The kernel's
    time is linear in the key tiles a workgroup walks: the slope is the steady-state tile period, the
    intercept everything else a launch pays (dispatch, prologue up to the first MFMA, pipeline fill and
    drain, the causal segment's extra cost, epilogue, end of kernel).  Prints one JSON line."""
    hq, hkv, d, lq = 32, 8, 128, 256
    heads = ba.Heads(hq, hkv, d, 500000.0)
    n_layers = 8
    points = []
    for t_ctx in (7936, 15872, 31744, 47616, 63488):
        cu_q, cu_ctx = np.array([0, lq], dtype=np.int32), np.array([0, t_ctx], dtype=np.int32)
        items = ba.ba_schedule_final_block(heads, cu_q, cu_ctx, 256)
        n_splits = items[0].n_splits
        tiles = max((w.ctx_end - w.ctx_begin + w.self_end - w.self_begin + 63) // 64 for w in items)
        L = [dict(kc=randn_bf16(100 + 10 * i, (t_ctx, hkv, d)), vc=randn_bf16(101 + 10 * i, (t_ctx, hkv, d)),
                  q=randn_bf16(102 + 10 * i, (lq, hq, d)), kf=randn_bf16(103 + 10 * i, (lq, hkv, d)),
                  vf=randn_bf16(104 + 10 * i, (lq, hkv, d))) for i in range(n_layers)]
        o = torch.empty((lq, hq, d), dtype=torch.bfloat16, device=dev)
        ws = torch.empty(ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx), dtype=torch.uint8, device=dev)

        def step():
            for t in L:
                ba.ba_final_block_attention(heads, t["q"], t["kc"], t["vc"], t["kf"], t["vf"], o, None, cu_q, cu_ctx,
                                            None, ba.ROPE_APPLY, ws)
        for _ in range(60):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            step()
        e1.record()
        torch.cuda.synchronize()
        call_us = e0.elapsed_time(e1) / (20 * n_layers) * 1e3
        ba.ba_profile_begin(1 << 12)
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        ms, n = ba.ba_profile_end()
        points.append({"context_tokens": t_ctx, "kv_splits": n_splits, "key_tiles_per_workgroup": int(tiles),
                       "attention_kernel_us": round(ms[0] / n[0] * 1e3, 2), "rope_prepass_us": round(ms[1] / n[1] * 1e3, 2),
                       "merge_us": round(ms[2] / max(n[2], 1) * 1e3, 2), "call_us": round(call_us, 2)})
        del L, o, ws
        torch.cuda.empty_cache()
    x = np.array([p["key_tiles_per_workgroup"] for p in points], dtype=np.float64)
    out = {"geometry": "256 query tokens x 32/8 heads x 128, 256 workgroups", "points": points}
    for key in ("attention_kernel_us", "call_us"):
        y = np.array([p[key] for p in points])
        slope, icpt = np.polyfit(x, y, 1)
        out[key + "_fit"] = {"us_per_key_tile": round(float(slope), 4), "fixed_us": round(float(icpt), 2),
                             "largest_residual_us": round(float(np.abs(y - (slope * x + icpt)).max()), 2)}
    c = ((stored_counters() or {}).get("attn_kernel_final_cfg5") or {}).get("clock_ghz")
    if c:
        out["at_sustained_clock_GHz"] = c
        out["cycles_per_key_tile"] = round(out["attention_kernel_us_fit"]["us_per_key_tile"] * c * 1e3)
        out["fixed_cycles"] = round(out["attention_kernel_us_fit"]["fixed_us"] * c * 1e3)
        out["mfma_cycles_per_key_tile_at_full_pipe"] = 2048
    # the same launch from the inside: wave 0 of every workgroup reads the real-time counter at its phase
    # boundaries.  Equal splits and splits sized by the calibration's figures take turns (the clocks settle
    # over the first milliseconds of a busy spell: a column measured behind a pause reads faster than one
    # measured in the middle of the work), and the first turn is left out.
    wsp = torch.empty(ba.ba_measure_xcd_speed_workspace_bytes(), dtype=torch.uint8, device=dev)
    speeds = ba.ba_measure_xcd_speed(wsp)
    turns = {"equal": [], "sized": []}
    for turn in range(5):
        turns["equal"].append(ba.ba_diag_final_block_phases(wsp))
        turns["sized"].append(ba.ba_diag_final_block_phases(wsp, xcd_speed=speeds))
    mean = lambda rows: {k: round(float(np.mean([r[k] for r in rows[1:]])), 2) for k in rows[0]}
    out["marks_inside_one_launch_us"] = mean(turns["equal"])
    out["marks_with_splits_sized_by_xcd_speed_us"] = mean(turns["sized"])
    out["xcd_speed"] = [round(x, 4) for x in speeds]
    out["marks_note"] = ("means over the 256 workgroups of the probe's launches (31,744 context tokens, queries scaled in "
                         "the kernel; four launches per reading, four readings per column, the two columns taking turns); "
                         "the last two are single numbers: the launch, and the longest walk")
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=8)  # (the first six steps run below the steady clock)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rows", action="store_true", help="skip the secondary rows (config 3/4, single block)")
    ap.add_argument("--equal-splits", action="store_true",
                    help="skip the XCD speed calibration: KV splits of equal size")
    ap.add_argument("--phase-budget", action="store_true",
                    help="instead of the benchmark: the attention core's time at the headline geometry over several "
                         "context lengths, and from their differences the time per key tile and the fixed part of a launch")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size reference for HBM byte counters")
    ap.add_argument("--only", default="", help="run only one secondary row in a loop (for profiling): reencode|single|encode3|final3|query50|cfg2|prompts|smallblocks|cached")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_2409_15355_amd import binding as ba
    from paper_2409_15355_amd import workloads as wl
    ba.load()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)

    def randn_bf16(seed, shape):
        g = torch.Generator(device=dev).manual_seed(seed)
        return torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)

    def timed(fn, steps, warmup, per_step=False):
        # a full collection of the interpreter's garbage takes tens of milliseconds in this process
        # and would land in the middle of a timed region every few hundred calls; it runs before the
        # warm-up, so that the GPU does not sit idle (and drop its clock) right before the timed region
        gc.collect()
        gc.disable()
        try:
            # per_step: one event behind every step (no synchronisation between them): the mean over the
            # whole region is the figure reported, the steps' own times give its median and minimum
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            # at least `warmup` calls, and at least about 30 ms of work: the clock needs that long to
            # settle after an idle spell (allocating the next row's tensors is one)
            fn()
            torch.cuda.synchronize()
            t_est = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            est = max(time.perf_counter() - t_est, 1e-6)
            for _ in range(max(warmup - 2, 0, min(3000, int(0.03 / est)))):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            marks[0].record()
            for i in range(steps):
                fn()
                if per_step or i == steps - 1:  # (an event costs microseconds: only where a step lasts milliseconds)
                    marks[i + 1].record()
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3
        finally:
            gc.enable()
        if per_step:
            each = sorted(max(marks[i].elapsed_time(marks[i + 1]), 0.0) for i in range(steps))
            timed.last_median_min = (each[len(each) // 2], each[0], each[-1]) if each else (0.0, 0.0, 0.0)
        return max(marks[0].elapsed_time(marks[-1]), 0.0) / steps, wall_ms / steps

    if args.phase_budget:
        return phase_budget(args, torch, ba, dev, randn_bf16)

    # ------------------------------------------------------------------ headline: config 5
    w = wl.config5(n_layers=args.layers)
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    t_ctx, l_q = w.prompts[0].t_ctx, w.prompts[0].final_len
    cu_q, cu_ctx = w.cu_q(), w.cu_ctx()
    # one-time calibration, as a serving process would do at start-up: the relative speed of the eight
    # XCDs under the attention core's load; the final-block planner sizes its KV splits by it
    xcd_speed = None
    if not args.equal_splits:
        ws_probe = torch.empty(ba.ba_measure_xcd_speed_workspace_bytes(), dtype=torch.uint8, device=dev)
        xcd_speed = ba.ba_measure_xcd_speed(ws_probe)
        del ws_probe
        torch.cuda.empty_cache()
    heads = ba.Heads(hq, hkv, d, w.rope_base, xcd_speed=xcd_speed)
    layers = []
    host0 = None
    for layer in range(w.n_layers):
        if layer == 0 and not args.no_cpu_baseline:
            # layer 0 comes from the host generator so that the oracle sees the same arrays
            host0 = dict(kc=wl.normal_bf16_bits(wl.tensor_seed(5, 0), (t_ctx, hkv, d)),
                         vc=wl.normal_bf16_bits(wl.tensor_seed(5, 1), (t_ctx, hkv, d)),
                         q=wl.normal_bf16_bits(wl.tensor_seed(5, 2), (l_q, hq, d)),
                         kf=wl.normal_bf16_bits(wl.tensor_seed(5, 3), (l_q, hkv, d)),
                         vf=wl.normal_bf16_bits(wl.tensor_seed(5, 4), (l_q, hkv, d)))
            t = {k: dev_bf16(v) for k, v in host0.items()}
        else:
            s = wl.tensor_seed(5, 100 + 10 * layer)
            t = dict(kc=randn_bf16(s, (t_ctx, hkv, d)), vc=randn_bf16(s + 1, (t_ctx, hkv, d)),
                     q=randn_bf16(s + 2, (l_q, hq, d)), kf=randn_bf16(s + 3, (l_q, hkv, d)),
                     vf=randn_bf16(s + 4, (l_q, hkv, d)))
        t["o"] = torch.empty((l_q, hq, d), dtype=torch.bfloat16, device=dev)
        layers.append(t)
    ws_bytes = ba.ba_final_block_attention_workspace_bytes(heads, cu_q, cu_ctx, ba.ROPE_APPLY, False)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step_final():
        for t in layers:
            ba.ba_final_block_attention(heads, t["q"], t["kc"], t["vc"], t["kf"], t["vf"], t["o"], None, cu_q, cu_ctx,
                                        None, ba.ROPE_APPLY, ws)

    if args.only == "":
        ms_step, wall_ms_step = timed(step_final, args.steps, args.warmup, per_step=True)
    else:
        ms_step, wall_ms_step = timed(step_final, 1, 1, per_step=True)
    step_median_ms, step_min_ms, step_max_ms = timed.last_median_min
    flops_layer = 4.0 * d * hq * visible_pairs_final(t_ctx, l_q)
    ms_layer = ms_step / w.n_layers
    tflops = flops_layer / (ms_layer * 1e-3) / 1e12

    # per-kernel times of the same steps, from the library's own events on the launch stream (a few
    # steps without events go first, with no synchronisation in between, so that the recorded ones run
    # at the steady clock like the timed region did)
    prof_steps = min(args.steps, 10) if args.only == "" else 1
    if args.only == "":
        for _ in range(min(args.warmup, 4)):
            step_final()
    ba.ba_profile_begin(1 << 16)
    for _ in range(prof_steps):
        step_final()
    torch.cuda.synchronize()
    prof_ms, prof_n = ba.ba_profile_end()
    attn_us = prof_ms[ba.PROFILE_ATTENTION] / max(prof_n[ba.PROFILE_ATTENTION], 1) * 1e3
    achieved = flops_layer / (attn_us * 1e-6) / 1e12
    # HBM bytes per launch and the sustained shader clock come from committed rocprofv3 --pmc readings
    # (FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB copy; GRBM_GUI_ACTIVE cycles over the kernel's
    # duration); they are quoted only while the kernel sources are the ones they were collected with
    counters = stored_counters()
    head_c = (counters or {}).get("attn_kernel_final_cfg5") or {}
    traffic = head_c.get("bytes_per_launch")
    clock_ghz = head_c.get("clock_ghz")
    roofline = {"bound": "mfma", "kernel": "attn_kernel<128, FinalMeta>", "achieved": round(achieved, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": traffic, "avg_launch_us": round(attn_us, 2),
                "launches_timed": prof_n[ba.PROFILE_ATTENTION],
                "avg_launch_us_kernel_trace": head_c.get("kernel_trace_avg_us"),
                # the same achieved rate against the peak at the clock the part sustains under this load
                "clock_measured": None if not clock_ghz else {
                    "sustained_clock_GHz": clock_ghz,
                    "peak_at_that_clock": round(MFMA_BF16_PEAK_TFLOPS * clock_ghz / NOMINAL_CLOCK_GHZ, 1),
                    "frac": round(achieved / (MFMA_BF16_PEAK_TFLOPS * clock_ghz / NOMINAL_CLOCK_GHZ), 4),
                    "source": "profiles/counters.json"},
                "counters_current": counters is not None,
                "note": "avg_launch_us is bracketed by HIP events on the launch stream, which keep neighbouring "
                        "kernels from overlapping and read up to 5 % above the kernel trace's duration of the "
                        "same kernel (the small kernels about 2 us above): frac is conservative by that much at most",
                "other_kernels_us_per_layer": {
                    "rope_final_block_keys": round(prof_ms[ba.PROFILE_REENCODE] / max(prof_n[ba.PROFILE_REENCODE], 1) * 1e3, 2),
                    "split_combine": round(prof_ms[ba.PROFILE_COMBINE] / max(prof_n[ba.PROFILE_COMBINE], 1) * 1e3, 2)}}

    # ------------------------------------------------------------------ what an MFMA loop sustains here
    # (the library's diagnostic: random bf16 operands, 8 waves per compute unit, with and without an
    # operand fragment from LDS per MFMA; the attention core reads one per MFMA)
    mfma_ceiling = None
    if args.only == "":
        mfma_ceiling = {}
        for name, reads in (("registers_only", 0), ("one_lds_fragment_per_two_mfma", 1), ("one_lds_fragment_per_mfma", 2)):
            r = ba.ba_diag_mfma_ceiling(reads)
            mfma_ceiling[name] = {"TFLOPs": round(r["TFLOPs"], 1), "clock_GHz": round(r["clock_GHz"], 3),
                                  "pipe_busy": round(r["pipe_busy"], 3),
                                  "frac_of_nominal_peak": round(r["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4)}
        roofline["sustained_mfma_loop"] = mfma_ceiling
        roofline["frac_of_sustained_loop_with_lds_operands"] = round(
            achieved / max(mfma_ceiling["one_lds_fragment_per_mfma"]["TFLOPs"], 1e-9), 4)

    # ------------------------------------------------------------------ cpu baseline (oracle)
    cpu_baseline = None
    if host0 is not None and args.only == "":
        import oracle
        f = oracle.bf16_bits_to_f64
        rows = list(range(0, l_q))  # every final-block row of layer 0: 256 rows x 32 heads
        th = oracle.theta(w.rope_base, d)
        kc64, vc64, q64, kf64, vf64 = f(host0["kc"]), f(host0["vc"]), f(host0["q"]), f(host0["kf"]), f(host0["vf"])
        t0 = time.perf_counter()
        ref = oracle.final_block(q64, kc64, vc64, kf64, vf64, cu_q, cu_ctx, th, rows=rows)
        cpu_s = time.perf_counter() - t0
        pairs = sum(t_ctx + r + 1 for r in rows) * hq
        got = layers[0]["o"].float().cpu().numpy().astype(np.float64)[rows]
        err = np.abs(got - ref)
        cpu_baseline = {"value": round(4.0 * d * pairs / cpu_s / 1e12, 6), "unit": "TFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"layer 0, {len(rows)} of {l_q} final-block rows x {hq} heads over all {t_ctx + l_q} keys "
                                  f"({cpu_s:.1f} s)",
                        "parity_on_sample": {"max_abs": float(err.max()), "mean_abs": float(err.mean())}}
        del kc64, vc64
    # ---- the same layers straight from the block cache (re-encoding folded into the attention kernel)
    #      against the two-step route (re-encode the layer's cached K, then the final block)
    cached_row = None
    if not args.no_rows and args.only in ("", "cached"):
        nb = len(w.prompts[0].passage_lens)
        L = t_ctx // nb
        b_off = (np.arange(nb) * L).astype(np.int32)
        b_len = np.full(nb, L, dtype=np.int32)
        cu_blk = np.array([0, nb], dtype=np.int32)
        wsc = torch.empty(ba.ba_final_block_attention_cached_workspace_bytes(heads, cu_q, cu_blk, b_len),
                          dtype=torch.uint8, device=dev)
        k_re = torch.empty_like(layers[0]["kc"])

        def step_cached():
            for t in layers:
                ba.ba_final_block_attention_cached(heads, t["q"], t["kc"], t["vc"], t["kf"], t["vf"], t["o"], None,
                                                   cu_q, cu_blk, b_off, b_len, None, None, None, wsc)

        def step_two():
            for t in layers:
                ba.ba_reencode_positions(heads, t["kc"], k_re, b_off, b_off, b_len, None, b_off, ba.REENC_SHIFT)
                ba.ba_final_block_attention(heads, t["q"], k_re, t["vc"], t["kf"], t["vf"], t["o"], None, cu_q,
                                            cu_ctx, None, ba.ROPE_APPLY, ws)

        n_rep = args.steps if args.only == "" else 10
        ms_c, _ = timed(step_cached, n_rep, 3)
        ms_2, _ = timed(step_two, n_rep, 3)
        cached_row = {"ms_per_layer": round(ms_c / w.n_layers, 5),
                      "TFLOPs": round(flops_layer / (ms_c / w.n_layers * 1e-3) / 1e12, 1),
                      "two_step_ms_per_layer": round(ms_2 / w.n_layers, 5),
                      "note": "31 cached blocks of 1024 tokens at local positions; two-step = ba_reencode_positions "
                              "of the layer's K + ba_final_block_attention"}
        del wsc, k_re
    del layers, ws
    torch.cuda.empty_cache()

    if args.calib_copy:
        # 2^29 bf16 elements = 1 GiB read + 1 GiB written by one elementwise copy kernel
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ secondary rows
    rows_out = {}
    if cached_row is not None:
        rows_out["final_from_block_cache_cfg5"] = cached_row
    if not args.no_rows:
        # a-2 at config 4: 32 layers x 32 passages x 1000 tokens, permuted slots, gather form
        if args.only in ("", "reencode"):
            w4 = wl.config4()
            P, L = 32, 1000
            cache = randn_bf16(wl.tensor_seed(4, 0), (w4.n_layers, P * L, hkv, d))
            host4 = None
            if not args.no_cpu_baseline and args.only == "":
                # layer 0 comes from the host generator, so that the oracle sees the same array
                host4 = wl.normal_bf16_bits(wl.tensor_seed(4, 1), (P * L, hkv, d))
                cache[0].copy_(dev_bf16(host4))
            dst = torch.empty_like(cache)
            src_off = (np.arange(P) * L).astype(np.int32)
            lens = np.full(P, L, dtype=np.int32)
            new_pos0 = w4.extra["new_pos0"]
            h4 = ba.Heads(hkv, hkv, d, w4.rope_base)
            nbytes = 2.0 * cache.numel() * 2
            reps = 20 if args.only == "" else 200

            def gather():
                ba.ba_reencode_positions(h4, cache, dst, src_off, new_pos0, lens, None, new_pos0, ba.REENC_SHIFT)

            def inplace():
                ba.ba_reencode_positions(h4, cache, cache, src_off, src_off, lens, None, new_pos0, ba.REENC_SHIFT)

            ms_g, _ = timed(gather, reps, 3)
            oracle4 = None
            if host4 is not None:
                import oracle
                th4 = oracle.theta(w4.rope_base, d)
                got_bits = dst[0].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
                k64 = oracle.bf16_bits_to_f64(host4)[None]
                t0 = time.perf_counter()
                ref4 = oracle.reencode(k64, src_off, new_pos0, lens, th4, new_pos0=new_pos0)[0]
                cpu4 = time.perf_counter() - t0
                got4 = oracle.bf16_bits_to_f64(got_bits)
                nrm = np.repeat(np.sqrt(ref4[..., 0::2] ** 2 + ref4[..., 1::2] ** 2), 2, axis=-1)
                exact = wl.f32_to_bf16_bits(ref4.astype(np.float32))
                oracle4 = {"seconds_one_layer": round(cpu4, 2), "cores": oracle.num_threads(),
                           "GBps": round(2.0 * host4.size * 2 / cpu4 / 1e9, 3),
                           "sample": "layer 0 of 32 (1/32 of the elements); the other layers hold device-drawn values",
                           "parity_on_sample": {
                               "max_err_over_pair_norm": float((np.abs(got4 - ref4) / np.maximum(nrm, 1e-30)).max()),
                               "fraction_equal_to_rounded_oracle": float((exact == got_bits).mean())}}
                del k64, ref4, got4, nrm, exact
            ms_i, _ = timed(inplace, reps, 3)
            rows_out["reencode_cfg4"] = {"bytes": nbytes, "gather_ms": round(ms_g, 4),
                                         "gather_GBps": round(nbytes / ms_g / 1e6, 1),
                                         "inplace_ms": round(ms_i, 4), "inplace_GBps": round(nbytes / ms_i / 1e6, 1),
                                         "frac_of_hbm_peak": round(nbytes / min(ms_g, ms_i) / 1e6 / HBM_PEAK_GBS, 4)}
            # the other forms of the same pass: every token at its own angle (a cache of un-rotated keys),
            # the half-split pair layout, and fp32 keys (twice the bytes)
            def absolute():
                ba.ba_reencode_positions(h4, cache, dst, src_off, new_pos0, lens, None, new_pos0, ba.REENC_ABSOLUTE)

            h4_half = ba.Heads(hkv, hkv, d, w4.rope_base, rope_layout=ba.ROPE_HALF)

            def half_layout():
                ba.ba_reencode_positions(h4_half, cache, dst, src_off, new_pos0, lens, None, new_pos0, ba.REENC_SHIFT)

            reps_o = max(reps // 2, 5)
            ms_abs, _ = timed(absolute, reps_o, 2)
            ms_half, _ = timed(half_layout, reps_o, 2)
            del dst
            torch.cuda.empty_cache()
            cache32 = cache.float()
            dst32 = torch.empty_like(cache32)
            del cache

            def f32_keys():
                ba.ba_reencode_positions(h4, cache32, dst32, src_off, new_pos0, lens, None, new_pos0, ba.REENC_SHIFT)

            ms_f32, _ = timed(f32_keys, reps_o, 2)
            rows_out["reencode_cfg4"].update({"absolute_mode_GBps": round(nbytes / ms_abs / 1e6, 1),
                                              "half_layout_GBps": round(nbytes / ms_half / 1e6, 1),
                                              "fp32_GBps": round(2 * nbytes / ms_f32 / 1e6, 1),
                                              "oracle": oracle4})
            del cache32, dst32
            torch.cuda.empty_cache()
        # a-1, full-attention mode: the same 32,000 tokens as ONE block
        if args.only in ("", "single"):
            T = t_ctx + l_q
            q = randn_bf16(wl.tensor_seed(5, 20), (T, hq, d))
            k = randn_bf16(wl.tensor_seed(5, 21), (T, hkv, d))
            v = randn_bf16(wl.tensor_seed(5, 22), (T, hkv, d))
            o = torch.empty_like(q)
            kl = torch.empty_like(k)
            offs = np.array([0, T], dtype=np.int32)
            ws_s = torch.empty(ba.ba_encode_blocks_workspace_bytes(heads, offs, ba.ROPE_APPLY, True),
                               dtype=torch.uint8, device="cuda")

            def single():
                ba.ba_encode_blocks(heads, q, k, v, o, kl, offs, ba.ROPE_APPLY, ws_s)

            ms_s, _ = timed(single, 3 if args.only == "" else 10, 1)
            fl = 4.0 * d * hq * (T * (T + 1) // 2)
            rows_out["encode_single_block_32k"] = {"ms_per_layer": round(ms_s, 3), "TFLOPs": round(fl / ms_s / 1e9, 1),
                                                   "frac_of_mfma_peak": round(fl / ms_s / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
            del q, k, v, o, kl, ws_s
            torch.cuda.empty_cache()
        # a-1 on config 3's 160 ragged passage blocks
        if args.only in ("", "encode3"):
            w3 = wl.config3()
            offs3 = w3.passage_block_offsets()
            T3 = int(offs3[-1])
            with_oracle = not args.no_cpu_baseline and args.only == ""
            if with_oracle:  # host-drawn arrays, the same for the oracle
                hb3 = [wl.normal_bf16_bits(wl.tensor_seed(3, i), (T3, h_, d)) for i, h_ in enumerate((hq, hkv, hkv))]
                q, k, v = (dev_bf16(b) for b in hb3)
            else:
                q = randn_bf16(wl.tensor_seed(3, 0), (T3, hq, d))
                k = randn_bf16(wl.tensor_seed(3, 1), (T3, hkv, d))
                v = randn_bf16(wl.tensor_seed(3, 2), (T3, hkv, d))
            o = torch.empty_like(q)
            kl = torch.empty_like(k)
            h3 = ba.Heads(hq, hkv, d, w3.rope_base)
            ws_3 = torch.empty(ba.ba_encode_blocks_workspace_bytes(h3, offs3, ba.ROPE_APPLY, True),
                               dtype=torch.uint8, device="cuda")

            def enc3():
                ba.ba_encode_blocks(h3, q, k, v, o, kl, offs3, ba.ROPE_APPLY, ws_3)

            ms_e, _ = timed(enc3, 20 if args.only == "" else 200, 3)
            lens3 = np.diff(offs3).astype(np.int64)
            fl = 4.0 * d * hq * float((lens3 * (lens3 + 1) // 2).sum())
            byts = 2.0 * T3 * d * (2 * hq + 3 * hkv)  # q, o, k, v read or written once, and one write of k_local
            # issued work: every (128-row tile, 32-key tile) pair the short-block schedule walks is computed
            # in full, masked or not (rows = tokens x query heads of a KV group)
            G3 = hq // hkv
            issued = 0
            for L in lens3.tolist():
                n_rows = L * G3
                for rt in range((n_rows + 127) // 128):
                    last_tok = (min(n_rows, (rt + 1) * 128) - 1) // G3
                    issued += 128 * 32 * (last_tok // 32 + 1)
            fl_issued = 4.0 * d * hkv * issued
            oracle3 = None
            if with_oracle:
                import oracle
                f = oracle.bf16_bits_to_f64
                th3 = oracle.theta(w3.rope_base, d)
                t0 = time.perf_counter()
                ref_o, _ = oracle.encode_blocks(f(hb3[0]), f(hb3[1]), f(hb3[2]), offs3, th3)
                cpu3 = time.perf_counter() - t0
                oracle3 = {"seconds": round(cpu3, 2), "cores": oracle.num_threads(), "TFLOPs": round(fl / cpu3 / 1e12, 5),
                           "sample": "all 160 blocks, every row",
                           "parity_on_sample": parity_figures(o.float().cpu().numpy().astype(np.float64), ref_o)}
                del ref_o, hb3
            rows_out["encode_cfg3_ragged"] = {"ms": round(ms_e, 4), "algorithmic_TFLOPs": round(fl / ms_e / 1e9, 1),
                                              "issued_TFLOPs": round(fl_issued / ms_e / 1e9, 1),
                                              "GBps": round(byts / ms_e / 1e6, 1),
                                              "frac_of_hbm_peak": round(byts / ms_e / 1e6 / HBM_PEAK_GBS, 4),
                                              "bound": "hbm (22 KB per token: q, o, k, v and one write of k_local, against about 100 keys of work each)",
                                              "tokens": T3, "oracle": oracle3}
            del q, k, v, o, kl, ws_3
        # a-3 batched: config 3's eight final blocks (32..128 query tokens over about 4,000 context tokens each)
        if args.only in ("", "final3"):
            w3 = wl.config3()
            cu_q3, cu_ctx3 = w3.cu_q(), w3.cu_ctx()
            Tq, Tc = int(cu_q3[-1]), int(cu_ctx3[-1])
            with_oracle = not args.no_cpu_baseline and args.only == ""
            shapes3 = [(Tq, hq), (Tc, hkv), (Tc, hkv), (Tq, hkv), (Tq, hkv)]
            if with_oracle:
                hf3 = [wl.normal_bf16_bits(wl.tensor_seed(3, 40 + i), (n_, h_, d)) for i, (n_, h_) in enumerate(shapes3)]
                qf3, kc3, vc3, kf3, vf3 = (dev_bf16(b) for b in hf3)
            else:
                qf3, kc3, vc3, kf3, vf3 = (randn_bf16(wl.tensor_seed(3, 40 + i), (n_, h_, d)) for i, (n_, h_) in enumerate(shapes3))
            o3 = torch.empty_like(qf3)
            h3 = ba.Heads(hq, hkv, d, w3.rope_base)
            ws_f3 = torch.empty(max(ba.ba_final_block_attention_workspace_bytes(h3, cu_q3, cu_ctx3, ba.ROPE_APPLY, False), 256),
                                dtype=torch.uint8, device="cuda")

            def fin3():
                ba.ba_final_block_attention(h3, qf3, kc3, vc3, kf3, vf3, o3, None, cu_q3, cu_ctx3, None, ba.ROPE_APPLY, ws_f3)

            ms_f3, _ = timed(fin3, 20 if args.only == "" else 200, 3)
            pairs3 = sum(visible_pairs_final(int(cu_ctx3[n + 1] - cu_ctx3[n]), int(cu_q3[n + 1] - cu_q3[n]))
                         for n in range(len(cu_q3) - 1))
            byts3 = 2.0 * d * (2 * Tc * hkv + 2 * Tq * hkv + 2 * Tq * hq)
            fl3 = 4.0 * d * hq * pairs3
            oracle3f = None
            if with_oracle:
                import oracle
                f = oracle.bf16_bits_to_f64
                t0 = time.perf_counter()
                ref3 = oracle.final_block(f(hf3[0]), f(hf3[1]), f(hf3[2]), f(hf3[3]), f(hf3[4]), cu_q3, cu_ctx3,
                                          oracle.theta(w3.rope_base, d))
                cpu3f = time.perf_counter() - t0
                oracle3f = {"seconds": round(cpu3f, 2), "cores": oracle.num_threads(), "TFLOPs": round(fl3 / cpu3f / 1e12, 5),
                            "sample": "all 8 prompts, every row",
                            "parity_on_sample": parity_figures(o3.float().cpu().numpy().astype(np.float64), ref3)}
                del ref3, hf3
            rows_out["final_cfg3_batched"] = {"ms": round(ms_f3, 4), "TFLOPs": round(fl3 / ms_f3 / 1e9, 1),
                                              "GBps": round(byts3 / ms_f3 / 1e6, 1),
                                              "frac_of_mfma_peak": round(fl3 / ms_f3 / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                                              "frac_of_hbm_peak": round(byts3 / ms_f3 / 1e6 / HBM_PEAK_GBS, 4),
                                              "bound": "at the ridge: %.1f us of MFMA at peak, %.1f us of HBM at peak"
                                                       % (fl3 / MFMA_BF16_PEAK_TFLOPS / 1e6, byts3 / HBM_PEAK_GBS / 1e3),
                                              "query_tokens": Tq, "context_tokens": Tc, "oracle": oracle3f}
            del qf3, kc3, vc3, kf3, vf3, o3, ws_f3
        # the paper's own efficiency shape (Section 3.4): a 50-token query block behind a 32K-token prompt
        if args.only in ("", "query50"):
            Lq5, Tc5 = 50, 32000 - 50
            cu_q5, cu_ctx5 = np.array([0, Lq5], dtype=np.int32), np.array([0, Tc5], dtype=np.int32)
            qf5 = randn_bf16(wl.tensor_seed(5, 50), (Lq5, hq, d))
            kc5 = randn_bf16(wl.tensor_seed(5, 51), (Tc5, hkv, d))
            vc5 = randn_bf16(wl.tensor_seed(5, 52), (Tc5, hkv, d))
            kf5 = randn_bf16(wl.tensor_seed(5, 53), (Lq5, hkv, d))
            vf5 = randn_bf16(wl.tensor_seed(5, 54), (Lq5, hkv, d))
            o5 = torch.empty_like(qf5)
            ws_5 = torch.empty(max(ba.ba_final_block_attention_workspace_bytes(heads, cu_q5, cu_ctx5, ba.ROPE_APPLY, False), 256),
                               dtype=torch.uint8, device="cuda")

            def fin5():
                ba.ba_final_block_attention(heads, qf5, kc5, vc5, kf5, vf5, o5, None, cu_q5, cu_ctx5, None, ba.ROPE_APPLY, ws_5)

            ms_5, _ = timed(fin5, 50 if args.only == "" else 500, 5)
            fl5 = 4.0 * d * hq * visible_pairs_final(Tc5, Lq5)
            rows_out["final_50_query_tokens_32k"] = {"ms_per_layer": round(ms_5, 4), "TFLOPs": round(fl5 / ms_5 / 1e9, 1),
                                                     "GBps": round(2.0 * d * 2 * Tc5 * hkv / ms_5 / 1e6, 1),
                                                     "frac_of_hbm_peak": round(2.0 * d * 2 * Tc5 * hkv / ms_5 / 1e6 / HBM_PEAK_GBS, 4),
                                                     "frac_of_mfma_peak": round(fl5 / ms_5 / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                                                     "note": "50 query tokens over 31,950 context tokens, one layer's K/V (131 MB) read once"}
            del qf5, kc5, vc5, kf5, vf5, o5, ws_5
        # config 2 end to end (10 passages of 200 tokens + 64 query tokens): the three steps one after
        # the other; microseconds each, bound by launch latency and by the host side of the calls
        if args.only in ("", "cfg2"):
            w2 = wl.config2()
            offs2 = w2.passage_block_offsets()
            cu_q2, cu_ctx2 = w2.cu_q(), w2.cu_ctx()
            T2, Lq2 = int(offs2[-1]), int(cu_q2[-1])
            h2 = ba.Heads(hq, hkv, d, w2.rope_base)
            # (small enough to draw on the host always: the oracle then sees the same arrays)
            hb2 = [wl.normal_bf16_bits(wl.tensor_seed(2, i), (n_, h_, d))
                   for i, (n_, h_) in enumerate([(T2, hq), (T2, hkv), (T2, hkv), (Lq2, hq), (Lq2, hkv), (Lq2, hkv)])]
            q2, k2, v2, qf2, kf2, vf2 = (dev_bf16(b) for b in hb2)
            o2, kl2, kre2 = torch.empty_like(q2), torch.empty_like(k2), torch.empty_like(k2)
            of2 = torch.empty_like(qf2)
            ws_e2 = torch.empty(max(ba.ba_encode_blocks_workspace_bytes(h2, offs2, ba.ROPE_APPLY, True), 256),
                                dtype=torch.uint8, device="cuda")
            ws_f2 = torch.empty(max(ba.ba_final_block_attention_workspace_bytes(h2, cu_q2, cu_ctx2, ba.ROPE_APPLY, False), 256),
                                dtype=torch.uint8, device="cuda")
            src2 = offs2[:-1].astype(np.int32)
            len2 = np.diff(offs2).astype(np.int32)

            def enc2():
                ba.ba_encode_blocks(h2, q2, k2, v2, o2, kl2, offs2, ba.ROPE_APPLY, ws_e2)

            def re2():
                ba.ba_reencode_positions(h2, kl2, kre2, src2, src2, len2, None, src2, ba.REENC_SHIFT)

            def fin2():
                ba.ba_final_block_attention(h2, qf2, kre2, v2, kf2, vf2, of2, None, cu_q2, cu_ctx2, None, ba.ROPE_APPLY, ws_f2)

            def all2():
                enc2(); re2(); fin2()

            n2 = 50 if args.only == "" else 500
            ms_e2, _ = timed(enc2, n2, 5)
            ms_r2, _ = timed(re2, n2, 5)
            ms_f2, _ = timed(fin2, n2, 5)
            ms_a2, _ = timed(all2, n2, 5)
            oracle2 = None
            if not args.no_cpu_baseline and args.only == "":
                import oracle
                f = oracle.bf16_bits_to_f64
                th2 = oracle.theta(w2.rope_base, d)
                to64 = lambda t_: t_.float().cpu().numpy().astype(np.float64)
                all2()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ref_o2, ref_kl2 = oracle.encode_blocks(f(hb2[0]), f(hb2[1]), f(hb2[2]), offs2, th2)
                t1 = time.perf_counter()
                # (each step's oracle starts from the bf16 values the device handed on, as the next call does)
                kl_bits = kl2.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
                ref_kre2 = oracle.reencode(f(kl_bits)[None], src2, src2, len2, th2, new_pos0=src2)[0]
                t2 = time.perf_counter()
                kre_bits = kre2.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
                ref_of2 = oracle.final_block(f(hb2[3]), f(kre_bits), f(hb2[2]), f(hb2[4]), f(hb2[5]), cu_q2, cu_ctx2, th2)
                t3 = time.perf_counter()
                nrm2 = np.repeat(np.sqrt(ref_kre2[..., 0::2] ** 2 + ref_kre2[..., 1::2] ** 2), 2, axis=-1)
                oracle2 = {"encode_s": round(t1 - t0, 3), "reencode_s": round(t2 - t1 - 0.0, 3), "final_s": round(t3 - t2, 3),
                           "cores": oracle.num_threads(), "sample": "every row of all three steps",
                           "parity": {"encode": parity_figures(to64(o2), ref_o2),
                                      "reencode_max_err_over_pair_norm": float((np.abs(f(kre_bits) - ref_kre2) / np.maximum(nrm2, 1e-30)).max()),
                                      "final": parity_figures(to64(of2), ref_of2)}}
            rows_out["cfg2_three_steps"] = {"encode_us": round(ms_e2 * 1e3, 1), "reencode_us": round(ms_r2 * 1e3, 1),
                                            "final_us": round(ms_f2 * 1e3, 1), "all_three_us": round(ms_a2 * 1e3, 1),
                                            "oracle": oracle2,
                                            "note": "calls issued back to back from Python; latency-bound, no roofline claim"}
            del q2, k2, v2, o2, kl2, kre2, qf2, kf2, vf2, of2, ws_e2, ws_f2
        # whole prompts in one call: config 3's eight prompts with their query blocks appended
        if args.only in ("", "prompts"):
            w3 = wl.config3()
            prompts = [list(pr.passage_lens) + [pr.final_len] for pr in w3.prompts]
            lens_p = np.array([l for pr in prompts for l in pr], dtype=np.int64)
            offs_p = np.concatenate([[0], np.cumsum(lens_p)]).astype(np.int32)
            cu_blk_p = np.concatenate([[0], np.cumsum([len(pr) for pr in prompts])]).astype(np.int32)
            Tp = int(offs_p[-1])
            q = randn_bf16(wl.tensor_seed(3, 60), (Tp, hq, d))
            k = randn_bf16(wl.tensor_seed(3, 61), (Tp, hkv, d))
            v = randn_bf16(wl.tensor_seed(3, 62), (Tp, hkv, d))
            o = torch.empty_like(q)
            kr = torch.empty_like(k)
            lse = torch.empty((Tp, hq), dtype=torch.float32, device="cuda")
            hp = ba.Heads(hq, hkv, d, w3.rope_base)
            ws_p = torch.empty(ba.ba_block_attention_prompts_workspace_bytes(hp, cu_blk_p, offs_p, ba.ROPE_APPLY, True),
                               dtype=torch.uint8, device="cuda")

            def whole():
                ba.ba_block_attention_prompts(hp, q, k, v, o, kr, lse, cu_blk_p, offs_p, ba.ROPE_APPLY, ws_p)

            ms_w, _ = timed(whole, 20 if args.only == "" else 200, 3)
            pairs = 0.0
            for n, pr in enumerate(prompts):
                pl = np.array(pr[:-1], dtype=np.int64)
                ctx, lf = int(pl.sum()), int(pr[-1])
                pairs += float((pl * (pl + 1) // 2).sum()) + lf * ctx + lf * (lf + 1) // 2
            byts = 2.0 * Tp * d * (2 * hq + 4 * hkv)
            rows_out["whole_prompts_cfg3"] = {"ms": round(ms_w, 4), "algorithmic_TFLOPs": round(4.0 * d * hq * pairs / ms_w / 1e9, 1),
                                              "GBps": round(byts / ms_w / 1e6, 1), "tokens": Tp,
                                              "note": "8 prompts x (20 ragged passages + query block), one call, mask of Section 2.4"}
            # ... and its backward pass (five products per visible pair against the forward's two)
            do = randn_bf16(wl.tensor_seed(3, 63), (Tp, hq, d))
            dq_, dk_, dv_ = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
            ws_b = torch.empty(ba.ba_block_attention_prompts_backward_workspace_bytes(hp, cu_blk_p, offs_p),
                               dtype=torch.uint8, device="cuda")

            def bwd():
                ba.ba_block_attention_prompts_backward(hp, q, k, v, o, lse, do, dq_, dk_, dv_, cu_blk_p, offs_p, ws_b)

            ms_bw, _ = timed(bwd, 20 if args.only == "" else 200, 3)
            rows_out["whole_prompts_backward_cfg3"] = {"ms": round(ms_bw, 4),
                                                       "algorithmic_TFLOPs": round(10.0 * d * hq * pairs / ms_bw / 1e9, 1),
                                                       "note": "gradients of q, k, v for the same prompts; deterministic (no atomics)"}
            del q, k, v, o, kr, lse, ws_p, do, dq_, dk_, dv_, ws_b
        # Appendix A's workload: a prompt of many small state blocks read straight from the block cache
        if args.only in ("", "smallblocks"):
            rng = np.random.Generator(np.random.Philox(wl.tensor_seed(6, 900)))
            n_blk, slot = 512, 64
            lens_s = rng.integers(20, 61, n_blk).astype(np.int32)
            offs_s = (np.arange(n_blk) * slot).astype(np.int32)
            cap, lq_s = n_blk * slot, 64
            kc = randn_bf16(wl.tensor_seed(6, 0), (cap, hkv, d))
            vc = randn_bf16(wl.tensor_seed(6, 1), (cap, hkv, d))
            qf = randn_bf16(wl.tensor_seed(6, 2), (lq_s, hq, d))
            kf = randn_bf16(wl.tensor_seed(6, 3), (lq_s, hkv, d))
            vf = randn_bf16(wl.tensor_seed(6, 4), (lq_s, hkv, d))
            o = torch.empty_like(qf)
            hs = ba.Heads(hq, hkv, d, 500000.0)
            cu_q_s, cu_blk_s = np.array([0, lq_s], dtype=np.int32), np.array([0, n_blk], dtype=np.int32)
            ws_s2 = torch.empty(ba.ba_final_block_attention_cached_workspace_bytes(hs, cu_q_s, cu_blk_s, lens_s),
                                dtype=torch.uint8, device="cuda")

            def small():
                ba.ba_final_block_attention_cached(hs, qf, kc, vc, kf, vf, o, None, cu_q_s, cu_blk_s, offs_s, lens_s,
                                                   None, None, None, ws_s2)

            ms_b, _ = timed(small, 20 if args.only == "" else 200, 3)
            ctx = int(lens_s.sum())
            pairs = lq_s * ctx + lq_s * (lq_s + 1) // 2
            rows_out["final_from_512_small_blocks"] = {"ms": round(ms_b, 4), "context_tokens": ctx, "final_len": lq_s,
                                                       "TFLOPs": round(4.0 * d * hq * pairs / ms_b / 1e9, 1),
                                                       "note": "512 cached blocks of 20-60 tokens (Appendix A's many small state blocks), none rewritten"}

    out = {
        "metric": "final-block prefill TFLOP/s at 32K ctx (ms/layer alongside)",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "ms_per_layer": round(ms_layer, 5),
        "ms_per_layer_median": round(step_median_ms / w.n_layers, 5),
        "ms_per_layer_min": round(step_min_ms / w.n_layers, 5),
        "ms_per_layer_max": round(step_max_ms / w.n_layers, 5),
        "host_wall_ms_per_step": round(wall_ms_step, 4),
        "frac_of_bf16_mfma_peak": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "layers": w.n_layers, "context_blocks": 31, "block_len": 1024,
                   "final_len": l_q, "total_tokens": t_ctx + l_q, "n_q_heads": hq, "n_kv_heads": hkv, "head_dim": d,
                   "rope": "applied to q_f/k_f inside the call", "flops_per_layer": flops_layer,
                   "kv_splits": "sized by measured XCD speed" if xcd_speed else "equal",
                   "xcd_speed": None if not xcd_speed else [round(x, 4) for x in xcd_speed]},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "rows": rows_out,
        "paper_context": {"ttft_block_32k_ms": 45, "ttft_vanilla_32k_ms": 3638, "hardware": "NVIDIA H20 (count unstated), bf16",
                          "note": "whole-model TTFT with a 50-token query; context only"},
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
