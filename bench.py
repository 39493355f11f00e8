#!/usr/bin/env python3
"""Benchmark of the streaming step: frames/s of one frame through all 24 global-attention layers
(attend over the budgeted 4-bit cache → score → top-k prune → re-quantize) on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--mode layerwise|batched] [--no-cpu]

Prints one JSON line.  A "step" is one frame of the 24-layer workload (cfg2-24-layer: 16 heads x 64,
1374 tokens per frame, budget 4096, 4-bit, group 64, drifting synthetic stream).  All inputs are
generated on the device before the timed region.  `value` is measured in the layer-by-layer form
(the only one a real model can use, since layer l+1's input depends on layer l's output); the
layer-batched form is reported beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0
# Not measurable from inside this process: HBM bytes per attend_kernel launch of this workload from the two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) summarized in profiles/attend_cfg2_hbm_traffic.md.  Reported under
# "traffic_from_profile" with the profile's date and only for the grid it was measured on; "traffic" itself stays null.
TRAFFIC_PROFILE = {"file": "profiles/attend_cfg2_hbm_traffic.md", "date": "2026-11-28", "workgroups": 240,
                   "fetch_bytes": 24.7e6, "write_bytes": 15.8e6}


def algorithmic_work(spec, Tc, Tn, P):
    """Per layer-step figures: attention flops, and bytes each stage must move."""
    n, D = spec.tokens_per_frame, spec.n_heads * spec.head_dim
    cq = spec.kv_bits / 8.0 + (8.0 / spec.group_size if spec.kv_bits != 16 else 0.0)
    Tk = Tc + n
    return {
        "attend_flop": 4.0 * n * Tk * D,
        "attend_bytes": 2 * n * D * 4 + 2 * Tc * D * cq,           # Q, O, K_t, V_t + packed cache
        "score_bytes": 2 * n * D + P * D * cq + 4 * P,
        "requant_bytes": 2 * (Tn - n) * D * cq + 4 * n * D + 2 * Tn * D * cq,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--mode", choices=["layerwise", "batched"], default="layerwise")
    ap.add_argument("--splits", type=int, default=0, help="key ranges per attention launch (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-steps", type=int, default=24, help="layer-steps the CPU-oracle baseline times (about 0.5 s each)")
    ap.add_argument("--one-form", dest="both_forms", action="store_false",
                    help="skip timing the other launch form (all layers per launch), reported as other_launch_form")
    ap.add_argument("--overlap", type=int, choices=[0, 1, 2], default=2,
                    help="0: prune chain after attention on one stream; 1: on a side stream, joined per call; "
                         "2: side stream, joined lazily (once per frame here)")
    ap.add_argument("--side-cus", type=int, default=-2, help="compute units left to the overlapped prune chain (-2 = library default, -1 = by launch size)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain streaming kernel of known size (1 GiB read + 1 GiB written, 4 times), the yardstick "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--stage-frames", type=int, default=6, help="frames of the per-stage event-timed pass")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one stream per GPU, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_21780_amd import xsv
    from paper_2602_21780_amd.inputs import CONFIGS, FrameSource

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    spec = CONFIGS[2]
    L, n = spec.n_layers, spec.tokens_per_frame
    W, K = max(args.warmup, 5), args.steps   # the cache saturates at the budget after 4 frames
    S = args.stage_frames

    # ---- inputs, resident in HBM before anything is timed -------------------------------------------
    src = FrameSource(spec, dev)
    frames = [src.frame(f) for f in range(max(W + K + 2 * S, 5 + args.cpu_steps))]
    out = torch.empty((L, spec.n_heads, n, spec.head_dim), dtype=torch.bfloat16, device=dev)
    ctx = xsv.Context.from_spec(spec)
    ctx.set_attend_splits(args.splits, args.splits)
    ctx.set_overlap(args.overlap)
    if args.side_cus >= -1:
        ctx.set_side_cus(args.side_cus)
    packed = [ctx.pack_layers(q, k, v, out) for (q, k, v) in frames]
    # one layer's arguments marshalled once per frame buffer (pointers and strides do not change between frames)
    packed_steps = [[ctx.pack_step(q[l], k[l], v[l], out[l]) for l in range(L)] for (q, k, v) in frames]
    torch.cuda.synchronize()

    def run_frame(f, mode):
        if mode == "batched":
            ctx.step_all_layers(packed=packed[f])
        else:
            for l in range(L):
                ctx.step_packed(l, packed_steps[f][l])
        ctx.join()   # the frame's last re-quantization is ordered before whatever follows on the stream

    def timed(mode, f0, count):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for f in range(f0, f0 + count):
            run_frame(f, mode)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def warm(mode):
        ctx.join()
        ctx.reset()
        for f in range(W):
            run_frame(f, mode)

    warm(args.mode)
    Tc = ctx.cache_len(0)
    elapsed = timed(args.mode, W, K)          # THE timed region: exactly K frames
    ms_per_step = elapsed / K * 1e3
    value = K / elapsed
    step_wgs = ctx.last_attend_workgroups()   # attention grid of the timed steps
    Tn = ctx.cache_len(0)
    P = Tc + n - 2 * n
    work = algorithmic_work(spec, Tc, Tn, P)

    # ---- the dominant kernel inside the timed configuration -------------------------------------------------
    # The same K frames again, free-running as above (chain beside attention, joins deferred), now with the
    # library's events around every attention launch on the launch stream: before the attention kernel, between it
    # and the merge kernel, after, and one more right behind (the last pair has nothing between its events: its span
    # is what an event pair itself adds, and is taken off).  These are the launches ms_per_step is made of.
    warm(args.mode)
    ctx.set_attend_timing(True)
    elapsed_with_events = timed(args.mode, W, K)
    n_timed_launches, attend_span_ms, merge_span_ms, event_ms = ctx.attend_times()
    ctx.set_attend_timing(False)
    attend_kernel_ms, merge_kernel_ms = attend_span_ms - event_ms, merge_span_ms - event_ms
    attend_tflops = work["attend_flop"] / (attend_kernel_ms * 1e-3) / 1e12

    # the library's default sequencing (every step joins its chain before it returns), same frames
    default_fps = None
    if args.overlap != 1:
        ctx.set_overlap(1)
        warm(args.mode)
        default_fps = K / timed(args.mode, W, K)
        ctx.set_overlap(args.overlap)

    # the other launch form on the same frames, for context
    other, other_fps = ("batched" if args.mode == "layerwise" else "layerwise"), None
    if args.both_forms:
        warm(other)
        other_fps = K / timed(other, W, K)

    # ---- per-stage durations, each stage alone (nothing beside it), events on the launch stream ------------------
    # Each stage is launched for all 24 layers back to back between two events (the layers are independent of each
    # other), so one event pair brackets 24 launches and its own cost is amortized.
    warm(args.mode)
    ctx.join()
    n_units = spec.n_heads * ((n + 511) // 512)
    if args.splits == 0 and step_wgs % n_units == 0:
        ctx.set_attend_splits(step_wgs // n_units, 0)   # as many key ranges as the timed steps used
    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_ms = {"attend": 0.0, "score_prune": 0.0, "quantize": 0.0}

    def stage_pass(f0):
        marks = []
        for f in range(f0, f0 + S):
            q, k, v = frames[f]
            e = [ev() for _ in range(4)]
            e[0].record()
            for l in range(L):
                ctx.dequant_attend(l, q[l], k[l], v[l], out[l])
            e[1].record()
            for l in range(L):
                ctx.score_prune(l, q[l])
            e[2].record()
            for l in range(L):
                ctx.quantize(l, k[l], v[l])
            e[3].record()
            marks.append(e)
        torch.cuda.synchronize()
        return marks

    marks = stage_pass(W)
    for e in marks:
        stage_ms["attend"] += e[0].elapsed_time(e[1]) / (L * len(marks))
        stage_ms["score_prune"] += e[1].elapsed_time(e[2]) / (L * len(marks))
        stage_ms["quantize"] += e[2].elapsed_time(e[3]) / (L * len(marks))
    ctx.set_attend_timing(True)                    # the same again with the library's events around each kernel
    stage_pass(W + S)
    iso_launches, iso_attend_span, iso_merge_span, iso_event = ctx.attend_times()
    ctx.set_attend_timing(False)
    iso_attend_ms = iso_attend_span - iso_event
    traffic_from_profile = None
    if TRAFFIC_PROFILE["fetch_bytes"] is not None and step_wgs == TRAFFIC_PROFILE["workgroups"]:
        traffic_from_profile = dict(TRAFFIC_PROFILE, bytes=TRAFFIC_PROFILE["fetch_bytes"] + TRAFFIC_PROFILE["write_bytes"],
                                    ratio_to_algorithmic=round((TRAFFIC_PROFILE["fetch_bytes"] + TRAFFIC_PROFILE["write_bytes"]) / work["attend_bytes"], 2))
    roofline = {
        "kernel": "attend_kernel<4,64,8,2>",
        "bound": "mfma", "achieved": round(attend_tflops, 2), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
        "frac": round(attend_tflops / PEAK_BF16_MFMA_TFLOPS, 4),
        "traffic": None, "traffic_from_profile": traffic_from_profile,
        "measured_on": "the launches of a second pass over the timed frames in the timed configuration (chain beside "
                       "attention, deferred joins), events of the library on the launch stream around every launch",
        "algorithmic_bytes": work["attend_bytes"],
        "flop_per_launch": work["attend_flop"], "avg_launch_ms": round(attend_kernel_ms, 4), "launches_timed": n_timed_launches,
        "workgroups": step_wgs,
        "merge_kernel_ms": round(merge_kernel_ms, 4), "event_pair_ms": round(event_ms, 4),
        "attend_plus_merge_TFLOPs": round(work["attend_flop"] / ((attend_kernel_ms + merge_kernel_ms) * 1e-3) / 1e12, 2),
        "frames_per_s_with_events": round(K / elapsed_with_events, 2),
        "isolated": {   # attention launches alone, 24 back to back, nothing running beside them
            "avg_launch_ms": round(iso_attend_ms, 4), "merge_kernel_ms": round(iso_merge_span - iso_event, 4),
            "launches_timed": iso_launches, "TFLOPs": round(work["attend_flop"] / (iso_attend_ms * 1e-3) / 1e12, 2),
            "attend_plus_merge_ms": round(stage_ms["attend"], 4),
        },
    }
    hbm = {
        "score_prune_GBs": round(work["score_bytes"] / (stage_ms["score_prune"] * 1e-3) / 1e9, 1),
        "quantize_GBs": round(work["requant_bytes"] / (stage_ms["quantize"] * 1e-3) / 1e9, 1),
        "score_prune_ms": round(stage_ms["score_prune"], 4), "quantize_ms": round(stage_ms["quantize"], 4),
        "score_bytes": work["score_bytes"], "requant_bytes": work["requant_bytes"], "peak_GBs": PEAK_HBM_GBS,
    }
    hbm["score_prune_frac"] = round(hbm["score_prune_GBs"] / PEAK_HBM_GBS, 4)
    hbm["quantize_frac"] = round(hbm["quantize_GBs"] / PEAK_HBM_GBS, 4)

    # ---- the HBM-bound stages with all 24 layers in one launch each (no overlap: kernel rates) ----------
    ctx.set_attend_splits(args.splits, args.splits)
    ctx.set_overlap(0)
    ctx.reset()
    for f in range(W):
        ctx.step_all_layers(packed=packed[f])
    ctx.set_attend_timing(True)
    for f in range(W, W + S):
        ctx.step_all_layers(packed=packed[f])
    n_chain, sp_ms, rq_ms = ctx.chain_times()
    ctx.set_attend_timing(False)
    hbm["all_layers_per_launch"] = {
        "frames_timed": n_chain,
        "score_prune_ms": round(sp_ms, 4), "quantize_ms": round(rq_ms, 4),
        "score_prune_GBs": round(L * work["score_bytes"] / (sp_ms * 1e-3) / 1e9, 1),
        "quantize_GBs": round(L * work["requant_bytes"] / (rq_ms * 1e-3) / 1e9, 1),
    }
    hbm["all_layers_per_launch"]["score_prune_frac"] = round(hbm["all_layers_per_launch"]["score_prune_GBs"] / PEAK_HBM_GBS, 4)
    hbm["all_layers_per_launch"]["quantize_frac"] = round(hbm["all_layers_per_launch"]["quantize_GBs"] / PEAK_HBM_GBS, 4)

    # ---- the oracle on the host cores, bounded sample ------------------------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import ref
        from paper_2602_21780_amd.inputs import to_u16
        ref.build()
        st = ref.RefStream(1, spec.n_heads, spec.head_dim, n, spec.n_special, spec.budget, spec.kv_bits,
                           spec.group_size, spec.pool_size)
        n_timed = args.cpu_steps
        host = [tuple(to_u16(t[0]) for t in frames[f]) for f in range(5 + n_timed)]
        for f in range(5):                       # reach the saturated cache (not timed)
            st.step(0, *host[f], attend=False)
        t0 = time.perf_counter()
        for f in range(5, 5 + n_timed):          # whole layer-steps: attention of all rows, score, select, quantize
            st.step(0, *host[f])
        t_step = (time.perf_counter() - t0) / n_timed
        cpu = {"value": round(1.0 / (L * t_step), 5), "unit": "frames/s", "cores": ref.num_threads(), "kind": "oracle",
               "sample": f"layer 0 of the same stream at the saturated cache: {n_timed} complete layer-steps (attention of all "
                         f"{n} query rows over {Tc + n} keys, score, select, gather, quantize), {t_step * 1e3:.0f} ms each, "
                         f"{n_timed * t_step:.1f} s in all; a frame is {L} such steps"}
        st.close()

    # the device's own yardsticks: a loop of nothing but the attention kernel's MFMA instruction, a plain copy
    mfma_peak, copy_peak = xsv.measure_peaks()
    roofline["measured_mfma_loop_TFLOPs"] = round(mfma_peak, 1)
    roofline["frac_of_measured_mfma_loop"] = round(attend_tflops / mfma_peak, 4)
    hbm["measured_copy_GBs"] = round(copy_peak, 1)

    result = {
        "metric": "streamed frames/s for 24-layer compressed global-attn step",
        "value": round(value, 2), "unit": "frames/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": spec.name, "layers": L, "heads": spec.n_heads, "head_dim": spec.head_dim,
                   "tokens_per_frame": n, "budget": spec.budget, "kv_bits": spec.kv_bits, "group_size": spec.group_size,
                   "cache_tokens": Tc, "keys_per_step": Tc + n, "launch_form": args.mode,
                   "attend_key_splits": args.splits or "auto", "overlap_mode": args.overlap},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "frames_per_s_default_mode": round(default_fps, 2) if default_fps else None,
        "other_launch_form": {"form": other, "frames_per_s": round(other_fps, 2)} if other_fps else None,
        "attention_TFLOPs_whole_step": round(work["attend_flop"] * L * value / 1e12, 2),
        "hbm_stages": hbm,
    }
    ctx.destroy()
    if args.calibrate_copy:
        src_t = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst_t = torch.empty_like(src_t)
        for _ in range(4):
            torch.mul(src_t, 2.0, out=dst_t)                                # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
