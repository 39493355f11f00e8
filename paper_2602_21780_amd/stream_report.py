#!/usr/bin/env python3
"""Secondary measurements of the streaming step (one GPU): the other workload shapes, and the constant-cost
claim of the method against an uncompressed cache (paper Sec. 3.2: once the budget is reached, memory and
per-frame cost stay constant; Sec. 4.4 reports the same comparison on video streams).

    python -m paper_2602_21780_amd.stream_report --configs 0,1,2,4
    python -m paper_2602_21780_amd.stream_report --long 200
    python -m paper_2602_21780_amd.stream_report --granularity
    python -m paper_2602_21780_amd.stream_report --selector-sweep
    python -m paper_2602_21780_amd.stream_report --frame-attention
    python -m paper_2602_21780_amd.stream_report --requant-study 300

`--configs`: frames/s of each listed workload at its saturated cache, layer by layer through xsv_step
(overlap mode 2, one xsv_join per frame), events on the launch stream around each frame's 24 (or 1) steps.
`--long N`: the 24-layer drifting stream for N frames, once with the 4-bit budgeted cache and once with an
unbounded bf16 cache (kv_bits 16, budget 0); prints ms/frame and cache bytes at checkpoints.
`--granularity`: mean squared error of the two grouping directions of the quantizer (per token: groups of G
channels; per channel: groups of G tokens) on the synthetic keys (with their outlier channels) and values, at
4 and 2 bits, G = 64 — the analogue of the paper's Table 1 (Sec. 3.3), through xsv_quantize_k / xsv_quantize_v.
`--selector-sweep`: one layer of the 24-layer workload's shape on the drifting stream, stepped side by side with an
unbounded bf16 cache; prints the relative RMS difference of the attention outputs (mean over the frames after
saturation) for token budgets 2748 (first + current only) .. 8192, pooling sizes 4 / 16 / 64, the per-head
selector (score_mode 1), pruning without quantization and quantization without pruning — the analogue of the
paper's cache-length ablation (Sec. 4.5) with output error standing in for the task metrics.
`--frame-attention`: the frame-wise attention of the alternating backbone (xsv_frame_attend: a frame's tokens over
themselves) at 1374 and 1041 tokens, 16 heads: time per launch over 24 x 20 launches issued back to back.
`--requant-study N`: one layer of the long stream for N frames: how many retained rows a re-quantization step leaves
bit-identical, the error of cached rows against the rows the frames delivered by time spent in the cache, and the
number of parameter rows a cache that quantized every token only once would have to keep (Sec. 3.3).
Inputs are synthetic (seeded), generated on the device outside the timed regions.  One JSON line per row.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def cache_bytes(spec, T):
    D = spec.n_heads * spec.head_dim
    per = 2.0 if spec.kv_bits == 16 else spec.kv_bits / 8.0 + 8.0 / spec.group_size
    return 2 * T * D * per * spec.n_layers


def run_stream(spec, frames, checkpoints, torch, xsv, FrameSource, window=5, score_mode=0, value_mode=0):
    """Steps `frames` frames; returns rows (frame, ms/frame averaged over the `window` frames ending there)."""
    dev = "cuda:0"
    L, n = spec.n_layers, spec.tokens_per_frame
    ctx = xsv.Context.from_spec(spec, max_frames=frames + 1, score_mode=score_mode, value_mode=value_mode)
    ctx.set_overlap(2)
    src = FrameSource(spec, dev)
    out = torch.empty((L, spec.n_heads, n, spec.head_dim), dtype=torch.bfloat16, device=dev)
    times, rows = [], []
    for f in range(frames):
        q, k, v = src.frame(f)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for l in range(L):
            ctx.step(l, q[l], k[l], v[l], out[l])
        ctx.join()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
        if (f + 1) in checkpoints:
            w = times[-window:]
            T = ctx.cache_len(0)
            rows.append({"frame": f + 1, "ms_per_frame": round(sum(w) / len(w), 4), "cache_tokens": T,
                         "cache_MB": round(cache_bytes(spec, T) / 1e6, 1), "attend_workgroups": ctx.last_attend_workgroups()})
    ctx.destroy()
    return rows


def granularity_table(torch, xsv, FrameSource, CONFIGS, G=64):
    """MSE of (codes - zero) * scale against the bf16 input for both grouping directions."""
    spec = CONFIGS[2]
    src = FrameSource(spec, "cuda:0", layers=[0])
    frames = [src.frame(f) for f in range(3)]
    rows = []
    for name, idx in (("keys", 1), ("values", 2)):
        x = torch.cat([fr[idx][0] for fr in frames], dim=1).contiguous()       # [H][3n][64] bf16
        xf = x.float()
        T = x.shape[1]
        for bits in (4, 2):
            mse = {}
            for label, fn in (("per_token", xsv.quantize_v), ("per_channel", xsv.quantize_k)):
                codes, scale, zero = fn(x, bits, G)
                if label == "per_channel":                                        # [H][ceil(T/G)][64] -> tokens
                    scale, zero = (t.repeat_interleave(G, dim=1)[:, :T] for t in (scale, zero))
                else:                                                             # [H][T][64/G] -> channels
                    scale, zero = (t.repeat_interleave(G, dim=2) for t in (scale, zero))
                xhat = (codes.float() - zero) * scale
                mse[label] = float(((xhat - xf) ** 2).mean())
            rows.append({"tensor": name, "bits": bits, "group_size": G, "tokens": T, "mse_per_token": mse["per_token"],
                         "mse_per_channel": mse["per_channel"],
                         "ratio_token_over_channel": round(mse["per_token"] / mse["per_channel"], 3)})
    return rows


def selector_sweep(torch, xsv, FrameSource, CONFIGS, frames=14):
    """Output difference against the uncompressed cache for variants of budget, pooling size, selector and width."""
    base = CONFIGS[2].with_(n_layers=1, frames=frames)
    n = base.tokens_per_frame
    variants = [("budget 4096, 4-bit, g 16 (the benchmarked setting)", {})]
    variants += [(f"budget {b}", {"budget": b}) for b in (2 * n, 6144, 8192)]
    variants += [(f"pooling size {g}", {"pool_size": g}) for g in (4, 64)]
    variants += [("per-head selection", {"score_mode": 1}),
                 ("pruning only (bf16 cache)", {"kv_bits": 16}),
                 ("quantization only (unbounded 4-bit cache)", {"budget": 0}),
                 ("budget 4096, 2-bit", {"kv_bits": 2})]
    src = FrameSource(base, "cuda:0", layers=[0])
    inputs = [src.frame(f) for f in range(frames)]
    ref_ctx = xsv.Context.from_spec(base, budget=0, kv_bits=16, max_frames=frames + 1)
    ref_out = [ref_ctx.step(0, q[0], k[0], v[0]).float() for q, k, v in inputs]
    torch.cuda.synchronize()
    ref_ctx.destroy()
    rows = []
    for label, over in variants:
        ctx = xsv.Context.from_spec(base, max_frames=frames + 1, **over)
        errs, T = [], 0
        for f, (q, k, v) in enumerate(inputs):
            out = ctx.step(0, q[0], k[0], v[0]).float()
            if f >= frames - 6:
                errs.append(float(((out - ref_out[f]) ** 2).mean().sqrt() / (ref_out[f] ** 2).mean().sqrt()))
            T = ctx.cache_len(0)
        spec = base.with_(**{k_: v_ for k_, v_ in over.items() if k_ in ("budget", "kv_bits")})
        rows.append({"variant": label, "cache_tokens": T, "cache_MB_per_layer": round(cache_bytes(spec, T) / 1e6, 2),
                     "rel_rms_vs_uncompressed": round(sum(errs) / len(errs), 4), "frames_averaged": len(errs)})
        ctx.destroy()
    return rows


def requant_study(torch, xsv, FrameSource, CONFIGS, frames):
    """What re-quantizing the whole retained cache every step (Sec. 3.3: quantization is applied to the final cache
    of a step) does to tokens that stay for many steps, on one layer of the long drifting stream:
      - how many retained value rows / key groups come out of a step bit-identical to what went in (a row that does
        is a fixed point: carrying its codes over would give the same bytes);
      - the error of the cached (dequantized) rows against the ORIGINAL bf16 rows the frames delivered, by how long
        a token has been cached - against the error of a single quantization (tokens of the newest frame);
      - what a cache that quantized every token ONCE (immutable key groups of 64 consecutive tokens of a frame) would
        have to keep: the number of distinct (frame, group) parameter rows its retained middle tokens point to.
    Runs on the device through xsv_step / xsv_cache_export; the bookkeeping is host-side numpy."""
    import numpy as np
    from paper_2602_21780_amd.inputs import to_u16
    spec = CONFIGS[3].with_(n_layers=1, frames=frames)
    n, H, G = spec.tokens_per_frame, spec.n_heads, spec.group_size
    ctx = xsv.Context.from_spec(spec)
    src = FrameSource(spec, "cuda:0", layers=[0])
    f32 = lambda u16: (np.asarray(u16, np.uint32) << 16).view(np.float32)
    orig_k = orig_v = None           # [H][T][d] fp32: what the frames delivered for the tokens now cached
    prev = None                      # last step's export, and token ids -> row
    rows = []
    buckets = ((0, 0), (1, 1), (2, 5), (6, 20), (21, 100), (101, 10 ** 9))
    acc = {b: {"k_se": 0.0, "v_se": 0.0, "k_ref": 0.0, "v_ref": 0.0, "count": 0} for b in buckets}
    same_v = same_k = seen_v = seen_k = 0
    once_groups = []
    for f in range(frames):
        q, k, v = src.frame(f)
        ctx.step(0, q[0], k[0], v[0])
        _, keep = ctx.last_selection(0)
        kf, vf = f32(to_u16(k[0])), f32(to_u16(v[0]))
        both_k = kf if orig_k is None else np.concatenate([orig_k, kf], axis=1)
        both_v = vf if orig_v is None else np.concatenate([orig_v, vf], axis=1)
        orig_k, orig_v = both_k[:, keep], both_v[:, keep]
        c = ctx.cache_export(0)
        age = f - c.token_frame                                     # frames a token has been cached
        if prev is not None:
            # rows kept from the previous cache: position in the old cache = keep[i] for keep[i] < T_old
            old = keep[keep < prev.T]
            new_pos = np.nonzero(keep < prev.T)[0]
            v_same = (np.all(c.v_codes[:, new_pos] == prev.v_codes[:, old], axis=2)
                      & np.all(c.v_scale[:, new_pos] == prev.v_scale[:, old], axis=2)
                      & np.all(c.v_zero[:, new_pos] == prev.v_zero[:, old], axis=2))
            same_v += int(v_same.sum()); seen_v += v_same.size
            k_same = np.all(c.k_codes[:, new_pos] == prev.k_codes[:, old], axis=2)     # key rows: codes only
            same_k += int(k_same.sum()); seen_k += k_same.size
        if f >= 5:
            kd, vd = f32(c.k_bf16), f32(c.v_bf16)
            for b in buckets:
                sel = (age >= b[0]) & (age <= b[1])
                if sel.any():
                    a = acc[b]
                    a["k_se"] += float(((kd[:, sel] - orig_k[:, sel]) ** 2).sum()); a["k_ref"] += float((orig_k[:, sel] ** 2).sum())
                    a["v_se"] += float(((vd[:, sel] - orig_v[:, sel]) ** 2).sum()); a["v_ref"] += float((orig_v[:, sel] ** 2).sum())
                    a["count"] += int(sel.sum())
            mid = (np.arange(c.T) >= n) & (np.arange(c.T) < c.T - n)
            once_groups.append(len(set(zip(c.token_frame[mid].tolist(), (c.token_index[mid] // G).tolist()))))
        prev = c
    ctx.destroy()
    rows.append({"study": "bit-identical after a re-quantization step", "frames": frames,
                 "value_rows_identical": round(same_v / max(seen_v, 1), 5), "value_rows_seen": seen_v,
                 "key_rows_with_identical_codes": round(same_k / max(seen_k, 1), 5), "key_rows_seen": seen_k})
    for b in buckets:
        a = acc[b]
        if a["count"]:
            rows.append({"study": "error against the original bf16 rows", "cached_for_frames": f"{b[0]}..{b[1] if b[1] < 10 ** 9 else 'end'}",
                         "tokens_averaged": a["count"], "key_rel_rms": round((a["k_se"] / a["k_ref"]) ** 0.5, 5),
                         "value_rel_rms": round((a["v_se"] / a["v_ref"]) ** 0.5, 5)})
    rows.append({"study": "parameter rows a quantize-once cache would hold for the retained middle (groups of 64 tokens of a frame)",
                 "mean": round(float(np.mean(once_groups)), 1), "max": int(np.max(once_groups)),
                 "middle_tokens": spec.budget - 2 * n, "groups_of_the_regrouped_cache": -(-(spec.budget - 2 * n) // G)})
    return rows


def frame_attention(torch, xsv, FrameSource, CONFIGS, reps=20):
    rows = []
    for cid in (2, 4):
        spec = CONFIGS[cid].with_(n_layers=1)
        n, H = spec.tokens_per_frame, spec.n_heads
        q, k, v = (t[0] for t in FrameSource(spec, "cuda:0", layers=[0]).frame(0))
        ctx = xsv.Context.from_spec(spec)
        out = torch.empty_like(q)
        for _ in range(24):
            ctx.frame_attend(q, k, v, out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(24 * reps):
            ctx.frame_attend(q, k, v, out)
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / (24 * reps)
        flop = 4.0 * n * n * H * spec.head_dim
        rows.append({"kernel": "frame attention", "tokens": n, "heads": H, "us_per_launch": round(us, 2),
                     "GFLOP": round(flop / 1e9, 2), "TFLOPs": round(flop / us / 1e6, 1), "workgroups": ctx.last_attend_workgroups()})
        ctx.destroy()
    return rows


def value_mode_study(torch, xsv, FrameSource, CONFIGS):
    """Values quantized once (value_mode 1) against everything re-quantized every step (0), 24-layer workload at its
    saturated cache: the re-quantize launch with all layers per launch on one stream (events of the library), and
    frames/s layer by layer in both overlap modes (best of three runs of 20 frames)."""
    import time
    spec = CONFIGS[2]
    L, n = spec.n_layers, spec.tokens_per_frame
    src = FrameSource(spec, "cuda:0")
    frames = [src.frame(f) for f in range(28)]
    out = torch.empty((L, spec.n_heads, n, spec.head_dim), dtype=torch.bfloat16, device="cuda:0")
    requant_bytes = 2 * (4096 - n) * 1024 * 0.625 + 4 * n * 1024 + 2 * 4096 * 1024 * 0.625   # per layer, as in bench.py
    rows = []
    for vm in (0, 1):
        ctx = xsv.Context.from_spec(spec, value_mode=vm)
        ctx.set_overlap(0)
        packed = [ctx.pack_layers(q, k, v, out) for (q, k, v) in frames]
        for f in range(8):
            ctx.step_all_layers(packed=packed[f])
        ctx.set_attend_timing(True)
        for f in range(8, 14):
            ctx.step_all_layers(packed=packed[f])
        torch.cuda.synchronize()
        _, sp, rq = ctx.chain_times()
        ctx.destroy()
        row = {"value_mode": vm, "requant_24_layers_us": round(1e3 * rq, 1),
               "requant_GBs": round(L * requant_bytes / (rq * 1e-3) / 1e9, 0)}
        for mode in (2, 1):
            ctx = xsv.Context.from_spec(spec, value_mode=vm)
            ctx.set_overlap(mode)
            pk = [[ctx.pack_step(q[l], k[l], v[l], out[l]) for l in range(L)] for (q, k, v) in frames]
            for f in range(8):
                for l in range(L):
                    ctx.step_packed(l, pk[f][l])
                ctx.join()
            torch.cuda.synchronize()
            best = 0.0
            for _ in range(3):
                t0 = time.perf_counter()
                for f in range(8, 28):
                    for l in range(L):
                        ctx.step_packed(l, pk[f][l])
                    ctx.join()
                torch.cuda.synchronize()
                best = max(best, 20 / (time.perf_counter() - t0))
            row[f"frames_per_s_overlap_{mode}"] = round(best, 1)
            ctx.destroy()
        rows.append(row)
    return rows


def attend_shapes(torch, xsv, FrameSource, CONFIGS, reps=3):
    """Attention and merge kernel spans (library events on the launch stream, the span of an empty event pair taken
    off) for every workgroup shape and number of key ranges per unit, at the saturated cache of the 24-layer
    workload, one layer per launch, nothing running beside it."""
    spec = CONFIGS[2]
    L, n = spec.n_layers, spec.tokens_per_frame
    src = FrameSource(spec, "cuda:0")
    sat = spec.budget // n + 2
    out = torch.empty((L, spec.n_heads, n, spec.head_dim), dtype=torch.bfloat16, device="cuda:0")
    ctx = xsv.Context.from_spec(spec)
    ctx.set_overlap(0)
    for f in range(sat + 1):
        q, k, v = src.frame(f)
        ctx.step_all_layers(q, k, v, out)
    q, k, v = src.frame(sat + 1)
    rows = []
    for variant, shape in ((3, "8 waves x 64 rows"), (2, "8 waves x 32 rows"), (0, "4 waves x 64 rows"), (1, "4 waves x 32 rows")):
        ctx.set_attend_variant(variant)
        for ranges in (0, 1, 2, 3, 4, 5, 6, 8):
            ctx.set_attend_splits(ranges, 0)
            ctx.set_attend_timing(True)
            for _ in range(reps):  # the same frame again: only the time matters, and the cache stays at its saturated length
                for l in range(L):
                    ctx.dequant_attend(l, q[l], k[l], v[l], out[l])
                for l in range(L):
                    ctx.score_prune(l, q[l])
                    ctx.quantize(l, k[l], v[l])
            nl, a, m, e = ctx.attend_times()
            ctx.set_attend_timing(False)
            rows.append({"shape": shape, "key_ranges": ranges or "auto", "workgroups": ctx.last_attend_workgroups(),
                         "attend_us": round(1e3 * (a - e), 1), "merge_us": round(1e3 * max(0.0, m - e), 1),
                         "sum_us": round(1e3 * (a - e + max(0.0, m - e)), 1), "launches": nl})
    ctx.destroy()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="", help="comma-separated workload ids of inputs.CONFIGS")
    ap.add_argument("--frames", type=int, default=0, help="frames per workload for --configs (0 = saturation + 12)")
    ap.add_argument("--score-mode", type=int, default=0, choices=(0, 1),
                    help="for --configs: 0 = one retained set per layer (the paper's score), 1 = one per head")
    ap.add_argument("--value-mode", type=int, default=0, choices=(0, 1),
                    help="for --configs: 0 = everything re-quantized every step, 1 = values quantized once")
    ap.add_argument("--long", type=int, default=0, help="frames of the long-stream comparison (0 = skip)")
    ap.add_argument("--granularity", action="store_true", help="per-token vs per-channel quantization error table")
    ap.add_argument("--frame-attention", action="store_true", help="time the frame-wise attention entry point")
    ap.add_argument("--selector-sweep", action="store_true", help="output error against an uncompressed cache per variant")
    ap.add_argument("--requant-study", type=int, default=0, metavar="FRAMES",
                    help="fixed points, error drift and the cost of quantizing once, over FRAMES frames of one layer")
    ap.add_argument("--value-mode-study", action="store_true",
                    help="re-quantize time and frames/s with values quantized once against re-quantized every step")
    ap.add_argument("--attend-shapes", action="store_true",
                    help="attention / merge time per workgroup shape and number of key ranges (24-layer workload)")
    args = ap.parse_args()

    import torch
    from paper_2602_21780_amd import xsv
    from paper_2602_21780_amd.inputs import CONFIGS, FrameSource
    if not torch.cuda.is_available():
        print("stream_report: no GPU visible", file=sys.stderr)
        sys.exit(2)

    for cid in [int(c) for c in args.configs.split(",") if c]:
        spec = CONFIGS[cid]
        n = spec.tokens_per_frame
        sat = (spec.budget // n + 2) if spec.budget else 2
        frames = args.frames or min(spec.frames, sat + 12)
        rows = run_stream(spec, frames, {frames}, torch, xsv, FrameSource, window=max(1, min(10, frames - sat)),
                          score_mode=args.score_mode, value_mode=args.value_mode)
        r = rows[-1]
        print(json.dumps({"workload": spec.name, "layers": spec.n_layers, "tokens_per_frame": n, "budget": spec.budget,
                          "kv_bits": spec.kv_bits, "group_size": spec.group_size, "score_mode": args.score_mode,
                          "value_mode": args.value_mode,
                          "frames_run": frames,
                          "frames_per_s": round(1e3 / r["ms_per_frame"], 2), **r}), flush=True)

    if args.granularity:
        for r in granularity_table(torch, xsv, FrameSource, CONFIGS):
            print(json.dumps(r), flush=True)

    if args.frame_attention:
        for r in frame_attention(torch, xsv, FrameSource, CONFIGS):
            print(json.dumps(r), flush=True)

    if args.value_mode_study:
        for r in value_mode_study(torch, xsv, FrameSource, CONFIGS):
            print(json.dumps(r), flush=True)

    if args.attend_shapes:
        for r in attend_shapes(torch, xsv, FrameSource, CONFIGS):
            print(json.dumps(r), flush=True)

    if args.selector_sweep:
        for r in selector_sweep(torch, xsv, FrameSource, CONFIGS):
            print(json.dumps(r), flush=True)

    if args.requant_study:
        for r in requant_study(torch, xsv, FrameSource, CONFIGS, args.requant_study):
            print(json.dumps(r), flush=True)

    if args.long:
        base = CONFIGS[3]
        marks = {m for m in (10, 25, 50, 100, 200, 500, 1000) if m <= args.long} | {args.long}
        for label, spec in (("4-bit cache, budget 4096", base),
                            ("bf16 cache, unbounded", base.with_(name="cfg3-unbounded-bf16", budget=0, kv_bits=16))):
            for r in run_stream(spec, args.long, marks, torch, xsv, FrameSource):
                print(json.dumps({"stream": label, **r, "frames_per_s": round(1e3 / r["ms_per_frame"], 2)}), flush=True)


if __name__ == "__main__":
    main()
