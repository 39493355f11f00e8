"""GPU parity of the streaming step against the oracle, frame by frame, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2602_21780_amd import xsv
from paper_2602_21780_amd.inputs import CONFIGS, FrameSource, to_u16
from oracle import ref
import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def cover_rows(n):
    """Sampled query rows that reach every 32-row block of the frame - so every wave of every attention
    workgroup, and both query blocks of a wave, whatever the workgroup shape - plus the special tokens, the
    first patch row and the last row."""
    blocks = [min(b + (7 * (b // 32) + 3) % 32, n - 1) for b in range(0, n, 32)]
    return np.unique(np.array([0, min(4, n - 1), min(5, n - 1), n - 1] + blocks, np.int32))


def run_stream(spec, frames, rows=None, splits=0, short=None, all_rows_from=None, **over):
    """`rows`: the query rows whose attention is compared (None = all); from frame `all_rows_from` on, all."""
    ctx, st = parity.make_pair(spec, **over)
    if splits:
        ctx.set_attend_splits(splits, splits)
    if short is not None:
        ctx.set_short_range(short)
    src = FrameSource(spec, DEV)
    worst = (0.0, 0.0)
    ties = 0
    for f in range(frames):
        q, k, v = src.frame(f)
        for l in range(spec.n_layers):
            print(f"  {spec.name} frame {f} layer {l} T={ctx.cache_len(l)}", flush=True)
            full = all_rows_from is not None and f >= all_rows_from
            (ma, rr), t = parity.step_and_compare(ctx, st, spec, l, l, q[l], k[l], v[l], rows=None if full else rows,
                                                  budget=over.get("budget"))
            worst = (max(worst[0], ma), max(worst[1], rr))
            ties += t
    print(f"  worst max_abs={worst[0]:.3e} rel_rms={worst[1]:.3e} ties={ties}", flush=True)
    ctx.destroy()
    return worst, ties


def test_tiny_config_full_stream():
    """cfg 0: every frame, every row, every exported byte."""
    run_stream(CONFIGS[0], CONFIGS[0].frames)


@pytest.mark.parametrize("splits", [1, 2, 5])
def test_tiny_config_key_range_splits(splits):
    run_stream(CONFIGS[0], 6, splits=splits)


@pytest.mark.parametrize("bits,G", [(4, 64), (2, 64), (2, 32), (16, 64)])
def test_mid_size_streams_all_code_widths(bits, G):
    # several query tiles and key tiles, ragged everywhere: n = 5 + 195, budget not a multiple of 64
    spec = CONFIGS[0].with_(name=f"mid-b{bits}-g{G}", n_heads=3, tokens_per_frame=200, budget=700, kv_bits=bits,
                            group_size=G, n_layers=2, seed=11)
    run_stream(spec, 6)


@pytest.mark.parametrize("short", [0, 10, 60, 100])
def test_short_extra_key_range(short):
    """The overlapped step's cut with one shorter key range per (head, query block), at several lengths."""
    spec = CONFIGS[0].with_(name=f"short{short}", n_heads=2, tokens_per_frame=200, budget=1500, n_layers=2, seed=13)
    run_stream(spec, 10, short=short)


def test_dominant_keys_whose_dequantized_values_are_rounding_ties():
    """A small cache with strong key outliers: single keys dominate the softmax, and (code - zero) * scale lands on
    bf16 midpoints for some of them, so the output shows whether attention reads exactly the cache's canonical view
    (a dequantization that rounds differently moves such a key's weight by a few percent)."""
    spec = CONFIGS[0].with_(name="ties", n_heads=2, tokens_per_frame=150, budget=520, kv_bits=4, group_size=32, n_layers=2, seed=17)
    run_stream(spec, 7)


@pytest.mark.parametrize("seed", range(30, 38))
@pytest.mark.parametrize("bits,G", [(4, 64), (2, 32)])
def test_small_caches_with_key_outliers_over_seeds(seed, bits, G):
    """The same kind of stream (few keys, single keys dominating the softmax) over more seeds and code widths."""
    spec = CONFIGS[0].with_(name=f"peaky-s{seed}", n_heads=2, tokens_per_frame=130, budget=450, kv_bits=bits, group_size=G,
                            n_layers=1, seed=seed)
    run_stream(spec, 6)


@pytest.mark.parametrize("bits,G,H", [(4, 32, 2), (4, 64, 5), (2, 64, 3), (16, 64, 2), (4, 64, 20)])
def test_per_head_selection(bits, G, H):
    """score_mode 1: every head scores its own keys and keeps its own top-k; lists, token ids, scores and
    the re-quantized cache against the oracle's per-head mode."""
    spec = CONFIGS[0].with_(name=f"perhead-b{bits}-g{G}-h{H}", n_heads=H, tokens_per_frame=150, budget=520, kv_bits=bits,
                            group_size=G, n_layers=2, seed=17)
    run_stream(spec, 7, score_mode=1)


@pytest.mark.parametrize("bits,G", [(4, 64), (2, 32)])
def test_more_heads_than_one_score_chunk_in_the_papers_mode(bits, G):
    """20 heads with the head-averaged score (Sec. 3.2): the score kernel walks the heads in chunks of 16 and
    carries the head sums from one chunk to the next; quantized cache."""
    spec = CONFIGS[0].with_(name=f"h20-b{bits}-g{G}", n_heads=20, tokens_per_frame=150, budget=520, kv_bits=bits,
                            group_size=G, n_layers=1, seed=29)
    run_stream(spec, 7)


@pytest.mark.parametrize("bits,G,H,score_mode", [(4, 64, 3, 0), (4, 32, 2, 0), (2, 64, 5, 0), (2, 32, 3, 1), (4, 64, 4, 1), (16, 64, 2, 0)])
def test_values_quantized_once(bits, G, H, score_mode):
    """value_mode 1: a retained value row keeps the codes, scale and zero point of the step that appended it; keys,
    scores and lists as ever.  Every step against the oracle's variant: caches bit for bit, attention within its
    tolerance.  (With a bf16 cache the mode changes nothing.)"""
    spec = CONFIGS[0].with_(name=f"vonce-b{bits}-g{G}-h{H}-m{score_mode}", n_heads=H, tokens_per_frame=150, budget=520,
                            kv_bits=bits, group_size=G, n_layers=2, seed=37)
    run_stream(spec, 8, score_mode=score_mode, value_mode=1)


def test_values_quantized_once_without_a_budget_and_batched():
    """The same variant in a cache that is never pruned (one buffer rewritten in place: every old block settles once
    its keys have, the values are not touched at all), and through the all-layers call at the benchmark's shape."""
    spec = CONFIGS[0].with_(name="vonce-inplace", n_heads=3, tokens_per_frame=150, budget=0, kv_bits=4, group_size=64,
                            n_layers=1, seed=39)
    ctx, st = parity.make_pair(spec, max_frames=9, value_mode=1)
    src = FrameSource(spec, DEV)
    for f in range(9):
        q, k, v = src.frame(f)
        parity.step_and_compare(ctx, st, spec, 0, 0, q[0], k[0], v[0], budget=0)
    assert ctx.settled_blocks(0)[0] >= 3 * ((8 * 150) // 64 - 4)
    ctx.destroy()
    spec = CONFIGS[2].with_(name="vonce-cfg2", n_layers=2)
    ctx, st = parity.make_pair(spec, value_mode=1)
    src = FrameSource(spec, DEV)
    rows = cover_rows(spec.tokens_per_frame)
    for f in range(5):
        q, k, v = src.frame(f)
        out = ctx.step_all_layers(q, k, v)
        for l in range(2):
            parity.step_and_compare(ctx, st, spec, l, l, q[l], k[l], v[l], rows=rows, stepped=True, out_gpu=out[l])
    ctx.destroy()


def test_per_head_selection_batched_equals_per_layer_steps():
    spec = CONFIGS[0].with_(name="perhead-batched", n_layers=3, n_heads=4, tokens_per_frame=150, budget=400, group_size=64, seed=19)
    ctx_a = xsv.Context.from_spec(spec, score_mode=1)
    ctx_b = xsv.Context.from_spec(spec, score_mode=1)
    src = FrameSource(spec, DEV)
    for f in range(6):
        q, k, v = src.frame(f)
        out_a = ctx_a.step_all_layers(q, k, v)
        out_b = torch.stack([ctx_b.step(l, q[l], k[l], v[l]) for l in range(spec.n_layers)])
        torch.cuda.synchronize()
        assert torch.equal(out_a, out_b)
        for l in range(spec.n_layers):
            parity.compare_cache(ctx_a.cache_export(l), ctx_b.cache_export(l), True)
            sa, sb = ctx_a.last_selection(l), ctx_b.last_selection(l)
            assert sa[1].shape == (4, ctx_a.cache_len(l))
            assert np.array_equal(sa[0], sb[0]) and np.array_equal(sa[1], sb[1])
    ctx_a.destroy()
    ctx_b.destroy()


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("splits", [0, 3])
def test_every_workgroup_shape_of_the_attention_kernel(variant, splits):
    """4 x 64, 4 x 32, 8 x 32 and 8 x 64 query rows per workgroup on a stream whose frame is ragged for all of them."""
    spec = CONFIGS[0].with_(name=f"shape{variant}", n_heads=3, tokens_per_frame=600, budget=2000, n_layers=1, group_size=64, seed=23)
    ctx, st = parity.make_pair(spec)
    ctx.set_attend_variant(variant)
    ctx.set_attend_splits(splits, splits)
    src = FrameSource(spec, DEV)
    rows = np.unique(np.concatenate([cover_rows(600), np.array([31, 32, 63, 64, 255, 256, 511, 512, 575, 576], np.int32)]))
    for f in range(5):
        q, k, v = src.frame(f)
        print(f"  {spec.name} frame {f} T={ctx.cache_len(0)}", flush=True)
        parity.step_and_compare(ctx, st, spec, 0, 0, q[0], k[0], v[0], rows=None if f == 4 else rows)
    ctx.destroy()


def test_budget_below_two_frames_keeps_first_and_current():
    spec = CONFIGS[0].with_(name="k0", budget=100)
    run_stream(spec, 4)


def test_unbounded_bf16_cache_matches_brute_force_attention():
    """No pruning, no quantization: the streamed GPU outputs are plain frame-causal attention."""
    spec = CONFIGS[0].with_(name="plain", budget=0, kv_bits=16)
    run_stream(spec, 5)


@pytest.mark.parametrize("bits,G", [(16, 64), (4, 64), (2, 32)])
def test_unpruned_cache_is_rewritten_in_place_and_settles(bits, G):
    """A cache without a budget keeps one buffer: every step rewrites only the block the frame is appended to and the
    old blocks that re-quantization has not yet reproduced bit for bit; the rest is left alone.  Every byte
    against the oracle (which re-quantizes everything every step), and the count of settled blocks grows."""
    spec = CONFIGS[0].with_(name=f"inplace-b{bits}", n_heads=3, tokens_per_frame=150, budget=0, kv_bits=bits, group_size=G,
                            n_layers=2, seed=41)
    ctx, st = parity.make_pair(spec, max_frames=12)
    src = FrameSource(spec, DEV)
    settled = []
    for f in range(12):
        q, k, v = src.frame(f)
        for l in range(spec.n_layers):
            parity.step_and_compare(ctx, st, spec, l, l, q[l], k[l], v[l], budget=0)
        settled.append(ctx.settled_blocks(1)[0])
    print("  settled (head, block) pairs per frame:", settled, flush=True)
    full_old_blocks = 3 * ((11 * 150) // 64)           # heads x whole blocks of tokens cached before the last step
    assert settled[-1] >= full_old_blocks - 3 * 6      # all but the most recent blocks (a couple of rounds to settle)
    assert all(b >= a for a, b in zip(settled, settled[1:]))
    ctx.destroy()


def test_blocks_settled_while_the_cache_grew_are_not_skipped_once_their_rows_move():
    """While a budgeted cache is still growing no row moves, and old blocks settle as they do without a budget;
    from the first pruning step on only the first frame's blocks keep their place.  The blocks beyond it lose their
    flag (they are re-quantized every step from then on), and every byte still equals the oracle's."""
    spec = CONFIGS[0].with_(name="grow-then-prune", n_heads=2, tokens_per_frame=96, n_special=5, budget=640, kv_bits=4,
                            group_size=64, n_layers=1, seed=43)
    ctx, st = parity.make_pair(spec)
    src = FrameSource(spec, DEV)
    settled = []
    for f in range(12):  # 6 frames fit the budget (576 tokens), the 7th triggers the first pruning
        q, k, v = src.frame(f)
        parity.step_and_compare(ctx, st, spec, 0, 0, q[0], k[0], v[0])
        settled.append(ctx.settled_blocks(0)[0])
    print("  settled (head, block) pairs per frame:", settled, flush=True)
    assert max(settled[:7]) > 2 * 1                    # during growth more than the first frame's one whole block per head
    assert all(x <= 2 * 1 for x in settled[8:])        # afterwards at most that block (96 tokens = 1 whole block of 64)
    ctx.destroy()


@pytest.mark.parametrize("rising", [True, False])
@pytest.mark.parametrize("bits,splits", [(16, 1), (4, 1), (4, 3)])
def test_logits_that_drift_far_along_the_key_axis(rising, bits, splits):
    """Logits that rise (or fall) by hundreds of powers of two from the oldest cached token to the
    current frame: the softmax reference taken from the first keys of a range must move (rising), or
    everything after it must underflow harmlessly (falling)."""
    spec = CONFIGS[0].with_(name="drift", n_heads=2, tokens_per_frame=96, budget=0, kv_bits=bits, group_size=64,
                            n_layers=1, seed=3)
    ctx, st = parity.make_pair(spec, max_frames=6)
    ctx.set_attend_splits(splits, splits)
    g = torch.Generator(device="cpu").manual_seed(7)
    sign = (torch.randint(0, 2, (spec.head_dim,), generator=g) * 2 - 1).float()
    worst = 0.0
    for f in range(5):
        level = (f + 1) if rising else (5 - f)
        # q.k = 64 * 4 * 2.5 * level = 640 * level: 115 powers of two per frame after the 1/8 scale
        q = (4.0 * sign + 0.25 * torch.randn(spec.n_heads, 96, 64, generator=g)).to(torch.bfloat16).to(DEV)
        k = (2.5 * level * sign + 0.25 * torch.randn(spec.n_heads, 96, 64, generator=g)).to(torch.bfloat16).to(DEV)
        v = torch.randn(spec.n_heads, 96, 64, generator=g).to(torch.bfloat16).to(DEV)
        print(f"  drift frame {f} level {level} T={ctx.cache_len(0)}", flush=True)
        (ma, rr), _ = parity.step_and_compare(ctx, st, spec, 0, 0, q, k, v, budget=0)
        worst = max(worst, ma)
    print(f"  worst max_abs={worst:.3e}", flush=True)
    ctx.destroy()


def test_batched_all_layers_equals_per_layer_steps():
    spec = CONFIGS[0].with_(name="batched", n_layers=3, n_heads=4, tokens_per_frame=150, budget=400, group_size=64, seed=5)
    ctx_a = xsv.Context.from_spec(spec)
    ctx_b = xsv.Context.from_spec(spec)
    for ctx in (ctx_a, ctx_b):
        ctx.set_attend_splits(2, 2)   # the same key ranges in both launch forms: outputs equal to the bit
    src = FrameSource(spec, DEV)
    for f in range(5):
        q, k, v = src.frame(f)
        out_a = ctx_a.step_all_layers(q, k, v)
        out_b = torch.stack([ctx_b.step(l, q[l], k[l], v[l]) for l in range(spec.n_layers)])
        torch.cuda.synchronize()
        assert torch.equal(out_a, out_b)
        for l in range(spec.n_layers):
            da, db = ctx_a.cache_export(l), ctx_b.cache_export(l)
            parity.compare_cache(da, db, True)
    ctx_a.destroy()
    ctx_b.destroy()


@pytest.mark.parametrize("batched", [False, True])
def test_deferred_join_gives_the_same_bytes_as_one_stream(batched):
    """Overlap mode 2 (the chain's join deferred to the layer's next use) against mode 0 (one stream)."""
    spec = CONFIGS[0].with_(name="deferred", n_layers=4, n_heads=4, tokens_per_frame=150, budget=400, group_size=64, seed=9)
    ctx_a = xsv.Context.from_spec(spec)
    ctx_b = xsv.Context.from_spec(spec)
    ctx_a.set_overlap(0)
    ctx_b.set_overlap(2)
    for ctx in (ctx_a, ctx_b):
        ctx.set_attend_splits(2, 2)
    src = FrameSource(spec, DEV)
    frames = [src.frame(f) for f in range(6)]     # inputs stay alive, as mode 2 requires
    outs_a, outs_b = [], []
    for f, (q, k, v) in enumerate(frames):
        if batched:
            outs_a.append(ctx_a.step_all_layers(q, k, v))
            outs_b.append(ctx_b.step_all_layers(q, k, v))
        else:
            outs_a.append(torch.stack([ctx_a.step(l, q[l], k[l], v[l]) for l in range(spec.n_layers)]))
            outs_b.append(torch.stack([ctx_b.step(l, q[l], k[l], v[l]) for l in range(spec.n_layers)]))
        if f % 2:
            ctx_b.join()                           # every other frame: an explicit join; else the next use joins
    ctx_b.join()
    torch.cuda.synchronize()
    for a, b in zip(outs_a, outs_b):
        assert torch.equal(a, b)
    for l in range(spec.n_layers):
        parity.compare_cache(ctx_a.cache_export(l), ctx_b.cache_export(l), True)
        sa, sb = ctx_a.last_selection(l), ctx_b.last_selection(l)
        assert np.array_equal(sa[0], sb[0]) and np.array_equal(sa[1], sb[1])
    ctx_a.destroy()
    ctx_b.destroy()


def test_free_running_overlapped_stream_equals_one_stream_at_full_size():
    """The 24-layer workload for 12 frames without any host synchronization, chain on the second stream with
    deferred joins (the form bench.py times), against the same stream on one stream: every output of the last
    three frames and the caches of three layers must be the same bytes.  (The events that order the two streams
    carry no system-scope fence; this is the check that device-scope ordering is enough.)"""
    spec = CONFIGS[2]
    L = spec.n_layers
    src = FrameSource(spec, DEV)
    frames = [src.frame(f) for f in range(12)]
    results = []
    for mode in (0, 2):
        ctx = xsv.Context.from_spec(spec)
        ctx.set_overlap(mode)
        ctx.set_attend_splits(4, 4)      # the same key ranges in both runs, so that the outputs round alike
        outs = torch.empty((3, L, spec.n_heads, spec.tokens_per_frame, spec.head_dim), dtype=torch.bfloat16, device=DEV)
        scratch = torch.empty_like(outs[0])
        for f, (q, k, v) in enumerate(frames):
            dst = outs[f - 9] if f >= 9 else scratch
            for l in range(L):
                ctx.step(l, q[l], k[l], v[l], dst[l])
            if mode == 2:
                ctx.join()
        torch.cuda.synchronize()
        results.append((outs, [ctx.cache_export(l) for l in (0, 11, 23)], [ctx.last_selection(l)[1] for l in (0, 11, 23)]))
        ctx.destroy()
    (oa, ca, ka), (ob, cb, kb) = results
    assert torch.equal(oa, ob)
    for x, y in zip(ca, cb):
        parity.compare_cache(x, y, True)
    for x, y in zip(ka, kb):
        assert np.array_equal(x, y)


def test_contexts_give_their_memory_back():
    """Create, step, export, destroy - sixty times; the device's free memory ends where it started."""
    spec = CONFIGS[0].with_(name="cycle", n_layers=3, n_heads=4, tokens_per_frame=150, budget=400, group_size=64)
    q, k, v = FrameSource(spec, DEV).frame(0)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for i in range(60):
        ctx = xsv.Context.from_spec(spec, score_mode=i % 2)
        ctx.set_overlap(i % 3)
        ctx.set_attend_timing(i % 4 == 0)
        for l in range(spec.n_layers):
            ctx.step(l, q[l], k[l], v[l])
        ctx.join()
        ctx.cache_export(1)
        ctx.destroy()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert abs(free0 - free1) < (64 << 20), (free0, free1)


def test_same_inputs_twice_give_identical_bytes():
    spec = CONFIGS[0].with_(name="determinism", n_heads=4, tokens_per_frame=150, budget=400, group_size=64)
    dumps = []
    for _ in range(2):
        ctx = xsv.Context.from_spec(spec)
        ctx.set_attend_splits(3, 0)
        src = FrameSource(spec, DEV)
        outs = []
        for f in range(5):
            q, k, v = src.frame(f)
            outs.append(ctx.step(0, q[0], k[0], v[0]).clone())
        torch.cuda.synchronize()
        dumps.append((torch.stack(outs).cpu(), ctx.cache_export(0), ctx.last_selection(0)))
        ctx.destroy()
    assert torch.equal(dumps[0][0], dumps[1][0])
    parity.compare_cache(dumps[0][1], dumps[1][1], True)
    assert np.array_equal(dumps[0][2][0], dumps[1][2][0]) and np.array_equal(dumps[0][2][1], dumps[1][2][1])


@pytest.mark.parametrize("score_mode", [0, 1])
def test_import_of_oracle_cache_then_attend(score_mode):
    """dequant_attend alone, on a cache produced by the oracle (isolates it from the GPU quantizer); with per-head
    selection the imported token ids are one row per head, and the stream continues from the imported state."""
    spec = CONFIGS[0].with_(name="import", n_heads=3, tokens_per_frame=100, budget=300, group_size=64)
    ctx, st = parity.make_pair(spec, score_mode=score_mode)
    src = FrameSource(spec, DEV)
    for f in range(4):
        q, k, v = src.frame(f)
        st.step(0, to_u16(q[0]), to_u16(k[0]), to_u16(v[0]), attend=False)
    c = st.export(0)
    ctx.cache_import(0, c, frames_seen=4)
    parity.compare_cache(ctx.cache_export(0), c, True)
    q, k, v = src.frame(4)
    out = ctx.dequant_attend(0, q[0], k[0], v[0])
    ctx.score_prune(0, q[0])
    ctx.quantize(0, k[0], v[0])
    _, keep = ctx.last_selection(0)
    expect, _ = st.step(0, to_u16(q[0]), to_u16(k[0]), to_u16(v[0]), forced_keep=keep)
    parity.check_attention(to_u16(out), expect)
    parity.compare_cache(ctx.cache_export(0), st.export(0), True)     # token ids travelled through the import
    ctx.destroy()


def test_call_order_is_enforced():
    spec = CONFIGS[0]
    ctx = xsv.Context.from_spec(spec)
    q, k, v = (t[0] for t in FrameSource(spec, DEV).frame(0))
    with pytest.raises(xsv.XsvError) as e:
        ctx.quantize(0, k, v)
    assert e.value.code == xsv.XSV_ERR_STATE
    ctx.dequant_attend(0, q, k, v)
    with pytest.raises(xsv.XsvError):
        ctx.dequant_attend(0, q, k, v)
    ctx.score_prune(0, q)
    ctx.quantize(0, k, v)
    assert ctx.cache_len(0) == spec.tokens_per_frame
    with pytest.raises(xsv.XsvError):
        ctx.step(1, q, k, v)  # no such layer
    ctx.reset()
    assert ctx.cache_len(0) == 0
    ctx.destroy()


def test_bad_arguments_are_rejected_before_anything_is_launched():
    """Misaligned or too narrow tensors, a NULL output, a cache that cannot hold another frame: error codes, and
    the context goes on working afterwards."""
    import ctypes as C
    spec = CONFIGS[0].with_(budget=0)
    n = spec.tokens_per_frame
    ctx = xsv.Context.from_spec(spec, max_frames=2)
    lib = xsv.lib()
    q, k, v = (t[0] for t in FrameSource(spec, DEV).frame(0))
    out = torch.empty_like(q)
    T = xsv.as_tensor
    odd = xsv.xsv_tensor(q.data_ptr() + 2, q.stride(0), q.stride(1))           # not 16-byte aligned
    narrow = xsv.xsv_tensor(q.data_ptr(), q.stride(0), 32)                      # rows overlap
    for bad in (odd, narrow, xsv.xsv_tensor(None, 0, 64)):
        assert lib.xsv_step(ctx._h, 0, bad, T(k), T(v), out.data_ptr()) == xsv.XSV_ERR_ARG
        assert lib.xsv_step(ctx._h, 0, T(q), bad, T(v), out.data_ptr()) == xsv.XSV_ERR_ARG
        assert lib.xsv_frame_attend(ctx._h, T(q), T(k), bad, out.data_ptr()) == xsv.XSV_ERR_ARG
    assert lib.xsv_step(ctx._h, 0, T(q), T(k), T(v), None) == xsv.XSV_ERR_ARG
    assert ctx.cache_len(0) == 0                                                # nothing happened
    ctx.step(0, q, k, v, out)
    ctx.step(0, q, k, v, out)
    assert ctx.cache_len(0) == 2 * n
    assert lib.xsv_step(ctx._h, 0, T(q), T(k), T(v), out.data_ptr()) == xsv.XSV_ERR_STATE   # room for max_frames = 2 only
    assert lib.xsv_dequant_attend(ctx._h, 0, T(q), T(k), T(v), out.data_ptr()) == xsv.XSV_ERR_STATE
    ctx.reset()
    ctx.step(0, q, k, v, out)
    torch.cuda.synchronize()
    assert ctx.cache_len(0) == n
    ctx.destroy()
    # K / V rows of one head that would spread over more than 2 GiB (32-bit byte offsets inside the kernel)
    spec2 = CONFIGS[0].with_(tokens_per_frame=150, budget=0)
    ctx2 = xsv.Context.from_spec(spec2, max_frames=2)
    q2, k2, v2 = (t[0] for t in FrameSource(spec2, DEV).frame(0))
    out2 = torch.empty_like(q2)
    wide = xsv.xsv_tensor(k2.data_ptr(), k2.stride(0), 1 << 24)
    assert lib.xsv_step(ctx2._h, 0, T(q2), wide, T(v2), out2.data_ptr()) == xsv.XSV_ERR_ARG
    assert lib.xsv_step(ctx2._h, 0, T(q2), T(k2), wide, out2.data_ptr()) == xsv.XSV_ERR_ARG
    assert lib.xsv_frame_attend(ctx2._h, T(q2), wide, T(v2), out2.data_ptr()) == xsv.XSV_ERR_ARG
    ctx2.step(0, q2, k2, v2, out2)
    assert ctx2.cache_len(0) == 150
    ctx2.destroy()


def test_batched_call_with_mismatched_strides_launches_nothing():
    """xsv_step_all_layers with one layer's K on other strides than the rest: an argument error before any
    launch - no layer changes phase, and the stream goes on afterwards."""
    spec = CONFIGS[0].with_(name="strides", n_layers=3, n_heads=2, tokens_per_frame=100, budget=300, group_size=64)
    ctx = xsv.Context.from_spec(spec)
    lib = xsv.lib()
    src = FrameSource(spec, DEV)
    q, k, v = src.frame(0)
    out = ctx.step_all_layers(q, k, v)
    q, k, v = src.frame(1)
    wide = torch.zeros((spec.n_heads, spec.tokens_per_frame, 128), dtype=torch.bfloat16, device=DEV)
    wide[:, :, :64] = k[1]
    k_odd = [k[0], wide[:, :, :64], k[2]]
    for which in ("k", "v", "q"):
        args = {"q": q, "k": k, "v": v}
        args[which] = k_odd if which == "k" else [args[which][0], wide[:, :, :64], args[which][2]]
        packed = ctx.pack_layers(args["q"], args["k"], args["v"], out)
        assert lib.xsv_step_all_layers(ctx._h, *packed) == xsv.XSV_ERR_ARG
    for l in range(spec.n_layers):
        assert ctx.cache_len(l) == spec.tokens_per_frame
    ctx.step_all_layers(q, k, v, out)                  # every layer is still idle: the frame steps normally
    torch.cuda.synchronize()
    for l in range(spec.n_layers):
        assert ctx.cache_len(l) == 2 * spec.tokens_per_frame
        ctx.step(l, q[l], k[l], v[l])
    ctx.destroy()


def test_one_layer_config_full_size():
    """cfg 1 at its real shape (16 heads, 1374 tokens, budget 2048 < first + current, so k = 0): cache bytes
    compared in full every frame; attention on rows that reach every wave of every workgroup, and on ALL rows
    once the cache has reached its steady length (frames 4 and 5: 2748 cached tokens, 4122 keys)."""
    spec = CONFIGS[1]
    run_stream(spec, 6, rows=cover_rows(spec.tokens_per_frame), all_rows_from=4)


def test_24_layer_config_shape_two_layers():
    """cfg 2 shape (budget 4096, top-k of 1348 from 2722 once saturated) on two of its layers; all query rows
    at the saturated cache (frame 5: 4096 cached tokens, 5470 keys)."""
    spec = CONFIGS[2].with_(n_layers=2)
    run_stream(spec, 6, rows=cover_rows(spec.tokens_per_frame), all_rows_from=5)


def test_24_layer_config_shape_per_head_selection():
    """cfg 2 shape with every head keeping its own top 1348 of 2722 (score_mode 1), two layers."""
    spec = CONFIGS[2].with_(n_layers=2)
    run_stream(spec, 6, rows=cover_rows(spec.tokens_per_frame), all_rows_from=5, score_mode=1)


def test_2bit_config_shape_one_layer():
    """cfg 4 shape (1041 tokens, 2-bit, budget 8192) on one layer past the first two prunes (frame 8: 7287
    cached, k = 6110 of 6246; frame 9: the saturated 8192, k = 6110 of 7151); all query rows on those two."""
    spec = CONFIGS[4].with_(n_layers=1)
    run_stream(spec, 10, rows=cover_rows(spec.tokens_per_frame), all_rows_from=8)


def _stack_as_benchmarked(spec, checked, n_frames, full_from):
    """All layers of `spec` in the launch configuration bench.py times (overlap mode 2, one join per frame,
    default attention grid); the oracle follows the `checked` layers (cache bytes in full, attention on rows
    that reach every wave, ALL rows from frame `full_from` on), the other layers only run."""
    ctx, st = parity.make_pair(spec, layers=checked)
    ctx.set_overlap(2)
    src = FrameSource(spec, DEV)
    rows = cover_rows(spec.tokens_per_frame)
    frames = [src.frame(f) for f in range(n_frames)]          # kept alive, as overlap mode 2 requires
    out = torch.empty((spec.n_layers, spec.n_heads, spec.tokens_per_frame, spec.head_dim), dtype=torch.bfloat16, device=DEV)
    worst, ties = (0.0, 0.0), 0
    for f, (q, k, v) in enumerate(frames):
        for l in range(spec.n_layers):
            if l in checked:
                print(f"  {spec.name} frame {f} layer {l} T={ctx.cache_len(l)}", flush=True)
                (ma, rr), t = parity.step_and_compare(ctx, st, spec, l, checked.index(l), q[l], k[l], v[l],
                                                      rows=None if f >= full_from else rows)
                worst, ties = (max(worst[0], ma), max(worst[1], rr)), ties + t
            else:
                ctx.step(l, q[l], k[l], v[l], out[l])
        ctx.join()
    torch.cuda.synchronize()
    assert ctx.last_attend_workgroups() > 0
    for l in range(spec.n_layers):
        assert ctx.cache_len(l) == spec.budget
    print(f"  worst max_abs={worst[0]:.3e} rel_rms={worst[1]:.3e} ties={ties} grid={ctx.last_attend_workgroups()}", flush=True)
    ctx.destroy()


def test_24_layer_config_as_benchmarked_three_layers_checked():
    """cfg 2, all 24 layers as bench.py runs them; layers 0, 11 and 23 against the oracle, every query row on
    the saturated frames 5 and 6."""
    _stack_as_benchmarked(CONFIGS[2], [0, 11, 23], 7, 5)


def test_2bit_24_layer_config_as_benchmarked_three_layers_checked():
    """cfg 4 (24 layers, 1041 tokens, 2-bit, budget 8192), all layers in the benchmarked launch form; layers
    0, 12 and 23 against the oracle, every query row on the saturated frame 9."""
    _stack_as_benchmarked(CONFIGS[4], [0, 12, 23], 10, 9)


@pytest.mark.timeout(900)
def test_long_drifting_stream_one_layer_1000_frames():
    """One layer of the long-horizon workload for all of its 1000 frames: keep lists and scores every frame,
    attention on sampled rows every frame (rows reaching every wave every 25th frame, all rows on the last),
    the whole cache every tenth frame.  Most of the time is the oracle's."""
    spec = CONFIGS[3].with_(n_layers=1)
    few = np.array([0, 5, 700, 1373], np.int32)
    cover = cover_rows(spec.tokens_per_frame)
    ctx, st = parity.make_pair(spec)
    src = FrameSource(spec, DEV, layers=[0])
    worst, ties = (0.0, 0.0), 0
    for f in range(spec.frames):
        q, k, v = src.frame(f)
        rows = None if f == spec.frames - 1 else (cover if f % 25 == 24 else few)
        (ma, rr), t = parity.step_and_compare(ctx, st, spec, 0, 0, q[0], k[0], v[0], rows=rows, check_cache=f % 10 == 9)
        worst, ties = (max(worst[0], ma), max(worst[1], rr)), ties + t
        if f % 50 == 49:
            print(f"  frame {f + 1}: worst max_abs={worst[0]:.3e} rel_rms={worst[1]:.3e} ties={ties}", flush=True)
    assert spec.frames == 1000 and ctx.cache_len(0) == spec.budget
    ctx.destroy()


@pytest.mark.parametrize("n,n_s,H,budget,bits,G", [
    (1, 1, 1, 3, 4, 32),       # one special token per frame and nothing else: no patch rows to pool
    (7, 5, 1, 16, 2, 32),      # two patch rows: a single short pooled group
    (6, 0, 2, 12, 4, 64),      # no special tokens; budget exactly first + current: k = 0 from the third frame on
    (33, 5, 3, 100, 4, 32),    # one row past a 32-row block; budget leaves k = 34 of a growing middle
    (65, 5, 2, 131, 16, 64),   # bf16 cache, one token past a key tile, k = 1
])
def test_degenerate_and_smallest_shapes(n, n_s, H, budget, bits, G):
    spec = CONFIGS[0].with_(name=f"small-n{n}", n_heads=H, tokens_per_frame=n, n_special=n_s, budget=budget,
                            kv_bits=bits, group_size=G, n_layers=1, seed=21 + n)
    run_stream(spec, 7)


@pytest.mark.parametrize("n,n_s,H,budget,bits,G,g,mode", [
    (79, 0, 3, 200, 4, 32, 3, 0),
    (122, 1, 2, 300, 16, 64, 1, 0),
    (282, 4, 5, 700, 4, 32, 1, 1),
    (25, 5, 2, 77, 2, 64, 1, 0),
    (317, 1, 1, 820, 4, 64, 3, 0),
    (90, 4, 5, 250, 4, 64, 16, 1),
    (122, 2, 4, 0, 2, 64, 16, 1),      # unbounded, quantized
    (195, 1, 4, 500, 2, 32, 7, 0),
    (60, 4, 3, 107, 4, 64, 16, 0),     # budget below first + current
    (10, 1, 2, 25, 16, 32, 1, 1),
    (300, 5, 2, 1000, 2, 64, 16, 0),
])
def test_assorted_shapes_and_settings(n, n_s, H, budget, bits, G, g, mode):
    """Frame sizes, head counts, budgets, pooling sizes and selectors that are no multiples of anything."""
    spec = CONFIGS[0].with_(name=f"mix-n{n}-h{H}", n_heads=H, tokens_per_frame=n, n_special=n_s, budget=budget, kv_bits=bits,
                            group_size=G, pool_size=g, n_layers=2, seed=100 + n, frames=8)
    run_stream(spec, 7, score_mode=mode)


def test_step_can_be_captured_in_a_graph_and_replayed():
    """xsv_step enqueues only kernels and event record/wait pairs, so a stream capture takes it whole (the
    side stream joins the capture through the fork event and leaves it through the join event).  A replay
    repeats the captured step from the same source buffer: every replay must reproduce the eager output,
    with eager work of this process between the replays."""
    spec = CONFIGS[0].with_(name="graph", n_layers=1, n_heads=4, tokens_per_frame=150, budget=400, group_size=64, seed=13)
    src = FrameSource(spec, DEV)
    frames = [src.frame(f) for f in range(5)]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ctx_e = xsv.Context.from_spec(spec)        # eager twin
        ctx_g = xsv.Context.from_spec(spec)        # the last step of this one is captured
        for ctx in (ctx_e, ctx_g):
            ctx.set_attend_splits(2, 2)
        for f in range(4):
            q, k, v = frames[f]
            ctx_e.step(0, q[0], k[0], v[0])
            ctx_g.step(0, q[0], k[0], v[0])
        q, k, v = frames[4]
        want = ctx_e.step(0, q[0], k[0], v[0]).clone()
        want_cache = ctx_e.cache_export(0)
        out = torch.zeros_like(want)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            ctx_g.step(0, q[0], k[0], v[0], out)
        torch.cuda.synchronize()
        for rep in range(3):
            out.zero_()
            scratch = (torch.randn(1 << 16, device=DEV) * 2).sum()     # unrelated eager work and a sync between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, want), f"replay {rep} differs from the eager step"
            assert torch.isfinite(scratch)
        parity.compare_cache(ctx_g.cache_export(0), want_cache, True)   # the host state advanced once, at capture
    ctx_e.destroy()
    ctx_g.destroy()


def test_attention_timing_series():
    spec = CONFIGS[0].with_(name="timing", n_layers=1, n_heads=4, tokens_per_frame=150, budget=400, group_size=64)
    ctx = xsv.Context.from_spec(spec)
    ctx.set_attend_splits(2, 2)
    src = FrameSource(spec, DEV)
    ctx.set_attend_timing(True)
    for f in range(4):
        q, k, v = src.frame(f)
        ctx.step(0, q[0], k[0], v[0])
    launches, attend_ms, merge_ms, event_ms = ctx.attend_times()
    assert launches == 4 and attend_ms > 0.0 and merge_ms > 0.0 and event_ms > 0.0
    steps, score_prune_ms, quantize_ms = ctx.chain_times()
    assert steps == 4 and score_prune_ms > 0.0 and quantize_ms > 0.0
    assert ctx.attend_times()[0] == 0                      # a call starts a new series
    ctx.set_attend_timing(False)
    q, k, v = src.frame(4)
    ctx.step(0, q[0], k[0], v[0])
    assert ctx.attend_times()[0] == 0                      # nothing is recorded while it is off
    ctx.destroy()
