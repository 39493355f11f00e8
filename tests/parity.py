"""Step-by-step comparison of the HIP path with the oracle (used by the GPU tests and the smoke check).

Holds no arithmetic of the method: it feeds both sides the same frames, applies the documented
near-tie protocol for the keep list, and compares outputs and exported caches.
"""
import numpy as np
import torch

from oracle import ref
from paper_2602_21780_amd import xsv
from paper_2602_21780_amd.inputs import to_u16
from util import bf16_to_f32, rel_rms

ATTN_MAX_ABS = 2e-2    # attention output vs oracle on the same dequantized cache
ATTN_REL_RMS = 1e-2
TIE_EPS = 1e-6         # keep lists may differ only on scores this close to the k-th largest


def make_pair(spec, layers=None, **over):
    """(GPU context, oracle stream) for a stream spec; the oracle tracks `layers` (default all)."""
    ctx = xsv.Context.from_spec(spec, **over)
    L = spec.n_layers if layers is None else len(layers)
    st = ref.RefStream(L, spec.n_heads, spec.head_dim, spec.tokens_per_frame, spec.n_special,
                       over.get("budget", spec.budget), over.get("kv_bits", spec.kv_bits),
                       over.get("group_size", spec.group_size), spec.pool_size, score_mode=over.get("score_mode", 0),
                       value_mode=over.get("value_mode", 0))
    return ctx, st


def oracle_keep_preview(st, layer, q16, n, n_special, pool, budget):
    """The keep list(s) the oracle is about to choose, from its stateless functions (no state change).
    One index set per layer: (keep [T'], scores [P] or None); one per head: ([H][T'], [H][P] or None)."""
    Tc = st.cache_len(layer)
    T = Tc + n
    sets = st.sets
    per_set = (lambda a: a) if sets == 1 else (lambda a: np.stack([a] * sets))
    if budget == 0 or T <= budget or Tc == 0:
        return per_set(np.arange(T, dtype=np.int32)), None
    P = T - 2 * n
    k = min(max(0, budget - 2 * n), P)
    if not (0 < k < P):
        return per_set(ref.select(np.zeros(P, np.float32), k, n, n)), None
    k_view, _ = st.view(layer)
    if sets == 1:
        scores, _ = ref.score(q16, np.ascontiguousarray(k_view[:, n:n + P]), n_special, pool)
        return ref.select(scores, k, n, n), scores
    # every head on its own: the oracle's score with that head as the only head
    scores = np.stack([ref.score(np.ascontiguousarray(q16[h:h + 1]), np.ascontiguousarray(k_view[h:h + 1, n:n + P]),
                                 n_special, pool)[0] for h in range(sets)])
    return np.stack([ref.select(scores[h], k, n, n) for h in range(sets)]), scores


def check_keep(keep_gpu, keep_ref, scores_ref, k, n_first):
    """Bit-exact keep lists, apart from documented near-ties.  Returns the number of tie swaps."""
    if np.array_equal(keep_gpu, keep_ref):
        return 0
    assert scores_ref is not None and len(keep_gpu) == len(keep_ref), "keep lists differ where no score was involved"
    assert np.all(np.diff(keep_gpu) > 0), "GPU keep list is not ascending"
    thr = np.sort(scores_ref)[::-1][k - 1]
    diff = np.setxor1d(keep_gpu, keep_ref)
    mid = diff - n_first
    assert np.all((mid >= 0) & (mid < len(scores_ref))), "keep lists differ outside the prunable middle"
    assert np.all(np.abs(scores_ref[mid] - thr) <= TIE_EPS), "keep lists differ beyond a near-tie"
    return len(diff) // 2


def compare_cache(dump, c, quant):
    if quant:
        assert np.array_equal(dump.k_codes, c.k_codes), "key codes differ"
        assert np.array_equal(dump.v_codes, c.v_codes), "value codes differ"
        assert np.array_equal(dump.k_scale, c.k_scale) and np.array_equal(dump.k_zero, c.k_zero), "key scale/zero differ"
        assert np.array_equal(dump.v_scale, c.v_scale) and np.array_equal(dump.v_zero, c.v_zero), "value scale/zero differ"
    else:
        assert np.array_equal(dump.k_bf16, c.k_bf16) and np.array_equal(dump.v_bf16, c.v_bf16), "bf16 rows differ"
    assert np.array_equal(dump.token_frame, c.token_frame) and np.array_equal(dump.token_index, c.token_index), "token ids differ"


def check_attention(out_gpu_u16, out_ref, what=""):
    g = bf16_to_f32(out_gpu_u16).astype(np.float64)
    max_abs = float(np.max(np.abs(g - out_ref)))
    rr = rel_rms(g, out_ref)
    assert max_abs <= ATTN_MAX_ABS and rr <= ATTN_REL_RMS, f"attention mismatch {what}: max_abs={max_abs:.3e} rel_rms={rr:.3e}"
    return max_abs, rr


def step_and_compare(ctx, st, spec, layer_gpu, layer_ref, q, k, v, rows=None, budget=None, out_gpu=None,
                     stepped=False, check_cache=True):
    """One frame of one layer on both sides.  q, k, v: bf16 device tensors [H][n][d].
    `stepped`: the GPU side already ran (e.g. by a batched call producing out_gpu)."""
    n = spec.tokens_per_frame
    budget = spec.budget if budget is None else budget
    q16, k16, v16 = to_u16(q), to_u16(k), to_u16(v)
    if not stepped:
        out_gpu = ctx.step(layer_gpu, q, k, v)
    scores_gpu, keep_gpu = ctx.last_selection(layer_gpu)
    keep_ref, scores_ref = oracle_keep_preview(st, layer_ref, q16, n, spec.n_special, spec.pool_size, budget)
    kk = keep_ref.shape[-1] - 2 * n
    if st.sets == 1:
        ties = check_keep(keep_gpu, keep_ref, scores_ref, kk, n)
    else:
        assert keep_gpu.shape == keep_ref.shape
        ties = sum(check_keep(keep_gpu[h], keep_ref[h], None if scores_ref is None else scores_ref[h], kk, n)
                   for h in range(st.sets))
    if scores_ref is not None:
        assert scores_gpu.shape == scores_ref.shape
        err = float(np.max(np.abs(scores_gpu - scores_ref)))
        assert err <= TIE_EPS * (1.0 + float(np.abs(scores_ref).max())), f"importance scores differ by {err:.3e}"
    out_ref, T_ref = st.step(layer_ref, q16, k16, v16, rows=rows, forced_keep=keep_gpu if ties else None)
    og = to_u16(out_gpu)
    if rows is not None:
        og = og[:, rows]
    stats = check_attention(og, out_ref, f"layer {layer_gpu}")
    assert ctx.cache_len(layer_gpu) == T_ref, "cache length differs"
    if check_cache:
        compare_cache(ctx.cache_export(layer_gpu), st.export(layer_ref), spec.kv_bits != 16)
    return stats, ties
