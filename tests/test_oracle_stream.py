"""Pins for the oracle's streaming state (paper Sec. 3.1-3.3 glued together).  CPU only."""
import numpy as np
import pytest
import torch

from paper_2602_21780_amd.inputs import CONFIGS, FrameSource, to_u16
from util import bf16_to_f32, randn_bf16


def run_stream(ref, spec, frames, **over):
    spec = spec.with_(**over) if over else spec
    st = ref.RefStream(spec.n_layers, spec.n_heads, spec.head_dim, spec.tokens_per_frame, spec.n_special,
                       spec.budget, spec.kv_bits, spec.group_size, spec.pool_size)
    src = FrameSource(spec, "cpu", layers=[0])
    return st, src, spec


def test_budget_invariant_and_saturation_on_tiny_config(ref):
    spec = CONFIGS[0]
    st, src, _ = run_stream(ref, spec, spec.frames)
    n = spec.tokens_per_frame
    lengths = []
    for f in range(spec.frames):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        _, T = st.step(0, q, k, v, attend=False)
        lengths.append(T)
        assert T <= max(spec.budget, 2 * n)
        c = st.export(0)
        ids = list(zip(c.token_frame.tolist(), c.token_index.tolist()))
        assert ids == sorted(ids) and len(set(ids)) == T           # temporal order, no duplicates
        assert ids[:n] == [(0, i) for i in range(n)]                # first frame always kept
        assert ids[-n:] == [(f, i) for i in range(n)] or f == 0     # current frame always kept
    # grows linearly to the budget, then stays fixed
    assert lengths == [64, 128, 192, 256, 256, 256, 256, 256]


def test_budget_below_first_plus_current_keeps_exactly_those(ref):
    # the one-layer config's situation, scaled down: budget < 2 n  →  k = 0
    spec = CONFIGS[0].with_(budget=100)
    st, src, _ = run_stream(ref, spec, 4)
    n = spec.tokens_per_frame
    for f in range(4):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        _, T = st.step(0, q, k, v, attend=False)
        assert T == (n if f == 0 else 2 * n)
        c = st.export(0)
        assert set(c.token_frame.tolist()) == ({0} if f == 0 else {0, f})
        assert len(c.last_scores) == 0


def test_kept_middle_is_the_top_k_of_the_recorded_scores(ref):
    spec = CONFIGS[0]
    st, src, _ = run_stream(ref, spec, 6)
    n = spec.tokens_per_frame
    for f in range(6):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        Tc = st.cache_len(0)
        k_view, _ = st.view(0)
        _, T = st.step(0, q, k, v, attend=False)
        c = st.export(0)
        if Tc + n > spec.budget:
            P = Tc + n - 2 * n
            kk = spec.budget - 2 * n
            assert len(c.last_scores) == P and len(c.last_keep) == spec.budget
            # scores are those of the stateless function on the middle of the old cache's view
            s, _ = ref.score(q, np.ascontiguousarray(k_view[:, n:n + P]), spec.n_special, spec.pool_size)
            assert np.array_equal(s, c.last_scores)
            mid = c.last_keep[n:n + kk] - n
            thr = np.sort(c.last_scores)[::-1][kk - 1]
            assert np.all(c.last_scores[mid] >= thr)
            dropped = np.setdiff1d(np.arange(P), mid)
            assert np.all(c.last_scores[dropped] <= thr)
        else:
            assert c.last_keep.tolist() == list(range(Tc + n))


def test_same_indices_for_keys_and_values_with_unquantized_cache(ref):
    # bits 16: the cache rows must be the original rows of the retained tokens, K and V alike
    spec = CONFIGS[0].with_(kv_bits=16)
    st, src, _ = run_stream(ref, spec, 7)
    hist_k, hist_v = [], []
    for f in range(7):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        hist_k.append(k)
        hist_v.append(v)
        st.step(0, q, k, v, attend=False)
    c = st.export(0)
    for pos, (fr, idx) in enumerate(zip(c.token_frame, c.token_index)):
        assert np.array_equal(c.k_bf16[:, pos], hist_k[fr][:, idx])
        assert np.array_equal(c.v_bf16[:, pos], hist_v[fr][:, idx])


def test_whole_retained_cache_is_requantized_every_step(ref):
    spec = CONFIGS[0]
    st, src, _ = run_stream(ref, spec, 6)
    G, bits = spec.group_size, spec.kv_bits
    for f in range(6):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        k_view, v_view = st.view(0)
        st.step(0, q, k, v, attend=False)
        c = st.export(0)
        k_all = np.concatenate([k_view, k], axis=1)[:, c.last_keep]
        v_all = np.concatenate([v_view, v], axis=1)[:, c.last_keep]
        kc, ks, kz = ref.quantize_k(np.ascontiguousarray(k_all), bits, G)
        vc, vs, vz = ref.quantize_v(np.ascontiguousarray(v_all), bits, G)
        assert np.array_equal(kc, c.k_codes) and np.array_equal(ks, c.k_scale) and np.array_equal(kz, c.k_zero)
        assert np.array_equal(vc, c.v_codes) and np.array_equal(vs, c.v_scale) and np.array_equal(vz, c.v_zero)


def test_step_attention_uses_the_dequantized_view(ref):
    spec = CONFIGS[0]
    st, src, _ = run_stream(ref, spec, 5)
    for f in range(5):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        k_view, v_view = st.view(0)
        out, _ = st.step(0, q, k, v)
        expect = ref.attend(q, np.concatenate([k_view, k], 1), np.concatenate([v_view, v], 1), st.scale)
        assert np.array_equal(out, expect)
    # and compression does change the result a little, but only a little (4-bit, outlier keys)
    spec16 = spec.with_(kv_bits=16, budget=0)
    st16, src16, _ = run_stream(ref, spec16, 5)
    for f in range(5):
        q, k, v = (to_u16(t[0]) for t in src16.frame(f))
        out16, _ = st16.step(0, q, k, v)
    err = np.sqrt(np.mean((out - out16) ** 2)) / np.sqrt(np.mean(out16 ** 2))
    assert 1e-4 < err < 0.5


def test_forced_keep_replaces_the_selection(ref):
    spec = CONFIGS[0]
    st, src, _ = run_stream(ref, spec, 6)
    n = spec.tokens_per_frame
    for f in range(5):
        q, k, v = (to_u16(t[0]) for t in src.frame(f))
        st.step(0, q, k, v, attend=False)
    q, k, v = (to_u16(t[0]) for t in src.frame(5))
    T = st.cache_len(0) + n
    forced = np.concatenate([np.arange(n), np.arange(n + 10, n + 10 + spec.budget - 2 * n), np.arange(T - n, T)])
    _, Tn = st.step(0, q, k, v, attend=False, forced_keep=forced)
    assert Tn == len(forced) and np.array_equal(st.export(0).last_keep, forced)
    with pytest.raises(ValueError):
        st.step(0, q, k, v, attend=False, forced_keep=np.array([3, 2, 1], np.int32))


def test_unbounded_and_multi_layer_independence(ref):
    rng = np.random.default_rng(0)
    H, n, d = 2, 16, 64
    st = ref.RefStream(2, H, d, n, 5, 0, 4, 32)
    for f in range(3):
        for layer in range(2):
            q, k, v = (randn_bf16(rng, (H, n, d)) for _ in range(3))
            _, T = st.step(layer, q, k, v, attend=False)
            assert T == (f + 1) * n
    assert st.cache_len(0) == st.cache_len(1) == 3 * n
    with pytest.raises(ValueError):
        ref.RefStream(1, 2, 64, 16, 5, 0, 3, 32)  # unsupported bit width
