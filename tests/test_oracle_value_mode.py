"""Pins for the oracle's "quantize once" variant for the values (value_mode 1): a value row is quantized when its
frame is appended (paper Sec. 3.3, Eq. 9-11 applied per token over groups of channels) and keeps those codes, its
scale and its zero point while it stays in the cache.  CPU only."""
import numpy as np
import pytest

from paper_2602_21780_amd.inputs import CONFIGS, FrameSource, to_u16
from util import bf16_to_f32


def stream(ref, spec, value_mode, score_mode=0):
    return ref.RefStream(spec.n_layers, spec.n_heads, spec.head_dim, spec.tokens_per_frame, spec.n_special,
                         spec.budget, spec.kv_bits, spec.group_size, spec.pool_size, score_mode=score_mode,
                         value_mode=value_mode)


def frames_of(spec, count):
    src = FrameSource(spec, "cpu", layers=[0])
    return [tuple(to_u16(t[0]) for t in src.frame(f)) for f in range(count)]


@pytest.mark.parametrize("bits,G", [(4, 32), (4, 64), (2, 64)])
def test_every_cached_value_row_is_the_one_time_quantization_of_its_original_row(ref, bits, G):
    """The token ids say which frame and which row a cached token came from; its value codes, scale and zero point
    must be exactly what the stateless value quantizer gives for THAT original bf16 row - at any age, through any
    number of prunings."""
    spec = CONFIGS[0].with_(kv_bits=bits, group_size=G, n_heads=3, seed=11)
    st = stream(ref, spec, 1)
    frames = frames_of(spec, 9)
    first = [ref.quantize_v(v, bits, G) for (_, _, v) in frames]     # (codes, scale, zero) of every frame's rows
    for f, (q, k, v) in enumerate(frames):
        st.step(0, q, k, v, attend=False)
        c = st.export(0)
        for i in range(st.cache_len(0)):
            tf, ti = int(c.token_frame[i]), int(c.token_index[i])
            codes, scale, zero = first[tf]
            assert np.array_equal(c.v_codes[:, i], codes[:, ti]), (f, i)
            assert np.array_equal(c.v_scale[:, i], scale[:, ti]) and np.array_equal(c.v_zero[:, i], zero[:, ti]), (f, i)
    assert st.cache_len(0) == spec.budget                            # the stream did prune


def test_keys_keep_lists_and_scores_do_not_depend_on_the_value_mode(ref):
    """The importance score reads keys only (Sec. 3.2), and keys are quantized anew in both modes."""
    spec = CONFIGS[0].with_(n_heads=2, seed=3)
    a, b = stream(ref, spec, 0), stream(ref, spec, 1)
    for q, k, v in frames_of(spec, 8):
        a.step(0, q, k, v, attend=False)
        b.step(0, q, k, v, attend=False)
        ca, cb = a.export(0), b.export(0)
        for name in ("k_codes", "k_scale", "k_zero", "last_keep", "last_scores", "token_frame", "token_index"):
            assert np.array_equal(getattr(ca, name), getattr(cb, name)), name


def test_the_two_modes_agree_until_a_row_is_quantized_a_second_time(ref):
    """After the first frame both caches hold once-quantized rows and are equal; from the second step on mode 0 has
    re-quantized the first frame's rows from their dequantized view, mode 1 has not - the caches may then differ in
    rows that came from the cache, never in the rows of the newest frame."""
    spec = CONFIGS[0].with_(n_heads=2, kv_bits=2, group_size=32, seed=8)      # coarse codes: re-quantization moves some
    a, b = stream(ref, spec, 0), stream(ref, spec, 1)
    n = spec.tokens_per_frame
    differed = False
    for f, (q, k, v) in enumerate(frames_of(spec, 6)):
        a.step(0, q, k, v, attend=False)
        b.step(0, q, k, v, attend=False)
        ca, cb = a.export(0), b.export(0)
        T = a.cache_len(0)
        assert np.array_equal(ca.v_codes[:, T - n:], cb.v_codes[:, T - n:])
        assert np.array_equal(ca.v_scale[:, T - n:], cb.v_scale[:, T - n:])
        if f == 0:
            assert np.array_equal(ca.v_codes, cb.v_codes) and np.array_equal(ca.v_zero, cb.v_zero)
        else:
            differed |= not (np.array_equal(ca.v_codes, cb.v_codes) and np.array_equal(ca.v_scale, cb.v_scale))
    assert differed


def test_error_of_a_once_quantized_row_stays_within_half_a_step(ref):
    """|x - dequantized| <= scale / 2 (+ the bf16 rounding of the view) against the ORIGINAL row, however old."""
    spec = CONFIGS[0].with_(n_heads=2, seed=21)
    st = stream(ref, spec, 1)
    frames = frames_of(spec, 9)
    for q, k, v in frames:
        st.step(0, q, k, v, attend=False)
    c = st.export(0)
    G, d = spec.group_size, spec.head_dim
    view = bf16_to_f32(ref.dequantize_v(c.v_codes, c.v_scale, c.v_zero, G))
    for i in range(st.cache_len(0)):
        orig = bf16_to_f32(frames[int(c.token_frame[i])][2][:, int(c.token_index[i])])     # [H][d]
        step = np.repeat(c.v_scale[:, i], G, axis=-1)                                        # [H][d]
        assert np.all(np.abs(view[:, i] - orig) <= 0.5 * step + 2.0 ** -8 * np.abs(orig) + 1e-6)


def test_bf16_cache_and_attention_are_untouched_by_the_mode(ref):
    """Nothing is quantized in a bf16 cache, so the mode changes nothing at all there; with a quantized cache the
    attention of the FIRST two frames is the same too (the second frame attends to once-quantized rows in both)."""
    spec = CONFIGS[0].with_(kv_bits=16, n_heads=2)
    a, b = stream(ref, spec, 0), stream(ref, spec, 1)
    for q, k, v in frames_of(spec, 5):
        oa, _ = a.step(0, q, k, v)
        ob, _ = b.step(0, q, k, v)
        assert np.array_equal(oa, ob)
    spec = CONFIGS[0].with_(n_heads=2)
    a, b = stream(ref, spec, 0), stream(ref, spec, 1)
    for f, (q, k, v) in enumerate(frames_of(spec, 2)):
        oa, _ = a.step(0, q, k, v)
        ob, _ = b.step(0, q, k, v)
        assert np.array_equal(oa, ob), f


def test_per_head_lists_carry_each_heads_own_rows(ref):
    """With one retained set per head (score_mode 1) a head's carried-over rows follow that head's own list."""
    spec = CONFIGS[0].with_(n_heads=3, seed=13)
    st = stream(ref, spec, 1, score_mode=1)
    frames = frames_of(spec, 8)
    first = [ref.quantize_v(v, spec.kv_bits, spec.group_size) for (_, _, v) in frames]
    for q, k, v in frames:
        st.step(0, q, k, v, attend=False)
    c = st.export(0)
    for h in range(3):
        for i in range(st.cache_len(0)):
            codes, scale, zero = first[int(c.token_frame[h][i])]
            ti = int(c.token_index[h][i])
            assert np.array_equal(c.v_codes[h, i], codes[h, ti]) and np.array_equal(c.v_scale[h, i], scale[h, ti])
