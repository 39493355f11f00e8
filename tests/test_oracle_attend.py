"""Pins for the oracle's attention (paper Sec. 3.1).  CPU only."""
import numpy as np

from util import bf16_to_f32, f32_to_bf16, randn_bf16


def softmax_attention_f64(q, k, v, scale, mask=None):
    """Textbook softmax(QK^T)V with numpy's fp64 matmul (library routine, different coding)."""
    s = np.einsum("hic,hjc->hij", q.astype(np.float64), k.astype(np.float64)) * scale
    if mask is not None:
        s = np.where(mask[None], s, -np.inf)
    s -= s.max(-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(-1, keepdims=True)
    return np.einsum("hij,hjc->hic", p, v.astype(np.float64))


def test_matches_fp64_library_attention(ref):
    rng = np.random.default_rng(0)
    H, n, Tk, d = 3, 37, 201, 64
    q, k, v = randn_bf16(rng, (H, n, d)), randn_bf16(rng, (H, Tk, d), 2.0), randn_bf16(rng, (H, Tk, d))
    out = ref.attend(q, k, v, 0.125)
    expect = softmax_attention_f64(bf16_to_f32(q), bf16_to_f32(k), bf16_to_f32(v), 0.125)
    assert np.max(np.abs(out - expect)) < 2e-5
    # non-square, non-symmetric shapes: a transposed operand or swapped K/V cannot pass
    out_swapped = ref.attend(q, v, k, 0.125)
    assert np.max(np.abs(out_swapped - expect)) > 1e-2


def test_scale_is_applied_to_logits(ref):
    rng = np.random.default_rng(1)
    H, n, Tk, d = 1, 5, 33, 64
    q, k, v = randn_bf16(rng, (H, n, d)), randn_bf16(rng, (H, Tk, d)), randn_bf16(rng, (H, Tk, d))
    for scale in (0.125, 0.5):
        expect = softmax_attention_f64(bf16_to_f32(q), bf16_to_f32(k), bf16_to_f32(v), scale)
        assert np.max(np.abs(ref.attend(q, k, v, scale) - expect)) < 2e-5


def test_equal_keys_give_mean_of_values(ref):
    rng = np.random.default_rng(2)
    H, n, Tk, d = 2, 4, 50, 64
    q = randn_bf16(rng, (H, n, d))
    k = np.repeat(randn_bf16(rng, (H, 1, d)), Tk, axis=1)
    v = randn_bf16(rng, (H, Tk, d))
    out = ref.attend(q, k, v, 0.125)
    expect = bf16_to_f32(v).astype(np.float64).mean(1, keepdims=True)
    assert np.max(np.abs(out - expect)) < 1e-5


def test_dominant_key_selects_its_value(ref):
    H, n, Tk, d = 1, 3, 20, 64
    rng = np.random.default_rng(3)
    q = f32_to_bf16(np.ones((H, n, d), np.float32))
    kf = np.zeros((H, Tk, d), np.float32)
    kf[0, 7] = 10.0  # logit 0.125*64*10 = 80 above all others
    v = randn_bf16(rng, (H, Tk, d))
    out = ref.attend(q, f32_to_bf16(kf), v, 0.125)
    assert np.max(np.abs(out - bf16_to_f32(v)[:, 7:8])) < 1e-6


def test_row_subset_equals_rows_of_full_result(ref):
    rng = np.random.default_rng(4)
    H, n, Tk, d = 2, 30, 70, 64
    q, k, v = randn_bf16(rng, (H, n, d)), randn_bf16(rng, (H, Tk, d)), randn_bf16(rng, (H, Tk, d))
    full = ref.attend(q, k, v, 0.125)
    rows = np.array([29, 0, 13], np.int32)
    assert np.array_equal(ref.attend(q, k, v, 0.125, rows=rows), full[:, rows])


def test_block_causal_checker_matches_masked_fp64_attention(ref):
    rng = np.random.default_rng(5)
    H, F, n, d = 2, 4, 9, 64
    T = F * n
    q, k, v = randn_bf16(rng, (H, T, d)), randn_bf16(rng, (H, T, d)), randn_bf16(rng, (H, T, d))
    frame = np.arange(T) // n
    mask = frame[None, :] <= frame[:, None]  # query i sees key j iff frame(j) <= frame(i)
    expect = softmax_attention_f64(bf16_to_f32(q), bf16_to_f32(k), bf16_to_f32(v), 0.125, mask)
    out = ref.block_causal_attention(q, k, v, F, n, 0.125)
    assert np.max(np.abs(out - expect)) < 2e-5


def test_streamed_steps_equal_one_pass_block_causal_attention_exactly(ref):
    """With an unquantized cache and a budget that is never exceeded, streaming frame by frame
    is the same computation as one frame-causal attention over the whole stream."""
    rng = np.random.default_rng(6)
    H, F, n, d = 2, 8, 64, 64  # the tiny config's shape, budget 512 >= F*n
    q = randn_bf16(rng, (F, H, n, d))
    k = randn_bf16(rng, (F, H, n, d), 2.0)
    v = randn_bf16(rng, (F, H, n, d))
    st = ref.RefStream(1, H, d, n, 5, 512, 16, 32)
    outs = []
    for f in range(F):
        o, T = st.step(0, q[f], k[f], v[f])
        assert T == (f + 1) * n
        outs.append(o)
    streamed = np.concatenate(outs, axis=1)  # [H][F*n][d]
    cat = lambda x: np.ascontiguousarray(np.concatenate(list(x), axis=1))
    brute = ref.block_causal_attention(cat(q), cat(k), cat(v), F, n, st.scale)
    assert np.array_equal(streamed, brute)
