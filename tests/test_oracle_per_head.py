"""Pins for the oracle's per-head selection (score_mode 1: the score of paper Sec. 3.2 with the
averages over heads left out, one retained index set per head).  CPU only."""
import numpy as np
import pytest

from paper_2602_21780_amd.inputs import CONFIGS, FrameSource, to_u16
from util import bf16_to_f32


def stream(ref, spec, mode):
    return ref.RefStream(spec.n_layers, spec.n_heads, spec.head_dim, spec.tokens_per_frame, spec.n_special,
                         spec.budget, spec.kv_bits, spec.group_size, spec.pool_size, score_mode=mode)


def frames_of(spec, count):
    src = FrameSource(spec, "cpu", layers=[0])
    return [tuple(to_u16(t[0]) for t in src.frame(f)) for f in range(count)]


def same_cache(a, b):
    for name in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name


def test_one_head_is_the_paper_mode_bit_for_bit(ref):
    spec = CONFIGS[0].with_(n_heads=1)
    a, b = stream(ref, spec, 0), stream(ref, spec, 1)
    for q, k, v in frames_of(spec, 7):
        oa, Ta = a.step(0, q, k, v)
        ob, Tb = b.step(0, q, k, v)
        assert Ta == Tb and np.array_equal(oa, ob)
        ca, cb = a.export(0), b.export(0)
        same_cache(ca, cb)
        assert np.array_equal(ca.last_scores, cb.last_scores) and np.array_equal(ca.last_keep, cb.last_keep)
        assert np.array_equal(ca.token_frame, cb.token_frame) and np.array_equal(ca.token_index, cb.token_index)


def test_identical_heads_choose_the_shared_list(ref):
    """Two heads fed the same rows: averaging two equal numbers is exact, so the paper's shared score equals each
    head's own score and both modes must keep the same tokens."""
    spec = CONFIGS[0]
    a, b = stream(ref, spec, 0), stream(ref, spec, 1)
    for q, k, v in frames_of(spec, 7):
        q, k, v = (np.ascontiguousarray(np.stack([t[0], t[0]])) for t in (q, k, v))
        a.step(0, q, k, v, attend=False)
        b.step(0, q, k, v, attend=False)
        ca, cb = a.export(0), b.export(0)
        same_cache(ca, cb)
        for h in range(2):
            assert np.array_equal(cb.last_keep[h], ca.last_keep)
            assert np.array_equal(cb.token_frame[h], ca.token_frame) and np.array_equal(cb.token_index[h], ca.token_index)
            if len(ca.last_scores):
                assert np.array_equal(cb.last_scores[h], ca.last_scores)


def test_scores_and_lists_against_the_definition_in_fp64(ref):
    """Head h's score of middle token j = mean over the pooled query rows of head h of (pooled row . key j of head h);
    its list = first frame, the k best of the middle, current frame."""
    spec = CONFIGS[0].with_(n_heads=3, seed=5)
    st = stream(ref, spec, 1)
    n, n_s, g, H = spec.tokens_per_frame, spec.n_special, spec.pool_size, spec.n_heads
    groups = [[i] for i in range(n_s)] + [list(range(r, min(r + g, n))) for r in range(n_s, n, g)]
    scored = 0
    for f, (q, k, v) in enumerate(frames_of(spec, 7)):
        Tc = st.cache_len(0)
        k_view, _ = st.view(0)
        st.step(0, q, k, v, attend=False)
        c = st.export(0)
        assert c.last_keep.shape == (H, st.cache_len(0))
        if Tc + n <= spec.budget:
            assert c.last_scores.shape == (H, 0)
            continue
        P, kk = Tc - n, spec.budget - 2 * n
        qf, kf = bf16_to_f32(q).astype(np.float64), bf16_to_f32(k_view).astype(np.float64)
        for h in range(H):
            pooled = np.stack([qf[h, rows].mean(0) for rows in groups])
            expect = (pooled @ kf[h, n:n + P].T).mean(0)
            assert np.max(np.abs(c.last_scores[h] - expect)) < 1e-5
            order = np.argsort(-expect, kind="stable")
            gap = expect[order[kk - 1]] - expect[order[kk]]
            if gap > 1e-4:   # the cut is not a near-tie: the list is fixed by the definition
                want = np.concatenate([np.arange(n), n + np.sort(order[:kk]), np.arange(Tc, Tc + n)])
                assert np.array_equal(c.last_keep[h], want)
                scored += 1
    assert scored >= 6


def test_heads_are_independent(ref):
    """Changing head 1's keys leaves head 0's list and cache rows untouched (and would not in the paper's mode)."""
    spec = CONFIGS[0].with_(seed=7)
    frames = frames_of(spec, 6)
    dumps = {}
    for mode in (0, 1):
        for variant in (0, 1):
            st = stream(ref, spec, mode)
            for f, (q, k, v) in enumerate(frames):
                if variant and f >= 1:
                    k = k.copy()
                    k[1] = np.roll(k[1], 3, axis=0)     # other rows for head 1's keys
                st.step(0, q, k, v, attend=False)
            dumps[(mode, variant)] = st.export(0)
    a, b = dumps[(1, 0)], dumps[(1, 1)]
    assert np.array_equal(a.last_keep[0], b.last_keep[0]) and np.array_equal(a.k_codes[0], b.k_codes[0])
    assert np.array_equal(a.token_frame[0], b.token_frame[0]) and np.array_equal(a.token_index[0], b.token_index[0])
    assert not np.array_equal(a.last_keep[1], b.last_keep[1])
    assert not np.array_equal(dumps[(0, 0)].last_keep, dumps[(0, 1)].last_keep)


def test_every_head_keeps_first_and_current_and_the_same_count(ref):
    spec = CONFIGS[0].with_(n_heads=4, seed=3)
    st = stream(ref, spec, 1)
    n = spec.tokens_per_frame
    for f, (q, k, v) in enumerate(frames_of(spec, 8)):
        _, T = st.step(0, q, k, v, attend=False)
        assert T <= max(spec.budget, 2 * n)
        c = st.export(0)
        assert c.token_frame.shape == (4, T)
        for h in range(4):
            ids = list(zip(c.token_frame[h].tolist(), c.token_index[h].tolist()))
            assert ids == sorted(ids) and len(set(ids)) == T
            assert ids[:n] == [(0, i) for i in range(n)]
            assert ids[-n:] == [(f, i) for i in range(n)] or f == 0
    lists = {tuple(c.token_index[h].tolist()) for h in range(4)}
    assert len(lists) > 1   # with different heads the sets do differ


def test_forced_lists_are_taken_per_head(ref):
    spec = CONFIGS[0].with_(seed=2)
    a, b = stream(ref, spec, 1), stream(ref, spec, 1)
    for q, k, v in frames_of(spec, 6):
        a.step(0, q, k, v, attend=False)
        forced = a.export(0).last_keep
        b.step(0, q, k, v, attend=False, forced_keep=forced)
        same_cache(a.export(0), b.export(0))
        assert np.array_equal(a.export(0).token_index, b.export(0).token_index)


def test_mode_is_validated(ref):
    spec = CONFIGS[0]
    with pytest.raises(ValueError):
        stream(ref, spec, 2)
