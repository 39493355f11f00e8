"""Pins for the oracle's importance score and selection (paper Sec. 3.2).  CPU only."""
import numpy as np
import pytest

from util import bf16_to_f32, f32_to_bf16, randn_bf16


def brute_score(q, k_mid, n_s, g):
    """The definition with python loops in fp64 (tiny inputs only)."""
    H, n, d = q.shape
    P = k_mid.shape[1]
    groups = [[i] for i in range(n_s)]
    r = n_s
    while r < n:
        groups.append(list(range(r, min(r + g, n))))
        r += g
    pooled = np.zeros((H, len(groups), d))
    for h in range(H):
        for i, rows in enumerate(groups):
            for row in rows:
                pooled[h, i] += q[h, row]
            pooled[h, i] /= len(rows)
    qbar = pooled.sum(0) / H
    kbar = k_mid.astype(np.float64).sum(0) / H
    s = np.zeros(P)
    for j in range(P):
        for i in range(len(groups)):
            s[j] += float(qbar[i] @ kbar[j])
        s[j] /= len(groups)
    return s, len(groups)


@pytest.mark.parametrize("n,n_s,g", [(64, 5, 16), (23, 5, 4), (21, 5, 16), (12, 0, 5)])
def test_score_matches_definition_by_loops(ref, n, n_s, g):
    rng = np.random.default_rng(n)
    H, P, d = 3, 17, 64
    q, k = randn_bf16(rng, (H, n, d)), randn_bf16(rng, (H, P, d), 2.0)
    s, n_pooled = ref.score(q, k, n_s, g)
    expect, n_groups = brute_score(bf16_to_f32(q), bf16_to_f32(k), n_s, g)
    assert n_pooled == n_groups == n_s + -(-(n - n_s) // g)
    assert np.max(np.abs(s - expect)) < 1e-5


def test_pooled_counts_of_the_paper_shapes(ref):
    # 1+4+59, 1+4+37*37, 1+4+37*28 tokens with pooling size 16
    for n, expect in ((64, 9), (1374, 91), (1041, 70)):
        q = np.zeros((1, n, 64), np.uint16)
        _, n_pooled = ref.score(q, np.zeros((1, 3, 64), np.uint16), 5, 16)
        assert n_pooled == expect


def test_single_head_no_pooling_reduces_to_mean_query_dot_key(ref):
    rng = np.random.default_rng(1)
    n, P, d = 20, 31, 64
    q, k = randn_bf16(rng, (1, n, d)), randn_bf16(rng, (1, P, d))
    s, n_pooled = ref.score(q, k, 5, 1)
    assert n_pooled == n
    expect = bf16_to_f32(k)[0].astype(np.float64) @ bf16_to_f32(q)[0].astype(np.float64).mean(0)
    assert np.max(np.abs(s - expect)) < 1e-5


def test_constant_query_closed_form(ref):
    # every query row equal to a: pooled rows are all a, so S_j = a . mean_h K[h][j]
    rng = np.random.default_rng(2)
    H, n, P, d = 4, 37, 25, 64
    a = randn_bf16(rng, (d,))
    q = np.broadcast_to(a, (H, n, d)).copy()
    k = randn_bf16(rng, (H, P, d))
    s, _ = ref.score(q, k, 5, 16)
    expect = bf16_to_f32(k).astype(np.float64).mean(0) @ bf16_to_f32(a).astype(np.float64)
    assert np.max(np.abs(s - expect)) < 1e-5


def test_short_last_group_is_averaged_over_its_real_size(ref):
    # n_s = 5, 21 patch rows, g = 16 → groups of 16 and 5; N_pooled = 7.
    H, n, d = 1, 26, 64
    k = f32_to_bf16(np.ones((1, 1, d), np.float32))
    def s_of_row(row):
        qf = np.zeros((H, n, d), np.float32)
        qf[0, row, 0] = 1.0
        return ref.score(f32_to_bf16(qf), k, 5, 16)[0][0]
    assert s_of_row(0) == pytest.approx(1.0 / 7)            # special row: weight 1/N_pooled
    assert s_of_row(5) == pytest.approx(1.0 / (7 * 16))     # full group
    assert s_of_row(25) == pytest.approx(1.0 / (7 * 5))     # short last group
    # special tokens come first and are not pooled with patches
    assert s_of_row(4) == pytest.approx(1.0 / 7)


def test_heads_are_averaged_before_the_product(ref):
    # the score is a product of head means, not a mean of per-head products
    H, n, d = 2, 5, 64
    qf = np.zeros((H, n, d), np.float32)
    kf = np.zeros((H, 1, d), np.float32)
    qf[0, :, 0] = 2.0   # head 0 query along channel 0
    kf[1, 0, 0] = 4.0   # head 1 key along channel 0
    s, _ = ref.score(f32_to_bf16(qf), f32_to_bf16(kf), 5, 16)
    assert s[0] == pytest.approx((2.0 / 2) * (4.0 / 2))  # per-head products would give 0


def test_select_equals_stable_descending_sort(ref):
    rng = np.random.default_rng(3)
    for P, k in ((1, 1), (50, 0), (50, 50), (257, 100), (1000, 333)):
        scores = rng.integers(0, 40, P).astype(np.float32) / 8  # many exact ties
        keep = ref.select(scores, k, 7, 5)
        order = np.argsort(-scores, kind="stable")[:k]
        expect = np.concatenate([np.arange(7), 7 + np.sort(order), 7 + P + np.arange(5)])
        assert np.array_equal(keep, expect)
        assert len(keep) == 7 + k + 5 and np.all(np.diff(keep) > 0)


def test_select_ties_go_to_smaller_index(ref):
    scores = np.array([1, 3, 3, 3, 0, 3], np.float32)
    assert ref.select(scores, 2, 0, 0).tolist() == [1, 2]
    assert ref.select(scores, 5, 2, 1).tolist() == [0, 1, 2, 3, 4, 5, 7, 8]
