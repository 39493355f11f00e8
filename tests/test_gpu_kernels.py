"""GPU parity of the stateless entry points against the oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from paper_2602_21780_amd import xsv
from paper_2602_21780_amd.inputs import to_u16
from oracle import ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def randn_bf16(shape, seed, scale=1.0, outliers=()):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(shape, generator=g) * scale
    for c in outliers:
        x[..., c] *= 8.0
    return x.to(torch.bfloat16).to(DEV)


@pytest.mark.parametrize("bits,G", [(4, 64), (4, 32), (2, 64), (2, 32)])
@pytest.mark.parametrize("H,T", [(2, 64), (3, 150), (1, 1), (16, 1374)])
def test_quantize_k_and_v_bit_exact(bits, G, H, T):
    print(f"quantize bits={bits} G={G} H={H} T={T}", flush=True)
    x = randn_bf16((H, T, 64), 17 * T + bits + G, 1.5, outliers=(3, 40))
    x16 = to_u16(x)
    for fn_gpu, fn_ref in ((xsv.quantize_k, ref.quantize_k), (xsv.quantize_v, ref.quantize_v)):
        codes, scale, zero = fn_gpu(x, bits, G)
        rc, rs, rz = fn_ref(x16, bits, G)
        assert np.array_equal(codes.cpu().numpy(), rc)
        assert np.array_equal(scale.cpu().numpy(), rs)
        assert np.array_equal(zero.cpu().numpy(), rz)


def test_quantize_degenerate_groups():
    # constant groups (s = 1 fallback), groups away from zero (zero point outside the code range),
    # exact half-way values (ties to even)
    x = torch.zeros((1, 64, 64))
    x[0, :, 0] = 3.0
    x[0, :, 1] = torch.linspace(5, 6, 64)
    x[0, :, 2] = torch.arange(64) * 0.5
    x[0, 5, :] = 7.0
    xb = x.to(torch.bfloat16).to(DEV)
    for fn_gpu, fn_ref in ((xsv.quantize_k, ref.quantize_k), (xsv.quantize_v, ref.quantize_v)):
        for bits in (2, 4):
            codes, scale, zero = fn_gpu(xb, bits, 64)
            rc, rs, rz = fn_ref(to_u16(xb), bits, 64)
            assert np.array_equal(codes.cpu().numpy(), rc)
            assert np.array_equal(scale.cpu().numpy(), rs) and np.array_equal(zero.cpu().numpy(), rz)


@pytest.mark.parametrize("bits", [2, 4])
def test_quantize_quotients_on_and_next_to_rounding_boundaries(bits):
    """Groups whose scale is exactly 1, 1/2 or 3 (quotients that are exact half-integers: ties to even, and
    thirds next to them), groups far from zero (large zero points, large quotients) and tiny magnitudes: every
    code must be the one IEEE division and round-half-to-even give."""
    top = (1 << bits) - 1
    g = torch.Generator().manual_seed(5)
    x = torch.zeros((2, 256, 64))
    k = torch.randint(0, 2 * top + 1, (2, 256, 64), generator=g).float() * 0.5       # multiples of 1/2 in [0, top]
    x[:] = k
    x[:, :, 0] = 0.0
    x[:, :, 1] = float(top)                                                          # every token group spans [0, top]: s = 1
    x[0, :, 8:16] = k[0, :, 8:16] * 0.5                                              # quarters
    x[0, :, 16:24] = k[0, :, 16:24] * 3.0 + 300.0                                    # s = 3 on [300, 300 + 3 top]: zero point -100
    x[1, :, 24:32] = k[1, :, 24:32] * 2.0 ** -100                                    # tiny scale
    x[1, :, 32:40] = -4096.0 + k[1, :, 32:40]                                        # quotients in the thousands
    x[0, 0::64, :] = 0.0
    x[0, 1::64, :] = float(top)                                                      # every channel group spans at least [0, top]
    xb = x.to(torch.bfloat16).to(DEV)
    for fn_gpu, fn_ref in ((xsv.quantize_k, ref.quantize_k), (xsv.quantize_v, ref.quantize_v)):
        for G in (32, 64):
            codes, scale, zero = fn_gpu(xb, bits, G)
            rc, rs, rz = fn_ref(to_u16(xb), bits, G)
            assert np.array_equal(scale.cpu().numpy(), rs) and np.array_equal(zero.cpu().numpy(), rz)
            assert np.array_equal(codes.cpu().numpy(), rc)


@pytest.mark.parametrize("bits", [2, 4])
def test_quantize_extreme_magnitudes_next_to_ordinary_groups(bits):
    """Groups of huge (1e30), tiny (1e-30) and ordinary values side by side, per channel and per token: the
    quantizer's quotient takes its division-free form only where no intermediate can leave the normal range,
    and both forms must give the oracle's codes."""
    g = torch.Generator().manual_seed(9)
    x = torch.randn((2, 192, 64), generator=g)
    x[0, :, 5] *= 1e30
    x[0, :, 6] *= 1e-30
    x[1, 10:20, :] *= 3e25
    x[1, 100:110, :] *= 1e-28
    x[1, 64:128, 40] = 2.5e20 + x[1, 64:128, 40] * 1e18
    xb = x.to(torch.bfloat16).to(DEV)
    for fn_gpu, fn_ref in ((xsv.quantize_k, ref.quantize_k), (xsv.quantize_v, ref.quantize_v)):
        for G in (32, 64):
            codes, scale, zero = fn_gpu(xb, bits, G)
            rc, rs, rz = fn_ref(to_u16(xb), bits, G)
            assert np.array_equal(scale.cpu().numpy(), rs) and np.array_equal(zero.cpu().numpy(), rz)
            assert np.array_equal(codes.cpu().numpy(), rc)


@pytest.mark.parametrize("H,n,n_s,P,g", [(2, 64, 5, 192, 16), (16, 1374, 5, 2722, 16), (3, 37, 5, 70, 4), (1, 21, 0, 1, 1),
                                         (20, 150, 5, 333, 16), (37, 90, 3, 100, 7)])
def test_score_matches_oracle(H, n, n_s, P, g):
    print(f"score H={H} n={n} P={P}", flush=True)
    q = randn_bf16((H, n, 64), n + P)
    k = randn_bf16((H, P, 64), n + P + 1, outliers=(7, 21, 33))
    s = xsv.score(q, k, n_s, g).cpu().numpy()
    expect, _ = ref.score(to_u16(q), to_u16(k), n_s, g)
    # fp32 sums in a different order: a few ulp of the largest score
    err = float(np.max(np.abs(s - expect)))
    assert err <= 1e-6 * (1.0 + float(np.abs(expect).max())), err
    # strided query tensor (a view into a larger buffer) gives the same bits
    big = torch.zeros((H, n, 128), dtype=torch.bfloat16, device=DEV)
    big[:, :, :64] = q
    s2 = xsv.score(big[:, :, :64], k, n_s, g).cpu().numpy()
    assert np.array_equal(s, s2)


@pytest.mark.parametrize("P,k", [(1, 1), (50, 0), (50, 50), (257, 100), (2722, 1348), (7151, 6110), (40000, 12345)])
def test_topk_keep_bit_exact_with_ties(P, k):
    print(f"topk P={P} k={k}", flush=True)
    g = torch.Generator().manual_seed(P)
    tied = (torch.randint(0, 50, (P,), generator=g).float() / 8 - 3).to(DEV)        # many exact ties, both signs
    smooth = torch.randn(P, generator=g).to(DEV)
    for scores in (tied, smooth):
        keep = xsv.topk_keep(scores, k, 7, 5).cpu().numpy()
        assert np.array_equal(keep, ref.select(scores.cpu().numpy(), k, 7, 5))


def test_topk_keep_all_equal_scores_take_smallest_positions():
    scores = torch.zeros(1000, device=DEV)
    keep = xsv.topk_keep(scores, 10, 0, 0).cpu().numpy()
    assert keep.tolist() == list(range(10))


@pytest.mark.parametrize("H,n,splits", [(2, 64, 0), (3, 150, 2), (16, 1374, 0), (16, 1041, 0), (1, 1, 0)])
def test_frame_attention_matches_oracle(H, n, splits):
    """Attention inside one frame (no cache): the oracle's attention over the frame's own keys; the context's
    streaming state is not touched."""
    print(f"frame attention H={H} n={n}", flush=True)
    q, k, v = (randn_bf16((H, n, 64), 3 * n + i, outliers=((5, 50) if i == 1 else ())) for i in range(3))
    ctx = xsv.Context(1, H, 64, n, min(5, n), 4 * n, 4, 64)
    ctx.set_attend_splits(splits, splits)
    ctx.step(0, q, k, v)                         # a cached frame that frame attention must ignore
    out = ctx.frame_attend(q, k, v)
    rows = np.unique(np.array([0, n // 3, n // 2, n - 1], np.int32))
    expect = ref.attend(to_u16(q), to_u16(k), to_u16(v), 0.125, rows=rows)
    got = to_u16(out)[:, rows].astype(np.uint32) << 16
    got = got.view(np.float32).astype(np.float64)
    assert float(np.max(np.abs(got - expect))) <= 2e-2
    rms = float(np.sqrt(np.mean((got - expect) ** 2)) / np.sqrt(np.mean(expect ** 2)))
    assert rms <= 1e-2
    assert ctx.cache_len(0) == n
    ctx.step(0, q, k, v)                         # the stream goes on as if nothing had happened
    assert ctx.cache_len(0) == 2 * n
    ctx.destroy()


def test_measured_peaks_are_plausible():
    """The library's two yardsticks: an MFMA-only loop and a streaming copy, against the published peaks."""
    mfma, copy = xsv.measure_peaks()
    print(f"measured: MFMA loop {mfma:.0f} TFLOP/s, copy {copy:.0f} GB/s", flush=True)
    assert 800.0 < mfma < 2600.0
    assert 1500.0 < copy < 8200.0
