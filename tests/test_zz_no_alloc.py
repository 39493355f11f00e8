"""The entry point that allocates nothing (xsv_score_noalloc) against xsv_score, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2602_21780_amd import xsv
from paper_2602_21780_amd.inputs import to_u16
from oracle import ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _randn_bf16(shape, seed, outliers=()):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(shape, generator=g)
    for c in outliers:
        x[..., c] *= 8.0
    return x.to(torch.bfloat16).to(DEV)


def test_score_noalloc_equals_score_on_two_calls_the_second_smaller():
    """Two calls in a row on one device (they share the library's fixed scratch array), the second with fewer
    heads, fewer queries and fewer keys: each must give xsv_score's scores (same kernels: the same bits) and
    stay within the score tolerance of the oracle; nothing of the first call may leak into the second."""
    cases = [(16, 1374, 5, 2722, 16), (3, 150, 5, 333, 4)]
    inputs = [(_randn_bf16((H, n, 64), 7 * H + n), _randn_bf16((H, P, 64), 11 * H + P, outliers=(7, 21, 33))) for H, n, _, P, _ in cases]
    want = [xsv.score(q, k, n_s, g).cpu().numpy() for (q, k), (_, _, n_s, _, g) in zip(inputs, cases)]
    outs = [torch.full((P,), float("nan"), dtype=torch.float32, device=DEV) for _, _, _, P, _ in cases]
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for (q, k), (_, _, n_s, _, g), out in zip(inputs, cases, outs):          # back to back, no wait in between
        xsv.score_noalloc(q, k, n_s, g, out)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert abs(free_after - free_before) <= (2 << 20)                       # no device allocation of any size that shows
    for (q, k), (_, _, n_s, _, g), out, w in zip(inputs, cases, outs, want):
        got = out.cpu().numpy()
        assert np.array_equal(got, w)
        expect, _ = ref.score(to_u16(q), to_u16(k), n_s, g)
        assert float(np.max(np.abs(got - expect))) <= 1e-6 * (1.0 + float(np.abs(expect).max()))


def test_score_noalloc_rejects_more_heads_than_its_scratch_holds():
    H = 65
    q = torch.zeros((H, 8, 64), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((H, 8, 64), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(8, dtype=torch.float32, device=DEV)
    rc = xsv.lib().xsv_score_noalloc(None, xsv.as_tensor(q), k.data_ptr(), H, 8, 0, 8, 64, 1, out.data_ptr())
    assert rc == xsv.XSV_ERR_UNSUPPORTED
    assert xsv.lib().xsv_score_noalloc(None, xsv.as_tensor(q), None, 4, 8, 0, 8, 64, 1, out.data_ptr()) == xsv.XSV_ERR_ARG
