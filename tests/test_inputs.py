"""The synthetic stream generator: determinism, shapes, statistics.  CPU only."""
import numpy as np
import torch

from paper_2602_21780_amd.inputs import CONFIGS, FrameSource, normal_table, to_u16


def test_shapes_and_token_counts():
    assert CONFIGS[1].tokens_per_frame == 1 + 4 + 37 * 37
    assert CONFIGS[4].tokens_per_frame == 1 + 4 + 37 * 28
    assert CONFIGS[0].tokens_per_frame == 1 + 4 + 59
    q, k, v = FrameSource(CONFIGS[0]).frame(3)
    assert q.shape == k.shape == v.shape == (1, 2, 64, 64) and q.dtype == torch.bfloat16


def test_deterministic_and_layer_subset_consistent():
    spec = CONFIGS[2].with_(tokens_per_frame=37, n_layers=3)
    a = FrameSource(spec)
    b = FrameSource(spec, layers=[2])
    for f in range(3):
        qa, ka, va = a.frame(f)
        qb, kb, vb = b.frame(f)
        assert torch.equal(qa[2], qb[0]) and torch.equal(ka[2], kb[0]) and torch.equal(va[2], vb[0])
    assert not torch.equal(qa[0], qa[1])


def test_statistics_outliers_and_drift():
    t = normal_table("cpu").float()
    assert abs(t.mean()) < 1e-3 and abs(t.std() - 1.0) < 5e-3
    spec = CONFIGS[1].with_(tokens_per_frame=300)
    q, k, v = FrameSource(spec).frame(0)
    assert abs(q.float().std() - 1) < 0.02 and abs(v.float().std() - 1) < 0.02
    per_ch = k[0].float().std(dim=1)  # [H][d]
    assert torch.all((per_ch > 6).sum(-1) == spec.n_outlier)
    assert torch.all((per_ch < 1.3).sum(-1) == 64 - spec.n_outlier)
    spec = CONFIGS[2].with_(tokens_per_frame=300, n_layers=1)
    src = FrameSource(spec)
    q0, _, _ = src.frame(0)
    q1, _, _ = src.frame(1)
    r = torch.corrcoef(torch.stack([q0.float().flatten(), q1.float().flatten()]))[0, 1]
    assert 0.85 < r < 0.93 and abs(q1.float().std() - 1) < 0.03
