"""Seeded synthetic streams shaped like the paper's workloads (device-agnostic torch code).

This module holds NO arithmetic of the method (no attention, scoring, pruning or quantization):
it only produces the Q/K/V tensors a global-attention layer would receive for each frame, so the
HIP path and the CPU oracle can be fed identical bits.  It is the one module both sides use.

Recipe (stands in for the video streams of the paper's efficiency sweep, whose datasets and
trained weights are not available):
  * token layout per frame: [1 camera][4 register][N patch] rows, N = 37x37, 37x28 or 59;
  * values: a counter-based 64-bit integer hash of (seed, layer, tensor, frame, head, token,
    channel) picks one of 65 536 standard-normal quantile mid-points, rounded to bf16 — the same
    bits on any device, no device RNG involved;
  * keys carry a few fixed outlier channels per (layer, head) with a gain (the paper's finding
    that key tensors have channel-wise outliers while values do not);
  * optional frame-to-frame drift x_f = 0.9 x_{f-1} + 0.44 eps_f (video redundancy), evaluated
    as three separately rounded fp32 operations so CPU and GPU agree bit for bit.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int → the int64 value with the same low 64 bits."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _mix_int(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix_tensor(x: torch.Tensor) -> torch.Tensor:
    """The same finalizer on int64 tensors (wrap-around arithmetic)."""
    x = x + _GOLDEN
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


_table_cache: dict = {}


def normal_table(device) -> torch.Tensor:
    """65 536 standard-normal quantile mid-points as bf16."""
    key = str(device)
    if key not in _table_cache:
        u = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
        t = math.sqrt(2.0) * torch.erfinv(2.0 * u - 1.0)
        _table_cache[key] = t.to(torch.float32).to(torch.bfloat16).to(device)
    return _table_cache[key]


@dataclass(frozen=True)
class StreamSpec:
    name: str
    n_layers: int
    n_heads: int
    head_dim: int
    tokens_per_frame: int
    n_special: int
    frames: int
    budget: int
    kv_bits: int
    group_size: int
    pool_size: int
    seed: int
    seed_per_layer: bool
    n_outlier: int
    outlier_gain: float
    drift: bool

    def with_(self, **kw) -> "StreamSpec":
        return replace(self, **kw)


# The five workloads of the build's baseline description.
CONFIGS = {
    0: StreamSpec("cfg0-tiny", 1, 2, 64, 64, 5, 8, 256, 4, 32, 16, 0, False, 4, 8.0, False),
    1: StreamSpec("cfg1-one-layer", 1, 16, 64, 1374, 5, 32, 2048, 4, 64, 16, 1, False, 6, 8.0, False),
    2: StreamSpec("cfg2-24-layer", 24, 16, 64, 1374, 5, 100, 4096, 4, 64, 16, 100, True, 6, 8.0, True),
    3: StreamSpec("cfg3-long", 24, 16, 64, 1374, 5, 1000, 4096, 4, 64, 16, 100, True, 6, 8.0, True),
    4: StreamSpec("cfg4-2bit", 24, 16, 64, 1041, 5, 500, 8192, 2, 64, 16, 4, False, 8, 12.0, False),
}


class FrameSource:
    """Produces frame after frame of (Q, K, V), each bf16 [layers][H][n][d], on `device`.

    Frames must be requested in order when the spec has drift (each depends on the previous one).
    `layers` restricts generation to a subset of layer indices (values are those of the full stream).
    """

    def __init__(self, spec: StreamSpec, device="cpu", layers=None):
        self.spec = spec
        self.device = torch.device(device)
        self.layers = list(range(spec.n_layers)) if layers is None else list(layers)
        self._table = normal_table(self.device)
        H, n, d = spec.n_heads, spec.tokens_per_frame, spec.head_dim
        self._elem = torch.arange(H * n * d, dtype=torch.int64, device=self.device).view(1, 1, H, n, d)
        keys = []
        for l in self.layers:
            s = spec.seed + l if spec.seed_per_layer else spec.seed
            keys.append(_s64(_mix_int(_mix_int(s) ^ (l * 0x100000001B3 & _MASK64))))
        self._key = torch.tensor(keys, dtype=torch.int64, device=self.device).view(-1, 1, 1, 1, 1)
        self._tensor = torch.arange(3, dtype=torch.int64, device=self.device).view(1, 3, 1, 1, 1)
        self._gain = self._outlier_gain().to(self.device)
        self._prev = None
        self._next_frame = 0

    def _outlier_gain(self) -> torch.Tensor:
        """[layers][H][1][d] fp32: gain on the outlier channels of K, 1 elsewhere."""
        spec = self.spec
        g = torch.ones(len(self.layers), spec.n_heads, 1, spec.head_dim, dtype=torch.float32)
        for i, l in enumerate(self.layers):
            s = spec.seed + l if spec.seed_per_layer else spec.seed
            for h in range(spec.n_heads):
                base = _mix_int(_mix_int(s) ^ 0xC0FFEE ^ (l << 20) ^ (h << 8))
                order = sorted(range(spec.head_dim), key=lambda c: _mix_int(base + c))
                for c in order[: spec.n_outlier]:
                    g[i, h, 0, c] = spec.outlier_gain
        return g

    def _noise(self, frame: int) -> torch.Tensor:
        """bf16 [layers][3][H][n][d] of hashed standard normals for this frame."""
        ctr = self._elem + (self._tensor + 3 * frame) * self._elem.numel()
        bits = _mix_tensor(_mix_tensor(ctr) ^ self._key)
        return self._table[_lsr(bits, 48)]

    def frame(self, f: int):
        spec = self.spec
        if spec.drift:
            if f != self._next_frame:
                raise ValueError(f"drifting stream: frame {f} requested, expected {self._next_frame}")
            eps = self._noise(f).to(torch.float32)
            if f == 0:
                x = eps
            else:
                a = self._prev * 0.9
                b = eps * 0.44
                x = (a + b).to(torch.bfloat16).to(torch.float32)
            self._prev = x
            self._next_frame = f + 1
        else:
            x = self._noise(f).to(torch.float32)
        q = x[:, 0].to(torch.bfloat16).contiguous()
        k = (x[:, 1] * self._gain).to(torch.bfloat16).contiguous()
        v = x[:, 2].to(torch.bfloat16).contiguous()
        return q, k, v


def to_u16(t: torch.Tensor):
    """bf16 tensor → numpy uint16 array of its bit patterns (host copy)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view("uint16")
