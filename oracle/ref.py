"""ctypes front end of the CPU oracle (oracle/xsv_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg; never by the product package.  It only marshals numpy arrays into the C++
functions, every piece of arithmetic lives in xsv_ref.cpp.

bf16 tensors travel as numpy uint16 arrays holding the raw bf16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xsv_ref.cpp")
_LIB = os.path.join(_HERE, "libxsv_ref.so")


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no contraction, OpenMP over independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _Config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
        ("tokens_per_frame", C.c_int32), ("n_special", C.c_int32), ("budget", C.c_int32),
        ("kv_bits", C.c_int32), ("group_size", C.c_int32), ("pool_size", C.c_int32),
        ("softmax_scale", C.c_float), ("score_mode", C.c_int32), ("value_mode", C.c_int32),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.xsv_ref_create.restype = C.c_void_p
        _lib.xsv_ref_create.argtypes = [C.POINTER(_Config)]
        _lib.xsv_ref_destroy.argtypes = [C.c_void_p]
        _lib.xsv_ref_num_sets.argtypes = [C.c_void_p]
        _lib.xsv_ref_num_sets.restype = C.c_int
        for name in ("xsv_ref_cache_len", "xsv_ref_last_scores_len", "xsv_ref_last_keep_len"):
            getattr(_lib, name).argtypes = [C.c_void_p, C.c_int]
            getattr(_lib, name).restype = C.c_int
        _lib.xsv_ref_step.restype = C.c_int
        _lib.xsv_ref_step.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 4 + [C.c_int, C.c_void_p, C.c_void_p, C.c_int]
        _lib.xsv_ref_export.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 12
        _lib.xsv_ref_cache_view.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        _lib.xsv_ref_score.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def num_threads() -> int:
    return int(lib().xsv_ref_num_threads())


# ---- stateless functions -------------------------------------------------------------------

def quantize_k(k, bits, G):
    k = _u16(k)
    H, T, d = k.shape
    ng = (T + G - 1) // G
    codes = np.zeros((H, T, d), np.uint8)
    scale = np.zeros((H, ng, d), np.float32)
    zero = np.zeros((H, ng, d), np.float32)
    lib().xsv_ref_quantize_k(_p(k), H, T, d, bits, G, _p(codes), _p(scale), _p(zero))
    return codes, scale, zero


def quantize_v(v, bits, G):
    v = _u16(v)
    H, T, d = v.shape
    codes = np.zeros((H, T, d), np.uint8)
    scale = np.zeros((H, T, d // G), np.float32)
    zero = np.zeros((H, T, d // G), np.float32)
    lib().xsv_ref_quantize_v(_p(v), H, T, d, bits, G, _p(codes), _p(scale), _p(zero))
    return codes, scale, zero


def dequantize_k(codes, scale, zero, G):
    codes = np.ascontiguousarray(codes, np.uint8)
    H, T, d = codes.shape
    out = np.zeros((H, T, d), np.uint16)
    lib().xsv_ref_dequantize_k(_p(codes), _p(np.ascontiguousarray(scale, np.float32)),
                               _p(np.ascontiguousarray(zero, np.float32)), H, T, d, G, _p(out))
    return out


def dequantize_v(codes, scale, zero, G):
    codes = np.ascontiguousarray(codes, np.uint8)
    H, T, d = codes.shape
    out = np.zeros((H, T, d), np.uint16)
    lib().xsv_ref_dequantize_v(_p(codes), _p(np.ascontiguousarray(scale, np.float32)),
                               _p(np.ascontiguousarray(zero, np.float32)), H, T, d, G, _p(out))
    return out


def attend(q, k, v, scale, rows=None):
    q, k, v = _u16(q), _u16(k), _u16(v)
    H, n, d = q.shape
    Tk = k.shape[1]
    assert k.shape == (H, Tk, d) and v.shape == (H, Tk, d)
    if rows is not None:
        rows = np.ascontiguousarray(rows, np.int32)
    n_rows = n if rows is None else len(rows)
    out = np.zeros((H, n_rows, d), np.float32)
    lib().xsv_ref_attend(_p(q), _p(k), _p(v), H, n, Tk, d, C.c_float(scale), _p(rows), n_rows, _p(out))
    return out


def block_causal_attention(q, k, v, F, n, scale):
    q, k, v = _u16(q), _u16(k), _u16(v)
    H, T, d = q.shape
    assert T == F * n
    out = np.zeros((H, T, d), np.float32)
    lib().xsv_ref_block_causal_attention(_p(q), _p(k), _p(v), H, F, n, d, C.c_float(scale), _p(out))
    return out


def score(q, k_mid, n_special, pool):
    q, k_mid = _u16(q), _u16(k_mid)
    H, n, d = q.shape
    P = k_mid.shape[1]
    out = np.zeros(P, np.float32)
    n_pooled = lib().xsv_ref_score(_p(q), _p(k_mid), H, n, n_special, P, d, pool, _p(out))
    return out, n_pooled


def select(scores, k, T_first, T_cur):
    scores = np.ascontiguousarray(scores, np.float32)
    P = len(scores)
    keep = np.zeros(T_first + k + T_cur, np.int32)
    lib().xsv_ref_select(_p(scores), P, k, T_first, T_cur, _p(keep))
    return keep


# ---- the streaming state ---------------------------------------------------------------------

@dataclass
class RefCache:
    T: int
    k_codes: np.ndarray | None
    k_scale: np.ndarray | None
    k_zero: np.ndarray | None
    v_codes: np.ndarray | None
    v_scale: np.ndarray | None
    v_zero: np.ndarray | None
    k_bf16: np.ndarray | None
    v_bf16: np.ndarray | None
    token_frame: np.ndarray
    token_index: np.ndarray
    last_scores: np.ndarray
    last_keep: np.ndarray


class RefStream:
    """One oracle stream: `n_layers` independent caches stepped frame by frame."""

    def __init__(self, n_layers, n_heads, head_dim, tokens_per_frame, n_special, budget, kv_bits,
                 group_size, pool_size=16, softmax_scale=0.0, score_mode=0, value_mode=0):
        self.cfg = _Config(n_layers, n_heads, head_dim, tokens_per_frame, n_special, budget, kv_bits,
                           group_size, pool_size, softmax_scale, score_mode, value_mode)
        self._h = lib().xsv_ref_create(C.byref(self.cfg))
        if not self._h:
            raise ValueError("xsv_ref_create rejected the configuration")

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:     # at interpreter exit the module may already be gone
            _lib.xsv_ref_destroy(self._h)
        self._h = None

    def __del__(self):
        self.close()

    @property
    def scale(self):
        s = self.cfg.softmax_scale
        return s if s != 0.0 else 1.0 / np.sqrt(self.cfg.head_dim)

    @property
    def sets(self):
        """Index sets per layer: 1, or one per head when score_mode is 1."""
        return lib().xsv_ref_num_sets(self._h)

    def cache_len(self, layer=0):
        return lib().xsv_ref_cache_len(self._h, layer)

    def step(self, layer, q, k_new, v_new, rows=None, attend=True, forced_keep=None):
        """Returns (out fp32 [H][n_rows][d] or None, new cache length).
        forced_keep: [T'] (one index set per layer) or [sets][T']."""
        q, k_new, v_new = _u16(q), _u16(k_new), _u16(v_new)
        H, n, d = self.cfg.n_heads, self.cfg.tokens_per_frame, self.cfg.head_dim
        assert q.shape == (H, n, d) and k_new.shape == (H, n, d) and v_new.shape == (H, n, d)
        out = None
        n_rows = 0
        if attend:
            if rows is not None:
                rows = np.ascontiguousarray(rows, np.int32)
            n_rows = n if rows is None else len(rows)
            out = np.zeros((H, n_rows, d), np.float32)
        else:
            rows = None
        if forced_keep is not None:
            forced_keep = np.ascontiguousarray(forced_keep, np.int32).reshape(self.sets, -1)
        T = lib().xsv_ref_step(self._h, layer, _p(q), _p(k_new), _p(v_new), _p(rows), n_rows, _p(out),
                               _p(forced_keep), 0 if forced_keep is None else forced_keep.shape[1])
        if T < 0:
            raise ValueError(f"xsv_ref_step failed ({T})")
        return out, T

    def view(self, layer=0):
        """bf16 view of the cache (K, V) as uint16 [H][T][d]."""
        H, d = self.cfg.n_heads, self.cfg.head_dim
        T = self.cache_len(layer)
        k = np.zeros((H, T, d), np.uint16)
        v = np.zeros((H, T, d), np.uint16)
        lib().xsv_ref_cache_view(self._h, layer, _p(k), _p(v))
        return k, v

    def export(self, layer=0) -> RefCache:
        H, d, G = self.cfg.n_heads, self.cfg.head_dim, self.cfg.group_size
        T = self.cache_len(layer)
        quant = self.cfg.kv_bits != 16
        ng = (T + G - 1) // G if quant else 0
        kc = np.zeros((H, T, d), np.uint8) if quant else None
        ks = np.zeros((H, ng, d), np.float32) if quant else None
        kz = np.zeros((H, ng, d), np.float32) if quant else None
        vc = np.zeros((H, T, d), np.uint8) if quant else None
        vs = np.zeros((H, T, d // G), np.float32) if quant else None
        vz = np.zeros((H, T, d // G), np.float32) if quant else None
        kb = None if quant else np.zeros((H, T, d), np.uint16)
        vb = None if quant else np.zeros((H, T, d), np.uint16)
        # one index set per layer: 1-D arrays; one per head (score_mode 1): a leading axis of H sets
        lead = () if self.sets == 1 else (self.sets,)
        tf = np.zeros(lead + (T,), np.int32)
        ti = np.zeros(lead + (T,), np.int32)
        sc = np.zeros(lead + (lib().xsv_ref_last_scores_len(self._h, layer),), np.float32)
        kp = np.zeros(lead + (lib().xsv_ref_last_keep_len(self._h, layer),), np.int32)
        lib().xsv_ref_export(self._h, layer, _p(kc), _p(ks), _p(kz), _p(vc), _p(vs), _p(vz), _p(kb), _p(vb),
                             _p(tf), _p(ti), _p(sc), _p(kp))
        return RefCache(T, kc, ks, kz, vc, vs, vz, kb, vb, tf, ti, sc, kp)
