"""Thin binding of libxsv.so (include/xsv.h): argument marshalling only.

Every step of the path runs inside the HIP library; this module turns torch tensors into the
pointer/stride structs of the C ABI and numpy arrays into host buffers.  There is no fallback: if
the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxsv.so")

XSV_OK = 0
XSV_ERR_ARG, XSV_ERR_UNSUPPORTED, XSV_ERR_OOM, XSV_ERR_STATE, XSV_ERR_HIP = -1, -2, -3, -4, -5


class XsvError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


class xsv_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
        ("tokens_per_frame", C.c_int32), ("n_special", C.c_int32), ("budget", C.c_int32),
        ("kv_bits", C.c_int32), ("group_size", C.c_int32), ("pool_size", C.c_int32), ("score_mode", C.c_int32),
        ("softmax_scale", C.c_float), ("max_frames", C.c_int32), ("value_mode", C.c_int32),
    ]


class xsv_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_head", C.c_int64), ("stride_token", C.c_int64)]


# every symbol include/xsv.h declares
EXPORTS = (
    "xsv_create", "xsv_destroy", "xsv_reset", "xsv_dequant_attend", "xsv_frame_attend", "xsv_score_prune", "xsv_quantize",
    "xsv_step", "xsv_step_all_layers", "xsv_set_overlap", "xsv_join", "xsv_cache_len", "xsv_cache_export",
    "xsv_cache_import", "xsv_last_selection", "xsv_quantize_k", "xsv_quantize_v", "xsv_score", "xsv_score_noalloc",
    "xsv_topk_keep", "xsv_strerror",
)
# every symbol include/xsv_tune.h declares (launch tuning and measurement aids)
TUNE_EXPORTS = (
    "xsv_set_attend_splits", "xsv_set_attend_variant", "xsv_set_side_cus", "xsv_set_short_range", "xsv_set_frame_tile_cost",
    "xsv_last_attend_workgroups", "xsv_settled_blocks", "xsv_set_attend_timing", "xsv_attend_times", "xsv_chain_times", "xsv_measure_peaks",
    "xsv_key_ranges", "xsv_line_partition", "xsv_step_plan",
)

_lib = None


def lib():
    """The loaded library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with paper_2602_21780_amd/build.py "
                               "(or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int
        T = xsv_tensor
        L.xsv_create.argtypes = [C.POINTER(xsv_config), vp, C.POINTER(vp)]
        L.xsv_destroy.argtypes = [vp]
        L.xsv_reset.argtypes = [vp]
        L.xsv_join.argtypes = [vp]
        L.xsv_dequant_attend.argtypes = [vp, i32, T, T, T, vp]
        L.xsv_frame_attend.argtypes = [vp, T, T, T, vp]
        L.xsv_score_prune.argtypes = [vp, i32, T]
        L.xsv_quantize.argtypes = [vp, i32, T, T]
        L.xsv_step.argtypes = [vp, i32, T, T, T, vp]
        L.xsv_step_all_layers.argtypes = [vp, C.POINTER(T), C.POINTER(T), C.POINTER(T), C.POINTER(vp)]
        L.xsv_set_attend_splits.argtypes = [vp, i32, i32]
        L.xsv_set_attend_variant.argtypes = [vp, i32]
        L.xsv_set_overlap.argtypes = [vp, i32]
        L.xsv_set_side_cus.argtypes = [vp, i32]
        L.xsv_set_short_range.argtypes = [vp, i32]
        L.xsv_set_frame_tile_cost.argtypes = [vp, i32]
        L.xsv_last_attend_workgroups.argtypes = [vp, C.POINTER(C.c_int32)]
        L.xsv_set_attend_timing.argtypes = [vp, i32]
        L.xsv_settled_blocks.argtypes = [vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.xsv_chain_times.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.xsv_attend_times.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.xsv_cache_len.argtypes = [vp, i32, C.POINTER(C.c_int32)]
        L.xsv_cache_export.argtypes = [vp, i32] + [vp] * 10
        L.xsv_cache_import.argtypes = [vp, i32, C.c_int32, C.c_int32] + [vp] * 10
        L.xsv_last_selection.argtypes = [vp, i32, C.POINTER(C.c_int32), vp, C.POINTER(C.c_int32), vp]
        L.xsv_quantize_k.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.xsv_quantize_v.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.xsv_score.argtypes = [vp, T, vp, i32, i32, i32, i32, i32, i32, vp]
        L.xsv_score_noalloc.argtypes = [vp, T, vp, i32, i32, i32, i32, i32, i32, vp]
        L.xsv_topk_keep.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.xsv_measure_peaks.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.xsv_strerror.argtypes = [i32]
        L.xsv_strerror.restype = C.c_char_p
        for name in EXPORTS + TUNE_EXPORTS:
            if name != "xsv_strerror":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().xsv_strerror(code).decode()


def _check(code: int, what: str):
    if code != XSV_OK:
        raise XsvError(code, what)


def as_tensor(t: torch.Tensor) -> xsv_tensor:
    """bf16 device tensor [H][n][64], channel-contiguous → xsv_tensor (strides in elements)."""
    if t.dtype != torch.bfloat16 or t.dim() != 3 or t.stride(2) != 1 or not t.is_cuda:
        raise ValueError("expected a bf16 device tensor [H][n][d] with contiguous channels")
    return xsv_tensor(t.data_ptr(), t.stride(0), t.stride(1))


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class CacheDump:
    T: int
    k_codes: np.ndarray | None
    k_scale: np.ndarray | None
    k_zero: np.ndarray | None
    v_codes: np.ndarray | None
    v_scale: np.ndarray | None
    v_zero: np.ndarray | None
    k_bf16: np.ndarray
    v_bf16: np.ndarray
    token_frame: np.ndarray
    token_index: np.ndarray


class Context:
    """Owner of an xsv_ctx.  Method names follow the C entry points."""

    def __init__(self, n_layers, n_heads, head_dim, tokens_per_frame, n_special, budget, kv_bits, group_size,
                 pool_size=16, softmax_scale=0.0, max_frames=0, stream=None, score_mode=0, value_mode=0):
        self.cfg = xsv_config(n_layers, n_heads, head_dim, tokens_per_frame, n_special, budget, kv_bits, group_size,
                              pool_size, score_mode, softmax_scale, max_frames, value_mode)
        self._stream = stream
        self._h = C.c_void_p()
        _check(lib().xsv_create(C.byref(self.cfg), _stream_ptr(stream), C.byref(self._h)), "xsv_create")

    @classmethod
    def from_spec(cls, spec, stream=None, **over):
        kw = dict(n_layers=spec.n_layers, n_heads=spec.n_heads, head_dim=spec.head_dim,
                  tokens_per_frame=spec.tokens_per_frame, n_special=spec.n_special, budget=spec.budget,
                  kv_bits=spec.kv_bits, group_size=spec.group_size, pool_size=spec.pool_size,
                  max_frames=spec.frames)
        kw.update(over)
        return cls(stream=stream, **kw)

    def destroy(self):
        if self._h:
            lib().xsv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reset(self):
        _check(lib().xsv_reset(self._h), "xsv_reset")

    def set_attend_splits(self, per_layer_calls=0, batched_calls=0):
        _check(lib().xsv_set_attend_splits(self._h, per_layer_calls, batched_calls), "xsv_set_attend_splits")

    def set_attend_variant(self, variant):
        _check(lib().xsv_set_attend_variant(self._h, variant), "xsv_set_attend_variant")

    def set_overlap(self, mode):
        _check(lib().xsv_set_overlap(self._h, int(mode)), "xsv_set_overlap")

    def set_attend_timing(self, enabled):
        _check(lib().xsv_set_attend_timing(self._h, int(enabled)), "xsv_set_attend_timing")

    def attend_times(self):
        """(launches, attention-kernel span ms, merge-kernel span ms, span of an empty event pair ms), averages
        since the last call."""
        n, a, m, e = C.c_int32(), C.c_float(), C.c_float(), C.c_float()
        _check(lib().xsv_attend_times(self._h, C.byref(n), C.byref(a), C.byref(m), C.byref(e)), "xsv_attend_times")
        return n.value, a.value, m.value, e.value

    def chain_times(self):
        """(steps, score + select span ms, re-quantize span ms), averages since the last call."""
        n, a, b = C.c_int32(), C.c_float(), C.c_float()
        _check(lib().xsv_chain_times(self._h, C.byref(n), C.byref(a), C.byref(b)), "xsv_chain_times")
        return n.value, a.value, b.value

    def last_attend_workgroups(self) -> int:
        w = C.c_int32()
        _check(lib().xsv_last_attend_workgroups(self._h, C.byref(w)), "xsv_last_attend_workgroups")
        return w.value

    def settled_blocks(self, layer=0):
        """((head, block) pairs the re-quantization no longer touches, (head, block) pairs in the layer's cache)."""
        a, b = C.c_int32(), C.c_int32()
        _check(lib().xsv_settled_blocks(self._h, layer, C.byref(a), C.byref(b)), "xsv_settled_blocks")
        return a.value, b.value

    def join(self):
        _check(lib().xsv_join(self._h), "xsv_join")

    def set_short_range(self, percent):
        _check(lib().xsv_set_short_range(self._h, int(percent)), "xsv_set_short_range")

    def set_frame_tile_cost(self, percent):
        _check(lib().xsv_set_frame_tile_cost(self._h, int(percent)), "xsv_set_frame_tile_cost")

    def set_side_cus(self, compute_units):
        _check(lib().xsv_set_side_cus(self._h, int(compute_units)), "xsv_set_side_cus")

    def _out(self, q, out):
        if out is None:
            out = torch.empty((self.cfg.n_heads, self.cfg.tokens_per_frame, self.cfg.head_dim), dtype=torch.bfloat16,
                              device=q.device)
        return out

    def dequant_attend(self, layer, q, k_new, v_new, out=None):
        out = self._out(q, out)
        _check(lib().xsv_dequant_attend(self._h, layer, as_tensor(q), as_tensor(k_new), as_tensor(v_new), out.data_ptr()),
               "xsv_dequant_attend")
        return out

    def frame_attend(self, q, k, v, out=None):
        out = self._out(q, out)
        _check(lib().xsv_frame_attend(self._h, as_tensor(q), as_tensor(k), as_tensor(v), out.data_ptr()), "xsv_frame_attend")
        return out

    def score_prune(self, layer, q):
        _check(lib().xsv_score_prune(self._h, layer, as_tensor(q)), "xsv_score_prune")

    def quantize(self, layer, k_new, v_new):
        _check(lib().xsv_quantize(self._h, layer, as_tensor(k_new), as_tensor(v_new)), "xsv_quantize")

    def step(self, layer, q, k_new, v_new, out=None):
        out = self._out(q, out)
        _check(lib().xsv_step(self._h, layer, as_tensor(q), as_tensor(k_new), as_tensor(v_new), out.data_ptr()), "xsv_step")
        return out

    def pack_step(self, q, k_new, v_new, out):
        """Marshal one layer's tensors once, for repeated step_packed calls (the tensors must stay alive)."""
        return as_tensor(q), as_tensor(k_new), as_tensor(v_new), out.data_ptr()

    def step_packed(self, layer, packed):
        _check(lib().xsv_step(self._h, layer, *packed), "xsv_step")

    def pack_layers(self, q, k_new, v_new, out):
        """Marshal per-layer tensors ([L][H][n][d] or lists) once, for repeated step_all_layers calls."""
        L = self.cfg.n_layers
        arr = lambda ts: (xsv_tensor * L)(*[as_tensor(ts[l]) for l in range(L)])
        outs = (C.c_void_p * L)(*[out[l].data_ptr() for l in range(L)])
        return arr(q), arr(k_new), arr(v_new), outs

    def step_all_layers(self, q=None, k_new=None, v_new=None, out=None, packed=None):
        if packed is None:
            if out is None:
                out = torch.empty((self.cfg.n_layers, self.cfg.n_heads, self.cfg.tokens_per_frame, self.cfg.head_dim),
                                  dtype=torch.bfloat16, device=q[0].device)
            packed = self.pack_layers(q, k_new, v_new, out)
        _check(lib().xsv_step_all_layers(self._h, *packed), "xsv_step_all_layers")
        return out

    def cache_len(self, layer=0) -> int:
        T = C.c_int32()
        _check(lib().xsv_cache_len(self._h, layer, C.byref(T)), "xsv_cache_len")
        return T.value

    def cache_export(self, layer=0) -> CacheDump:
        H, d, G = self.cfg.n_heads, self.cfg.head_dim, self.cfg.group_size
        T = self.cache_len(layer)
        quant = self.cfg.kv_bits != 16
        ng = (T + G - 1) // G if quant else 0
        kc = np.zeros((H, T, d), np.uint8) if quant else None
        vc = np.zeros((H, T, d), np.uint8) if quant else None
        ks = np.zeros((H, ng, d), np.float32) if quant else None
        kz = np.zeros((H, ng, d), np.float32) if quant else None
        vs = np.zeros((H, T, d // G), np.float32) if quant else None
        vz = np.zeros((H, T, d // G), np.float32) if quant else None
        kb = np.zeros((H, T, d), np.uint16)
        vb = np.zeros((H, T, d), np.uint16)
        lead = (H,) if self.cfg.score_mode == 1 else ()     # one retained set per head, or one per layer
        tf = np.zeros(lead + (T,), np.int32)
        ti = np.zeros(lead + (T,), np.int32)
        _check(lib().xsv_cache_export(self._h, layer, _np_ptr(kc), _np_ptr(ks), _np_ptr(kz), _np_ptr(vc), _np_ptr(vs),
                                      _np_ptr(vz), _np_ptr(kb), _np_ptr(vb), _np_ptr(tf), _np_ptr(ti)), "xsv_cache_export")
        return CacheDump(T, kc, ks, kz, vc, vs, vz, kb, vb, tf, ti)

    def cache_import(self, layer, dump, frames_seen):
        """`dump`: any object with the fields of CacheDump (e.g. the oracle's export)."""
        c = lambda a, dt: None if a is None else np.ascontiguousarray(a, dt)
        quant = self.cfg.kv_bits != 16
        arrs = [c(dump.k_codes, np.uint8), c(dump.k_scale, np.float32), c(dump.k_zero, np.float32),
                c(dump.v_codes, np.uint8), c(dump.v_scale, np.float32), c(dump.v_zero, np.float32)] if quant else [None] * 6
        arrs += [None, None] if quant else [c(dump.k_bf16, np.uint16), c(dump.v_bf16, np.uint16)]
        arrs += [c(dump.token_frame, np.int32), c(dump.token_index, np.int32)]
        _check(lib().xsv_cache_import(self._h, layer, int(dump.T), int(frames_seen), *[_np_ptr(a) for a in arrs]),
               "xsv_cache_import")

    def last_selection(self, layer=0):
        ns, nk = C.c_int32(), C.c_int32()
        _check(lib().xsv_last_selection(self._h, layer, C.byref(ns), None, C.byref(nk), None), "xsv_last_selection")
        lead = (self.cfg.n_heads,) if self.cfg.score_mode == 1 else ()
        scores = np.zeros(lead + (ns.value,), np.float32)
        keep = np.zeros(lead + (nk.value,), np.int32)
        _check(lib().xsv_last_selection(self._h, layer, C.byref(ns), _np_ptr(scores), C.byref(nk), _np_ptr(keep)),
               "xsv_last_selection")
        return scores, keep


# ---- stateless entry points (device tensors in, device tensors out) ----------------------------------

def _quantize(fn, name, x, bits, G, stream):
    if x.dtype != torch.bfloat16 or not x.is_contiguous() or x.dim() != 3:
        raise ValueError("expected a contiguous bf16 device tensor [H][T][d]")
    H, T, d = x.shape
    codes = torch.empty((H, T, d), dtype=torch.uint8, device=x.device)
    shape = (H, (T + G - 1) // G, d) if name.endswith("_k") else (H, T, d // G)
    scale = torch.empty(shape, dtype=torch.float32, device=x.device)
    zero = torch.empty(shape, dtype=torch.float32, device=x.device)
    _check(fn(_stream_ptr(stream), x.data_ptr(), H, T, d, bits, G, codes.data_ptr(), scale.data_ptr(), zero.data_ptr()), name)
    return codes, scale, zero


def quantize_k(k, bits, G, stream=None):
    return _quantize(lib().xsv_quantize_k, "xsv_quantize_k", k, bits, G, stream)


def quantize_v(v, bits, G, stream=None):
    return _quantize(lib().xsv_quantize_v, "xsv_quantize_v", v, bits, G, stream)


def score(q, k_mid, n_special, pool_size, stream=None):
    H, n, d = q.shape
    P = k_mid.shape[1]
    if k_mid.dtype != torch.bfloat16 or not k_mid.is_contiguous():
        raise ValueError("k_mid must be a contiguous bf16 device tensor [H][P][d]")
    out = torch.empty(P, dtype=torch.float32, device=q.device)
    _check(lib().xsv_score(_stream_ptr(stream), as_tensor(q), k_mid.data_ptr(), H, n, n_special, P, d, pool_size,
                           out.data_ptr()), "xsv_score")
    return out


def score_noalloc(q, k_mid, n_special, pool_size, out, stream=None):
    """xsv_score_noalloc: asynchronous on the stream, writes the caller's `out` (float32 device tensor [P])."""
    H, n, d = q.shape
    P = k_mid.shape[1]
    if k_mid.dtype != torch.bfloat16 or not k_mid.is_contiguous():
        raise ValueError("k_mid must be a contiguous bf16 device tensor [H][P][d]")
    if out.dtype != torch.float32 or not out.is_contiguous() or out.numel() < P or not out.is_cuda:
        raise ValueError("out must be a contiguous float32 device tensor of at least P elements")
    _check(lib().xsv_score_noalloc(_stream_ptr(stream), as_tensor(q), k_mid.data_ptr(), H, n, n_special, P, d, pool_size,
                                   out.data_ptr()), "xsv_score_noalloc")
    return out


def topk_keep(scores, k, T_first, T_cur, stream=None):
    P = scores.numel()
    keep = torch.empty(T_first + k + T_cur, dtype=torch.int32, device=scores.device)
    _check(lib().xsv_topk_keep(_stream_ptr(stream), scores.data_ptr() if P else None, P, k, T_first, T_cur,
                               keep.data_ptr()), "xsv_topk_keep")
    return keep


def key_ranges(cache_tiles, frame_tiles, ranges, last_percent=100, frame_tile_cost=95):
    """xsv_key_ranges (host only): the tile index at which each of `ranges` key ranges begins, plus the total."""
    begin = (C.c_int32 * (ranges + 1))()
    _check(lib().xsv_key_ranges(cache_tiles, frame_tiles, ranges, last_percent, frame_tile_cost, begin), "xsv_key_ranges")
    return list(begin)


def measure_peaks(stream=None):
    """(bf16 MFMA loop TFLOP/s, streaming copy GB/s) of the current device."""
    a, b = C.c_float(), C.c_float()
    _check(lib().xsv_measure_peaks(_stream_ptr(stream), C.byref(a), C.byref(b)), "xsv_measure_peaks")
    return a.value, b.value
