"""Python face of the CPU oracle (oracle/tokfilt_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu-baseline leg may import this package.
It knows nothing about the HIP library and shares nothing with it.

Every function takes torch CPU tensors or numpy arrays (bf16 tensors are widened to float
exactly) in the [B, H, n, d] layout and returns numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tokfilt_oracle.c")
_LIB = os.path.join(_HERE, "libtokfilt_oracle.so")

FUSE_EQ2, FUSE_INVVAR, FUSE_KEY_ONLY, FUSE_VALUE_ONLY = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over (batch, head) only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.tfo_num_threads.restype = ctypes.c_int
        lib.tfo_set_num_threads.argtypes = [ctypes.c_int]
        lib.tfo_anchor_cosine.argtypes = [vp, i64, i64, i64, i64, ctypes.c_int, vp, vp]
        lib.tfo_anchor_cosine_ema.argtypes = [vp, i64, i64, i64, i64, dbl, ctypes.c_int, vp, vp]
        lib.tfo_fuse.argtypes = [vp, vp, i64, i64, i64, ctypes.c_int, vp, vp]
        lib.tfo_keep_count.argtypes = [i64, dbl]
        lib.tfo_tail_schedule.argtypes = [i64, dbl, dbl, vp]
        lib.tfo_tail_schedule.restype = i64
        flt = ctypes.c_float
        lib.tfo_select_online.argtypes = [vp, i64, i64, i64, flt, flt, flt, vp, vp, vp, vp, vp]
        lib.tfo_keep_count.restype = i64
        lib.tfo_select.argtypes = [vp, i64, i64, i64, i64, vp, vp, vp]
        lib.tfo_attend.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, vp, i64, dbl, vp]
        lib.tfo_attend_rows.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, vp, i64, dbl,
                                        vp, i64, vp]
        lib.tfo_decode_step.argtypes = [vp, vp, vp, i64, i64, i64, i64, ctypes.c_int, dbl,
                                        ctypes.c_int, ctypes.c_int, i64, flt, flt, dbl, vp, vp, vp, vp, vp, vp,
                                        vp, vp, vp, i64, vp, vp, vp]
        lib.tfo_decode_step.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().tfo_num_threads())


def set_num_threads(n: int) -> None:
    """How many threads the loops over (batch, head) use from now on."""
    _load().tfo_set_num_threads(int(n))


def _f32(x) -> np.ndarray:
    """Contiguous float32 numpy view/copy of a torch tensor or array (bf16 widened exactly)."""
    if hasattr(x, "detach"):
        x = x.detach().cpu().float().contiguous().numpy()
    return np.ascontiguousarray(x, dtype=np.float32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def anchor_cosine(x, return_anchors: bool = False, inclusive: bool = False):
    """Per-head cosine of each token's row with the mean of the rows before it (inclusive: of
    the rows up to and including it).
    x: [B, H, n, d] -> cos [B, H, n] (float64); optionally the anchors [B, H, n, d]."""
    xa = _f32(x)
    B, H, n, d = xa.shape
    cosv = np.empty((B, H, n), dtype=np.float64)
    anchors = np.empty((B, H, n, d), dtype=np.float64) if return_anchors else None
    _load().tfo_anchor_cosine(_p(xa), B, H, n, d, int(inclusive), _p(cosv),
                              _p(anchors) if return_anchors else None)
    return (cosv, anchors) if return_anchors else cosv


def anchor_cosine_ema(x, gamma: float, return_anchors: bool = False, inclusive: bool = False):
    """Per-head cosine of each token's row with the incremental anchor of Eq. 1 as it stands
    before that token (anchor <- gamma * anchor + (1 - gamma) * row, from zero; inclusive: as
    it stands after that token has been folded in).
    x: [B, H, n, d] -> cos [B, H, n] (float64); optionally the anchors [B, H, n, d]."""
    xa = _f32(x)
    B, H, n, d = xa.shape
    cosv = np.empty((B, H, n), dtype=np.float64)
    anchors = np.empty((B, H, n, d), dtype=np.float64) if return_anchors else None
    _load().tfo_anchor_cosine_ema(_p(xa), B, H, n, d, float(gamma), int(inclusive), _p(cosv),
                                  _p(anchors) if return_anchors else None)
    return (cosv, anchors) if return_anchors else cosv


def fuse(cos_k, cos_v, mode: int = FUSE_EQ2, return_stats: bool = False):
    """Across-head mean/variance and variance-aware fusion.
    cos_k, cos_v: [B, H, n] -> S [B, n]; stats [B, n, 5] = (s_k, s_v, var_k, var_v, alpha)."""
    ck = np.ascontiguousarray(cos_k, dtype=np.float64)
    cv = np.ascontiguousarray(cos_v, dtype=np.float64)
    B, H, n = ck.shape
    S = np.empty((B, n), dtype=np.float64)
    stats = np.empty((B, n, 5), dtype=np.float64) if return_stats else None
    _load().tfo_fuse(_p(ck), _p(cv), B, H, n, int(mode), _p(S),
                     _p(stats) if return_stats else None)
    return (S, stats) if return_stats else S


def tail_schedule(n_layers: int, p_global: float, y: float):
    """Per-layer pruning ratios of the tail-focused schedule (Eq. 3): the last fraction y of
    the layers at p_global / y, the rest at 0.  Returns (ratios [n_layers], n_tail)."""
    ratios = np.zeros(int(n_layers), dtype=np.float64)
    n_tail = int(_load().tfo_tail_schedule(int(n_layers), float(p_global), float(y), _p(ratios)))
    if n_tail < 0:
        raise ValueError("tail_schedule: arguments out of range")
    return ratios, n_tail


def keep_count(n: int, ratio: float) -> int:
    return int(_load().tfo_keep_count(int(n), float(ratio)))


def select(scores, ratio: float, warmup: int = 1):
    """Keep decision at an exact count.  scores: [B, n] (rounded to float32 first, the
    precision the decision is defined in).  Returns keep [B, n] uint8, kept_idx [B, m]
    int32, tau [B] float32."""
    s32 = np.ascontiguousarray(np.asarray(scores, dtype=np.float64).astype(np.float32))
    B, n = s32.shape
    m = keep_count(n, ratio)
    keep = np.empty((B, n), dtype=np.uint8)
    idx = np.empty((B, m), dtype=np.int32)
    tau = np.empty((B,), dtype=np.float32)
    _load().tfo_select(_p(s32), B, n, m, int(warmup), _p(keep), _p(idx), _p(tau))
    return keep, idx, tau


def _scale(d, scale):
    return float(scale) if scale else 1.0 / float(np.sqrt(d))


def select_online(scores, target: float, eta: float, tau0: float, warmup: int = 1,
                  return_trace: bool = False):
    """Online keep decision with the adaptive threshold of Eq. 4.  scores: [B, n] (rounded to
    float32 first).  Returns keep [B, n] uint8, kept_idx [B, n] int32 (padded with -1),
    count [B] int32, tau [B] float32 (threshold after the last token); with return_trace also
    the threshold every token was judged with, [B, n] float32."""
    s32 = np.ascontiguousarray(np.asarray(scores, dtype=np.float64).astype(np.float32))
    B, n = s32.shape
    keep = np.empty((B, n), dtype=np.uint8)
    idx = np.empty((B, n), dtype=np.int32)
    count = np.empty((B,), dtype=np.int32)
    tau = np.empty((B,), dtype=np.float32)
    trace = np.empty((B, n), dtype=np.float32) if return_trace else None
    _load().tfo_select_online(_p(s32), B, n, int(warmup), ctypes.c_float(target),
                              ctypes.c_float(eta), ctypes.c_float(tau0), _p(keep), _p(idx),
                              _p(count), _p(tau), _p(trace) if return_trace else None)
    if return_trace:
        return keep, idx, count, tau, trace
    return keep, idx, count, tau


def attend(q, k, v, kept_idx, scale: float = 0.0):
    """Causal softmax attention among kept tokens; zero rows elsewhere.  -> O [B, Hq, n, d]."""
    qa, ka, va = _f32(q), _f32(k), _f32(v)
    B, Hq, n, d = qa.shape
    Hkv = ka.shape[1]
    idx = np.ascontiguousarray(kept_idx, dtype=np.int32)
    m = idx.shape[1]
    O = np.empty((B, Hq, n, d), dtype=np.float64)
    _load().tfo_attend(_p(qa), _p(ka), _p(va), B, Hq, Hkv, n, d, _p(idx), m,
                       _scale(d, scale), _p(O))
    return O


def attend_rows(q, k, v, kept_idx, rows, scale: float = 0.0):
    """Selected output rows only.  rows: [R, 3] = (b, hq, kept rank).  -> [R, d]."""
    qa, ka, va = _f32(q), _f32(k), _f32(v)
    B, Hq, n, d = qa.shape
    Hkv = ka.shape[1]
    idx = np.ascontiguousarray(kept_idx, dtype=np.int32)
    m = idx.shape[1]
    r = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((r.shape[0], d), dtype=np.float64)
    _load().tfo_attend_rows(_p(qa), _p(ka), _p(va), B, Hq, Hkv, n, d, _p(idx), m,
                            _scale(d, scale), _p(r), r.shape[0], _p(out))
    return out


def filtered_attention(q, k, v, ratio: float, warmup: int = 1, mode: int = FUSE_EQ2,
                       scale: float = 0.0, with_attention: bool = True, ema_gamma=None,
                       inclusive: bool = False):
    """The whole path: score -> fuse -> select -> attend.  Returns a dict of numpy arrays.
    ema_gamma: None for the exact-mean anchor, else the smoothing factor of Eq. 1.
    inclusive: the anchor of a token includes that token."""
    if ema_gamma is None:
        ck = anchor_cosine(k, inclusive=inclusive)
        cv = anchor_cosine(v, inclusive=inclusive)
    else:
        ck = anchor_cosine_ema(k, ema_gamma, inclusive=inclusive)
        cv = anchor_cosine_ema(v, ema_gamma, inclusive=inclusive)
    S = fuse(ck, cv, mode)
    keep, idx, tau = select(S, ratio, warmup)
    out = {"sim_k": ck, "sim_v": cv, "fused": S, "keep": keep, "kept_idx": idx, "tau": tau}
    if with_attention:
        out["O"] = attend(q, k, v, idx, scale)
    return out


class DecodeState:
    """State of the per-token form of the layer (Algorithm 1 called once per new token): the
    anchors, the controller's counters and threshold, and the cache of kept keys / values.
    All arrays are numpy and may be inspected between steps."""

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, capacity: int,
                 target: float, eta: float, tau0: float, warmup: int = 1, mode: int = FUSE_EQ2,
                 scale: float = 0.0, ema_gamma=None, inclusive: bool = False):
        self.B, self.Hq, self.Hkv, self.d, self.capacity = batch, n_q_heads, n_kv_heads, head_dim, capacity
        self.target, self.eta, self.warmup, self.mode = float(target), float(eta), int(warmup), int(mode)
        self.scale = _scale(head_dim, scale)
        self.ema_gamma = ema_gamma
        self.inclusive = bool(inclusive)
        self.anchor_k = np.zeros((batch, n_kv_heads, head_dim), dtype=np.float64)
        self.anchor_v = np.zeros((batch, n_kv_heads, head_dim), dtype=np.float64)
        self.seen = np.zeros(batch, dtype=np.int32)
        self.skipped = np.zeros(batch, dtype=np.int32)
        self.tau = np.full(batch, tau0, dtype=np.float32)
        self.cache_len = np.zeros(batch, dtype=np.int32)
        self.k_cache = np.zeros((batch, n_kv_heads, capacity, head_dim), dtype=np.float32)
        self.v_cache = np.zeros((batch, n_kv_heads, capacity, head_dim), dtype=np.float32)

    def step(self, q, k, v, decide_on=None):
        """One new token per batch row.  q: [B, Hq, d]; k, v: [B, Hkv, d].  decide_on: optional
        [B] float32 scores to decide on instead of the ones computed here.
        Returns (o [B, Hq, d] float64, skip [B] uint8, fused [B] float64)."""
        qa, ka, va = _f32(q), _f32(k), _f32(v)
        assert qa.shape == (self.B, self.Hq, self.d) and ka.shape == va.shape == (self.B, self.Hkv, self.d)
        o = np.empty((self.B, self.Hq, self.d), dtype=np.float64)
        skip = np.empty(self.B, dtype=np.uint8)
        fused = np.empty(self.B, dtype=np.float64)
        dec = None if decide_on is None else np.ascontiguousarray(decide_on, dtype=np.float32)
        rc = _load().tfo_decode_step(
            _p(qa), _p(ka), _p(va), self.B, self.Hq, self.Hkv, self.d,
            0 if self.ema_gamma is None else 1,
            0.0 if self.ema_gamma is None else float(self.ema_gamma), int(self.inclusive),
            self.mode, self.warmup,
            ctypes.c_float(self.target), ctypes.c_float(self.eta), self.scale,
            None if dec is None else _p(dec), _p(self.anchor_k), _p(self.anchor_v),
            _p(self.seen), _p(self.skipped), _p(self.tau), _p(self.cache_len), _p(self.k_cache),
            _p(self.v_cache), self.capacity, _p(o), _p(skip), _p(fused))
        if rc != 0:
            raise OverflowError("decode step: a kept token does not fit the cache")
        return o, skip, fused
