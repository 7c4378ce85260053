"""ctypes binding of libtokfilt.so (include/tokfilt.h): same names, argument marshalling only.

PyTorch tensors are used as device buffers (data_ptr) and torch streams as HIP streams; every
step of the path runs in the library's kernels.  There is no fallback: if the shared object is
missing or cannot be loaded, importing a function from here raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TOKFILT_LIB names another build of the same library (e.g. a kernel variant under test)
LIB_PATH = os.environ.get("TOKFILT_LIB") or os.path.join(_HERE, "libtokfilt.so")

TF_OK, TF_ERR_INVALID_ARG, TF_ERR_UNSUPPORTED, TF_ERR_WORKSPACE_TOO_SMALL, TF_ERR_DEVICE = range(5)
TF_F32, TF_BF16 = 0, 1
TF_FUSE_EQ2, TF_FUSE_INVVAR, TF_FUSE_KEY_ONLY, TF_FUSE_VALUE_ONLY = range(4)
TF_ANCHOR_MEAN, TF_ANCHOR_EMA = 0, 1
TF_N_STAGES = 6
STAGE_NAMES = ("score", "fuse", "select", "compact", "zero_rows", "attend")

EXPORTS = ("tf_create", "tf_destroy", "tf_status_string", "tf_last_error", "tf_keep_count",
           "tf_workspace_bytes", "tf_score", "tf_select", "tf_attend", "tf_filtered_attention",
           "tf_stage_timing_enable", "tf_stage_timing_read", "tf_probe_hbm_read",
           "tf_probe_mfma_bf16", "tf_tail_schedule", "tf_filtered_attention_layers",
           "tf_select_online", "tf_attend_ragged", "tf_filtered_attention_online",
           "tf_decode_workspace_bytes", "tf_decode_init", "tf_decode_step", "tf_decode_prefill",
           "tf_filtered_attention_static")
TF_STATIC_SCRATCH_BYTES = 16 << 20


class tf_params(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("seq", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3),
                ("o_stride", ctypes.c_int64 * 3), ("prune_ratio", ctypes.c_double),
                ("warmup", ctypes.c_int32), ("fusion", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("anchor", ctypes.c_int32),
                ("ema_gamma", ctypes.c_float), ("anchor_inclusive", ctypes.c_int32)]


class tf_decode_state(ctypes.Structure):
    _fields_ = [("anchor_k", ctypes.c_void_p), ("anchor_v", ctypes.c_void_p),
                ("seen", ctypes.c_void_p), ("skipped", ctypes.c_void_p), ("tau", ctypes.c_void_p),
                ("cache_len", ctypes.c_void_p), ("overflow", ctypes.c_void_p),
                ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("capacity", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class TokfiltError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("tokfilt: %s (status %d)" % (message, status))
        self.status = status


_lib = None


def lib():
    """The loaded shared object.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2512_07090_amd.build` "
                              "(there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        pp = ctypes.POINTER(tf_params)
        L.tf_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
        L.tf_create.restype = ctypes.c_int
        L.tf_destroy.argtypes = [vp]
        L.tf_destroy.restype = None
        L.tf_status_string.argtypes = [ctypes.c_int]
        L.tf_status_string.restype = ctypes.c_char_p
        L.tf_last_error.argtypes = [vp]
        L.tf_last_error.restype = ctypes.c_char_p
        L.tf_keep_count.argtypes = [i32, ctypes.c_double]
        L.tf_keep_count.restype = i32
        L.tf_workspace_bytes.argtypes = [pp]
        L.tf_workspace_bytes.restype = sz
        L.tf_score.argtypes = [vp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tf_select.argtypes = [vp, pp, vp, vp, vp, vp, vp, sz, vp]
        L.tf_attend.argtypes = [vp, pp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.tf_filtered_attention.argtypes = [vp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tf_filtered_attention_static.argtypes = [vp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.tf_filtered_attention_static.restype = ctypes.c_int
        L.tf_stage_timing_enable.argtypes = [vp, ctypes.c_int]
        L.tf_stage_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        flt = ctypes.c_float
        L.tf_select_online.argtypes = [vp, pp, flt, flt, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tf_attend_ragged.argtypes = [vp, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tf_filtered_attention_online.argtypes = [vp, pp, flt, flt] + [vp] * 10 + [sz, vp]
        for name in ("tf_select_online", "tf_attend_ragged", "tf_filtered_attention_online"):
            getattr(L, name).restype = ctypes.c_int
        dp = ctypes.POINTER(ctypes.c_double)
        vpp = ctypes.POINTER(vp)
        L.tf_tail_schedule.argtypes = [i32, ctypes.c_double, ctypes.c_double, dp, ctypes.POINTER(i32)]
        L.tf_tail_schedule.restype = ctypes.c_int
        L.tf_filtered_attention_layers.argtypes = [vp, pp, i32, dp] + [vpp] * 8 + [vp, sz, vp]
        L.tf_filtered_attention_layers.restype = ctypes.c_int
        sp = ctypes.POINTER(tf_decode_state)
        L.tf_decode_workspace_bytes.argtypes = [pp]
        L.tf_decode_workspace_bytes.restype = sz
        L.tf_decode_init.argtypes = [vp, pp, sp, flt, vp]
        L.tf_decode_init.restype = ctypes.c_int
        L.tf_decode_step.argtypes = [vp, pp, flt, sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tf_decode_step.restype = ctypes.c_int
        L.tf_decode_prefill.argtypes = [vp, pp, flt, flt, sp] + [vp] * 9 + [sz, vp]
        L.tf_decode_prefill.restype = ctypes.c_int
        L.tf_probe_hbm_read.argtypes = [vp, vp, sz, vp, vp, ctypes.POINTER(ctypes.c_double)]
        L.tf_probe_mfma_bf16.argtypes = [vp, i32, vp, vp, ctypes.POINTER(ctypes.c_double)]
        for name in ("tf_score", "tf_select", "tf_attend", "tf_filtered_attention",
                     "tf_stage_timing_enable", "tf_stage_timing_read", "tf_probe_hbm_read",
                     "tf_probe_mfma_bf16"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_params(q_shape, kv_shape, dtype: torch.dtype, prune_ratio: float, warmup: int = 1,
                fusion: int = TF_FUSE_EQ2, softmax_scale: float = 0.0, q_stride=None,
                kv_stride=None, o_stride=None, ema_gamma=None,
                anchor_inclusive: bool = False) -> tf_params:
    """tf_params for contiguous [B, H, n, d] tensors unless strides (in elements, for batch,
    head, position) are given.  ema_gamma: None for the exact-mean anchor, else the smoothing
    factor of the incremental anchor.  anchor_inclusive: a token's anchor includes the token."""
    B, Hq, n, d = q_shape
    Hkv = kv_shape[1]
    p = tf_params()
    p.batch, p.n_q_heads, p.n_kv_heads, p.seq, p.head_dim = B, Hq, Hkv, n, d
    p.dtype = TF_F32 if dtype == torch.float32 else TF_BF16
    qs = q_stride or (Hq * n * d, n * d, d)
    ks = kv_stride or (Hkv * n * d, n * d, d)
    os_ = o_stride or (Hq * n * d, n * d, d)
    for i in range(3):
        p.q_stride[i], p.kv_stride[i], p.o_stride[i] = qs[i], ks[i], os_[i]
    p.prune_ratio, p.warmup, p.fusion = float(prune_ratio), int(warmup), int(fusion)
    p.softmax_scale, p.anchor_inclusive = float(softmax_scale), int(bool(anchor_inclusive))
    p.anchor = TF_ANCHOR_MEAN if ema_gamma is None else TF_ANCHOR_EMA
    p.ema_gamma = 0.0 if ema_gamma is None else float(ema_gamma)
    return p


def tf_tail_schedule(n_layers: int, p_global: float, tail_fraction: float):
    """Per-layer pruning ratios of the tail-focused schedule; returns (ratios, n_tail)."""
    ratios = (ctypes.c_double * max(int(n_layers), 1))()
    n_tail = ctypes.c_int32()
    st = lib().tf_tail_schedule(int(n_layers), float(p_global), float(tail_fraction), ratios,
                                ctypes.byref(n_tail))
    if st != TF_OK:
        raise TokfiltError(st, "tf_tail_schedule: " + tf_status_string(st))
    return [float(x) for x in ratios[:n_layers]], int(n_tail.value)


def tf_status_string(status: int) -> str:
    return lib().tf_status_string(int(status)).decode()


def tf_keep_count(seq: int, prune_ratio: float) -> int:
    return int(lib().tf_keep_count(int(seq), float(prune_ratio)))


def tf_workspace_bytes(p: tf_params) -> int:
    return int(lib().tf_workspace_bytes(ctypes.byref(p)))


def tf_decode_workspace_bytes(p: tf_params) -> int:
    return int(lib().tf_decode_workspace_bytes(ctypes.byref(p)))


class DecodeBuffers:
    """Device memory of one decoding sequence: the state tf_decode_state describes, the
    per-step outputs and the workspace (allocated through torch; nothing is computed here)."""

    def __init__(self, p: tf_params, capacity: int, device="cuda:0"):
        B, Hq, Hkv, d = p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim
        dt = torch.float32 if p.dtype == TF_F32 else torch.bfloat16
        i32 = dict(dtype=torch.int32, device=device)
        self.anchor_k = torch.empty((B, Hkv, d), dtype=torch.float64, device=device)
        self.anchor_v = torch.empty((B, Hkv, d), dtype=torch.float64, device=device)
        self.seen, self.skipped = torch.empty(B, **i32), torch.empty(B, **i32)
        self.cache_len, self.overflow = torch.empty(B, **i32), torch.empty(B, **i32)
        self.tau = torch.empty(B, dtype=torch.float32, device=device)
        self.k_cache = torch.empty((B, Hkv, capacity, d), dtype=dt, device=device)
        self.v_cache = torch.empty((B, Hkv, capacity, d), dtype=dt, device=device)
        self.o = torch.empty((B, Hq, d), dtype=dt, device=device)
        self.skip = torch.empty(B, dtype=torch.uint8, device=device)
        self.fused = torch.empty(B, dtype=torch.float32, device=device)
        self.ws = torch.empty((tf_decode_workspace_bytes(p),), dtype=torch.uint8, device=device)
        st = tf_decode_state()
        for name in ("anchor_k", "anchor_v", "seen", "skipped", "tau", "cache_len", "overflow",
                     "k_cache", "v_cache"):
            setattr(st, name, getattr(self, name).data_ptr())
        st.capacity, st.reserved = int(capacity), 0
        self.state = st


class Context:
    """Owns a tf_ctx.  Methods mirror the C entry points one to one."""

    def tf_decode_init(self, p, state, tau0, stream=None):
        self._check(lib().tf_decode_init(self._h, ctypes.byref(p), ctypes.byref(state),
                                         float(tau0), _stream(stream)))

    def tf_decode_prefill(self, p, eta, tau0, state, Q, K, V, keep, kept_idx, count, fused, O, ws,
                          stream=None):
        self._check(lib().tf_decode_prefill(
            self._h, ctypes.byref(p), float(eta), float(tau0), ctypes.byref(state), _ptr(Q),
            _ptr(K), _ptr(V), _ptr(keep), _ptr(kept_idx), _ptr(count), _ptr(fused), _ptr(O),
            _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))

    def tf_decode_step(self, p, eta, state, q, k, v, o, skip, fused, ws, stream=None):
        self._check(lib().tf_decode_step(
            self._h, ctypes.byref(p), float(eta), ctypes.byref(state), _ptr(q), _ptr(k), _ptr(v),
            _ptr(o), _ptr(skip), _ptr(fused), _ptr(ws),
            0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))

    def __init__(self, device: int = 0):
        self._h = ctypes.c_void_p()
        st = lib().tf_create(ctypes.byref(self._h), int(device))
        if st != TF_OK:
            raise TokfiltError(st, "tf_create failed: " + tf_status_string(st))
        self.device = device

    def close(self):
        if self._h:
            lib().tf_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def tf_last_error(self) -> str:
        return lib().tf_last_error(self._h).decode()

    def _check(self, st: int):
        if st != TF_OK:
            raise TokfiltError(st, self.tf_last_error() or tf_status_string(st))

    def tf_score(self, p, K, V, fused, sim_k, sim_v, ws, stream=None):
        self._check(lib().tf_score(self._h, ctypes.byref(p), _ptr(K), _ptr(V), _ptr(fused),
                                   _ptr(sim_k), _ptr(sim_v), _ptr(ws),
                                   0 if ws is None else ws.numel() * ws.element_size(),
                                   _stream(stream)))

    def tf_select(self, p, fused, keep, kept_idx, tau, ws, stream=None):
        self._check(lib().tf_select(self._h, ctypes.byref(p), _ptr(fused), _ptr(keep),
                                    _ptr(kept_idx), _ptr(tau), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(),
                                    _stream(stream)))

    def tf_attend(self, p, Q, K, V, kept_idx, m, O, ws, stream=None):
        self._check(lib().tf_attend(self._h, ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V),
                                    _ptr(kept_idx), int(m), _ptr(O), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(),
                                    _stream(stream)))

    def tf_filtered_attention(self, p, Q, K, V, keep, kept_idx, fused, tau, O, ws, stream=None):
        self._check(lib().tf_filtered_attention(
            self._h, ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(keep), _ptr(kept_idx),
            _ptr(fused), _ptr(tau), _ptr(O), _ptr(ws),
            0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))

    def tf_filtered_attention_static(self, p, Q, K, V, keep, kept_idx, fused, tau, O, stream=None):
        self._check(lib().tf_filtered_attention_static(
            self._h, ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(keep), _ptr(kept_idx),
            _ptr(fused), _ptr(tau), _ptr(O), _stream(stream)))

    def tf_select_online(self, p, eta, tau0, fused, keep, kept_idx, count, tau, ws, stream=None):
        self._check(lib().tf_select_online(
            self._h, ctypes.byref(p), float(eta), float(tau0), _ptr(fused), _ptr(keep),
            _ptr(kept_idx), _ptr(count), _ptr(tau), _ptr(ws),
            0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))

    def tf_attend_ragged(self, p, Q, K, V, kept_idx, count, O, ws, stream=None):
        self._check(lib().tf_attend_ragged(
            self._h, ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(kept_idx), _ptr(count),
            _ptr(O), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
            _stream(stream)))

    def tf_filtered_attention_online(self, p, eta, tau0, Q, K, V, keep, kept_idx, count, fused,
                                     tau, O, ws, stream=None):
        self._check(lib().tf_filtered_attention_online(
            self._h, ctypes.byref(p), float(eta), float(tau0), _ptr(Q), _ptr(K), _ptr(V),
            _ptr(keep), _ptr(kept_idx), _ptr(count), _ptr(fused), _ptr(tau), _ptr(O), _ptr(ws),
            0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))

    def tf_filtered_attention_layers(self, p, ratios, Q, K, V, keep, kept_idx, fused, tau, O, ws,
                                     stream=None):
        """Q .. O: lists of per-layer tensors (tau may be None)."""
        n_layers = len(ratios)

        def arr(ts):
            if ts is None:
                return None
            return (ctypes.c_void_p * n_layers)(*[None if t is None else t.data_ptr() for t in ts])
        r = (ctypes.c_double * n_layers)(*[float(x) for x in ratios])
        self._check(lib().tf_filtered_attention_layers(
            self._h, ctypes.byref(p), n_layers, r, arr(Q), arr(K), arr(V), arr(keep),
            arr(kept_idx), arr(fused), arr(tau), arr(O), _ptr(ws),
            0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)))

    def tf_stage_timing_enable(self, on: bool):
        self._check(lib().tf_stage_timing_enable(self._h, 1 if on else 0))

    def tf_stage_timing_read(self):
        ms = (ctypes.c_float * TF_N_STAGES)()
        n = ctypes.c_int32()
        self._check(lib().tf_stage_timing_read(self._h, ms, ctypes.byref(n)))
        return [float(x) for x in ms], int(n.value)


    def tf_probe_hbm_read(self, src: torch.Tensor, stream=None) -> float:
        sink = torch.zeros(1, dtype=torch.int32, device=src.device)
        out = ctypes.c_double()
        self._check(lib().tf_probe_hbm_read(self._h, _ptr(src), src.numel() * src.element_size(),
                                            _ptr(sink), _stream(stream), ctypes.byref(out)))
        return float(out.value)

    def tf_probe_mfma_bf16(self, iters: int, stream=None) -> float:
        sink = torch.zeros(1, dtype=torch.float32, device="cuda:%d" % self.device)
        out = ctypes.c_double()
        self._check(lib().tf_probe_mfma_bf16(self._h, iters, _ptr(sink), _stream(stream),
                                             ctypes.byref(out)))
        return float(out.value)


class Buffers:
    """Device outputs and workspace for one parameter set (allocated through torch)."""

    def __init__(self, p: tf_params, device="cuda:0", with_sims: bool = False):
        B, Hq, Hkv, n, d = p.batch, p.n_q_heads, p.n_kv_heads, p.seq, p.head_dim
        self.m = tf_keep_count(n, p.prune_ratio)
        dt = torch.float32 if p.dtype == TF_F32 else torch.bfloat16
        self.keep = torch.empty((B, n), dtype=torch.uint8, device=device)
        self.kept_idx = torch.empty((B, self.m), dtype=torch.int32, device=device)
        self.fused = torch.empty((B, n), dtype=torch.float32, device=device)
        self.tau = torch.empty((B,), dtype=torch.float32, device=device)
        self.O = torch.empty((B, Hq, n, d), dtype=dt, device=device)
        self.ws = torch.empty((tf_workspace_bytes(p),), dtype=torch.uint8, device=device)
        self.sim_k = self.sim_v = None
        if with_sims:
            self.sim_k = torch.empty((B, Hkv, n), dtype=torch.float32, device=device)
            self.sim_v = torch.empty((B, Hkv, n), dtype=torch.float32, device=device)
