"""Thin ctypes binding of libskd.so (include/skd.h): argument marshalling only.

Every step of the decode path runs inside the HIP library; there is no Python
or CPU fallback.  If the library has not been built, loading fails loudly.
PyTorch is used by callers only to own device memory and streams; this module
itself needs numpy and ctypes.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libskd.so")

OK, ERR_NULL, ERR_SHAPE, ERR_RANGE, ERR_ORDER, ERR_SCHEDULE, ERR_NOMEM, ERR_HIP = 0, -1, -2, -3, -4, -5, -6, -7
BF16, FP32 = 0, 1
HOST, DEVICE = 0, 1
W_FP32, W_BF16 = 0, 1

EXPORTS = ["skd_schedule", "skd_active_layers", "skd_create", "skd_create_with_schedule", "skd_state_active_layers", "skd_prefill", "skd_decode_step",
           "skd_logits_argmax", "skd_logits_argmax_noalloc", "skd_logits_sample", "skd_rewind", "skd_profile_enable", "skd_profile_read", "skd_kv_len", "skd_kv_pages_reserved", "skd_kv_pages_dense", "skd_synchronize",
           "skd_debug_read_hidden", "skd_debug_kv_load", "skd_debug_kv_read", "skd_destroy", "skd_strerror",
           "skd_last_hip_error"]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "L", "d_model", "n_heads", "ffn", "vocab", "max_pos",
        "batch", "prompt_size", "sequence_length", "n_min", "n_max", "warmup",
        "page_tokens", "dtype", "io_on_device")]


_PP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = ([("location", C.c_int32), ("elem", C.c_int32)] +
                [(n, C.c_void_p) for n in ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "lm_head")] +
                [(n, _PP) for n in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
                                    "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")])


PROF_CLASSES = ("embed_ln", "gemm_qkv", "attention", "gemm_out", "reduce_ln", "gemm_ffn1", "gemm_ffn2", "lm_head",
                "argmax", "other")
PER_LAYER = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")

_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Load libskd.so (built by paper_2307_02628_amd._build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2307_02628_amd._build); "
                               "there is no fallback path")
        l = C.CDLL(LIB_PATH)
        l.skd_schedule.argtypes = [C.c_int32] * 6
        l.skd_active_layers.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
        l.skd_create.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_create_with_schedule.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_state_active_layers.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        l.skd_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_decode_step.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        l.skd_logits_argmax.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_logits_argmax_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_logits_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        l.skd_rewind.argtypes = [C.c_void_p, C.c_int32]
        l.skd_profile_enable.argtypes = [C.c_void_p, C.c_int32]
        l.skd_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_kv_len.argtypes = [C.c_void_p, C.c_int32]
        l.skd_kv_pages_reserved.argtypes = [C.c_void_p]
        l.skd_kv_pages_reserved.restype = C.c_int64
        l.skd_kv_pages_dense.argtypes = [C.c_void_p]
        l.skd_kv_pages_dense.restype = C.c_int64
        l.skd_synchronize.argtypes = [C.c_void_p]
        l.skd_debug_read_hidden.argtypes = [C.c_void_p, C.c_void_p]
        l.skd_debug_kv_load.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        l.skd_debug_kv_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        l.skd_destroy.argtypes = [C.c_void_p]
        l.skd_destroy.restype = None
        l.skd_strerror.argtypes = [C.c_int]
        l.skd_strerror.restype = C.c_char_p
        l.skd_last_hip_error.argtypes = []
        _lib = l
    return _lib


class SkdError(RuntimeError):
    def __init__(self, code: int, where: str):
        msg = lib().skd_strerror(code).decode()
        extra = f" (hipError {lib().skd_last_hip_error()})" if code == ERR_HIP else ""
        super().__init__(f"{where}: {msg}{extra} [{code}]")
        self.code = code


def _check(rc: int, where: str) -> int:
    if rc < 0:
        raise SkdError(rc, where)
    return rc


def skd_schedule(t: int, prompt_size: int, sequence_length: int, n_min: int, n_max: int, L: int) -> int:
    """n(t), or a negative error code (no exception: mirrors the C call)."""
    return lib().skd_schedule(t, prompt_size, sequence_length, n_min, n_max, L)


def skd_active_layers(t: int, cfg: Config) -> List[int]:
    out = (C.c_int32 * max(cfg.L, 1))()
    n = _check(lib().skd_active_layers(t, C.byref(cfg), out), "skd_active_layers")
    return [int(out[i]) for i in range(n)]


def make_config(shape, batch: int, prompt_size: int, sequence_length: int, n_min: int, n_max: int, warmup: int = 0,
                dtype: int = BF16, page_tokens: int = 0, io_on_device: int = 0) -> Config:
    """`shape` needs attributes L, d, H, f, V, max_pos."""
    return Config(shape.L, shape.d, shape.H, shape.f, shape.V, shape.max_pos, batch, prompt_size, sequence_length,
                  n_min, n_max, warmup, page_tokens, dtype, io_on_device)


def _ptr_of(a) -> int:
    if a is None:
        return 0
    if isinstance(a, np.ndarray):
        return a.ctypes.data
    if hasattr(a, "data_ptr"):      # torch tensor (device or host)
        return a.data_ptr()
    return int(a)


class Decoder:
    """One decoding state (skd_create .. skd_destroy)."""

    def __init__(self, cfg: Config, weights: Dict[str, object], location: int = HOST, elem: int = W_FP32,
                 stream: int = 0, n_table=None):
        """weights: dict with tok_emb, pos_emb, lnf_g, lnf_b, optional lm_head, and per-layer lists named as in
        skd_weights.  Entries are numpy arrays (host), torch tensors, or raw addresses; fp32, or uint16/bfloat16
        bit patterns with elem=W_BF16."""
        self._lib = lib()
        self.cfg = cfg
        self._keep = []
        w = Weights()
        w.location, w.elem = location, elem

        def prep(a):
            if isinstance(a, np.ndarray):
                a = np.ascontiguousarray(a, dtype=np.float32 if elem == W_FP32 else np.uint16)
            self._keep.append(a)
            return _ptr_of(a)

        for n in ("tok_emb", "pos_emb", "lnf_g", "lnf_b"):
            setattr(w, n, prep(weights[n]))
        w.lm_head = prep(weights["lm_head"]) if weights.get("lm_head") is not None else None
        for n in PER_LAYER:
            lst = weights[n]
            if len(lst) != cfg.L:
                raise ValueError(f"{n}: expected {cfg.L} layers, got {len(lst)}")
            tab = (C.c_void_p * cfg.L)(*[prep(a) for a in lst])
            self._keep.append(tab)
            setattr(w, n, C.cast(tab, _PP))
        h = C.c_void_p()
        if n_table is None:
            _check(self._lib.skd_create(C.byref(cfg), C.byref(w), C.c_void_p(stream), C.byref(h)), "skd_create")
        else:
            tab = np.ascontiguousarray(n_table, dtype=np.int32)
            if tab.shape != (cfg.sequence_length,):
                raise ValueError("n_table needs one entry per position")
            _check(self._lib.skd_create_with_schedule(C.byref(cfg), C.byref(w), C.c_void_p(stream), tab.ctypes.data,
                                                      C.byref(h)), "skd_create_with_schedule")
        self._h = h
        self._keep = []   # the library has copied everything

    # -- lifecycle
    def close(self):
        if getattr(self, "_h", None):
            self._lib.skd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- the four calls of the path
    def prefill_rc(self, tokens, attn_mask=None) -> int:
        if isinstance(tokens, np.ndarray):
            tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        if isinstance(attn_mask, np.ndarray):
            attn_mask = np.ascontiguousarray(attn_mask, dtype=np.uint8)
        return self._lib.skd_prefill(self._h, _ptr_of(tokens), _ptr_of(attn_mask))

    def prefill(self, tokens, attn_mask=None):
        _check(self.prefill_rc(tokens, attn_mask), "skd_prefill")

    def decode_step_rc(self, t: int, tokens_in=None) -> int:
        if isinstance(tokens_in, np.ndarray):
            tokens_in = np.ascontiguousarray(tokens_in, dtype=np.int32)
        return self._lib.skd_decode_step(self._h, t, _ptr_of(tokens_in))

    def decode_step(self, t: int, tokens_in=None):
        _check(self.decode_step_rc(t, tokens_in), "skd_decode_step")

    def logits_argmax(self, want_logits: bool = True):
        """Host-I/O form: returns (tokens[B] int32, logits[B,V] float32 or None)."""
        assert not self.cfg.io_on_device
        tok = np.zeros(self.cfg.batch, dtype=np.int32)
        lg = np.zeros((self.cfg.batch, self.cfg.vocab), dtype=np.float32) if want_logits else None
        _check(self._lib.skd_logits_argmax(self._h, tok.ctypes.data, _ptr_of(lg)), "skd_logits_argmax")
        return tok, lg

    def logits_sample_rc(self, u, temperature: float, top_p: float, want_logits: bool = True):
        """Host-I/O form of skd_logits_sample: returns (rc, tokens[B], logits[B,V] or None)."""
        assert not self.cfg.io_on_device
        uu = np.ascontiguousarray(u, dtype=np.float32)
        tok = np.zeros(self.cfg.batch, dtype=np.int32)
        lg = np.zeros((self.cfg.batch, self.cfg.vocab), dtype=np.float32) if want_logits else None
        rc = self._lib.skd_logits_sample(self._h, uu.ctypes.data, temperature, top_p, tok.ctypes.data, _ptr_of(lg))
        return rc, tok, lg

    def logits_sample(self, u, temperature: float, top_p: float, want_logits: bool = True):
        rc, tok, lg = self.logits_sample_rc(u, temperature, top_p, want_logits)
        _check(rc, "skd_logits_sample")
        return tok, lg

    def logits_sample_device(self, u, temperature: float, top_p: float, tokens_out=None, logits_out=None):
        """Device-I/O form: u, tokens_out, logits_out are device pointers / torch tensors; asynchronous."""
        _check(self._lib.skd_logits_sample(self._h, _ptr_of(u), temperature, top_p, _ptr_of(tokens_out),
                                           _ptr_of(logits_out)), "skd_logits_sample")

    def logits_argmax_device(self, tokens_out=None, logits_out=None):
        """Device-I/O form: pointers / torch tensors on the device; asynchronous."""
        _check(self._lib.skd_logits_argmax(self._h, _ptr_of(tokens_out), _ptr_of(logits_out)), "skd_logits_argmax")

    def logits_argmax_noalloc_rc(self, tokens_out=None, logits_out=None) -> int:
        """skd_logits_argmax_noalloc (device I/O only): the return code, no exception."""
        return self._lib.skd_logits_argmax_noalloc(self._h, _ptr_of(tokens_out), _ptr_of(logits_out))

    def rewind(self, t: int):
        _check(self._lib.skd_rewind(self._h, t), "skd_rewind")

    def profile_enable(self, mode):
        """0 / False: off; 1 / True: each kernel's own begin and end time stamps; 2: event brackets on the stream."""
        _check(self._lib.skd_profile_enable(self._h, int(mode)), "skd_profile_enable")

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        ms = (C.c_double * len(PROF_CLASSES))()
        n = (C.c_int64 * len(PROF_CLASSES))()
        _check(self._lib.skd_profile_read(self._h, ms, n), "skd_profile_read")
        return {name: {"ms": float(ms[i]), "launches": int(n[i])} for i, name in enumerate(PROF_CLASSES)}

    def active_layers(self, t: int) -> List[int]:
        out = (C.c_int32 * max(self.cfg.L, 1))()
        n = _check(self._lib.skd_state_active_layers(self._h, t, out), "skd_state_active_layers")
        return [int(out[i]) for i in range(n)]

    # -- bookkeeping and hooks
    def kv_len(self, layer: int) -> int:
        return _check(self._lib.skd_kv_len(self._h, layer), "skd_kv_len")

    def kv_pages(self):
        return int(self._lib.skd_kv_pages_reserved(self._h)), int(self._lib.skd_kv_pages_dense(self._h))

    def synchronize(self):
        _check(self._lib.skd_synchronize(self._h), "skd_synchronize")

    def read_hidden(self) -> np.ndarray:
        x = np.zeros((self.cfg.batch, self.cfg.d_model), dtype=np.float32)
        _check(self._lib.skd_debug_read_hidden(self._h, x.ctypes.data), "skd_debug_read_hidden")
        return x

    def kv_load(self, cols: int, K: Sequence[Optional[np.ndarray]], V: Sequence[Optional[np.ndarray]], start=None):
        keep = []

        def tab(lst):
            ptrs = []
            for a in lst:
                if a is None:
                    ptrs.append(None)
                else:
                    a = np.ascontiguousarray(a, dtype=np.float32)
                    assert a.shape == (self.cfg.batch, cols, self.cfg.d_model)
                    keep.append(a)
                    ptrs.append(a.ctypes.data)
            return (C.c_void_p * self.cfg.L)(*ptrs)

        kt, vt = tab(K), tab(V)
        st = None if start is None else np.ascontiguousarray(start, dtype=np.int32)
        _check(self._lib.skd_debug_kv_load(self._h, cols, kt, vt, _ptr_of(st)), "skd_debug_kv_load")

    def kv_read(self, layer: int, b: int):
        n = self.kv_len(layer)
        k = np.zeros((n, self.cfg.d_model), dtype=np.float32)
        v = np.zeros((n, self.cfg.d_model), dtype=np.float32)
        _check(self._lib.skd_debug_kv_read(self._h, layer, b, k.ctypes.data, v.ctypes.data), "skd_debug_kv_read")
        return k, v
