"""ctypes front-end of the CPU oracle (oracle/skd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports it, and it
never imports the product package.  Argument marshalling only; all arithmetic
is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skd_oracle.c")

OK, ERR_NULL, ERR_SHAPE, ERR_RANGE, ERR_ORDER, ERR_SCHEDULE, ERR_NOMEM = 0, -1, -2, -3, -4, -5, -6


def lib_path(real: str) -> str:
    return os.path.join(_HERE, f"liboracle_{real}.so")


def build(real: str = "f64", force: bool = False) -> str:
    """Compile the oracle with gcc (double or float arithmetic)."""
    out = lib_path(real)
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
        return out
    ctype = {"f64": "double", "f32": "float"}[real]
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
           f"-DORA_REAL={ctype}", _SRC, "-o", out, "-lm"]
    subprocess.run(cmd, check=True)
    return out


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("L", "d", "H", "f", "V", "max_pos")]


_PP = C.POINTER(C.c_void_p)


class _Weights(C.Structure):
    _fields_ = ([(n, C.c_void_p) for n in ("tok_emb", "pos_emb", "lnf_g", "lnf_b", "lm_head")] +
                [(n, _PP) for n in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
                                    "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")])


_LIBS: Dict[str, C.CDLL] = {}


def _lib(real: str) -> C.CDLL:
    if real not in _LIBS:
        lib = C.CDLL(build(real))
        lib.ora_schedule.argtypes = [C.c_int32] * 6
        lib.ora_active_layers.argtypes = [C.c_int32] * 7 + [C.c_void_p]
        lib.ora_new.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        lib.ora_free.argtypes = [C.c_void_p]
        lib.ora_free.restype = None
        lib.ora_kv_len.argtypes = [C.c_void_p, C.c_int32]
        lib.ora_kv_load.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.ora_kv_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.ora_seek.argtypes = [C.c_void_p, C.c_int32]
        lib.ora_seek_ragged.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        lib.ora_column.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                   C.c_void_p, C.c_void_p]
        lib.ora_recompute.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        lib.ora_op_layernorm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        lib.ora_op_linear.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_void_p]
        lib.ora_op_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_void_p]
        lib.ora_op_sample.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_double, C.c_double, C.c_void_p]
        _LIBS[real] = lib
    return _LIBS[real]


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle {where} failed with code {code}")
        self.code = code


def _check(rc: int, where: str) -> int:
    if rc < 0:
        raise OracleError(rc, where)
    return rc


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def threads(real: str = "f64") -> int:
    """OpenMP threads the oracle's parallel loops use."""
    return int(_lib(real).ora_threads())


def schedule(i: int, P: int, N: int, n_min: int, n_max: int, L: int, real: str = "f64") -> int:
    """n(i); raises OracleError on invalid parameters."""
    return _check(_lib(real).ora_schedule(i, P, N, n_min, n_max, L), "schedule")


def schedule_rc(i: int, P: int, N: int, n_min: int, n_max: int, L: int, real: str = "f64") -> int:
    return _lib(real).ora_schedule(i, P, N, n_min, n_max, L)


def active_layers(i: int, P: int, N: int, n_min: int, n_max: int, warmup: int, L: int,
                  real: str = "f64") -> List[int]:
    out = np.zeros(max(L, 1), dtype=np.int32)
    c = _check(_lib(real).ora_active_layers(i, P, N, n_min, n_max, warmup, L, out.ctypes.data), "active_layers")
    return [int(v) for v in out[:c]]


class _Packed:
    """Keeps the fp32 arrays and the C structs that point into them alive."""

    def __init__(self, shape, weights: Dict[str, object]):
        self.shape = _Shape(shape.L, shape.d, shape.H, shape.f, shape.V, shape.max_pos)
        self.keep = []
        w = _Weights()
        for n in ("tok_emb", "pos_emb", "lnf_g", "lnf_b"):
            a = _f32(weights[n])
            self.keep.append(a)
            setattr(w, n, a.ctypes.data)
        lm = weights.get("lm_head")
        if lm is not None:
            a = _f32(lm)
            self.keep.append(a)
            w.lm_head = a.ctypes.data
        else:
            w.lm_head = None
        for n in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"):
            arrs = [_f32(x) for x in weights[n]]
            if len(arrs) != shape.L:
                raise ValueError(f"{n}: expected {shape.L} layers, got {len(arrs)}")
            tab = (C.c_void_p * shape.L)(*[a.ctypes.data for a in arrs])
            self.keep.extend(arrs)
            self.keep.append(tab)
            setattr(w, n, C.cast(tab, _PP))
        self.weights = w


class Decoder:
    """Cached column-by-column decoder (ora_column)."""

    def __init__(self, shape, weights, B: int, N: int, real: str = "f64"):
        self._lib = _lib(real)
        self._p = _Packed(shape, weights)
        self.shape, self.B, self.N = shape, B, N
        h = C.c_void_p()
        _check(self._lib.ora_new(C.byref(self._p.shape), C.byref(self._p.weights), B, N, C.byref(h)), "new")
        self._h = h

    def close(self):
        if self._h:
            self._lib.ora_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kv_len(self, layer: int) -> int:
        return _check(self._lib.ora_kv_len(self._h, layer), "kv_len")

    def kv_read(self, layer: int, b: int):
        """Keys and values layer `layer` holds for row b: two [len][d] float64 arrays."""
        n = self.kv_len(layer)
        K = np.zeros((n, self.shape.d), dtype=np.float64)
        V = np.zeros((n, self.shape.d), dtype=np.float64)
        got = _check(self._lib.ora_kv_read(self._h, layer, b, K.ctypes.data, V.ctypes.data), "kv_read")
        assert got == n
        return K, V

    def kv_load(self, layer: int, K: np.ndarray, V: np.ndarray):
        K, V = _f32(K), _f32(V)
        assert K.shape == V.shape and K.shape[0] == self.B and K.shape[2] == self.shape.d
        _check(self._lib.ora_kv_load(self._h, layer, K.shape[1], K.ctypes.data, V.ctypes.data), "kv_load")

    def seek(self, cols: int, start=None):
        if start is None:
            _check(self._lib.ora_seek(self._h, cols), "seek")
        else:
            st = np.ascontiguousarray(start, dtype=np.int32)
            _check(self._lib.ora_seek_ragged(self._h, cols, st.ctypes.data), "seek_ragged")

    def column_rc(self, i: int, tokens, layers: Sequence[int], real_tok=None, want_logits: bool = True):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        lay = np.ascontiguousarray(list(layers), dtype=np.int32)
        rt = None if real_tok is None else np.ascontiguousarray(real_tok, dtype=np.uint8)
        logits = np.zeros((self.B, self.shape.V), dtype=np.float64) if want_logits else None
        am = np.zeros(self.B, dtype=np.int32)
        rc = self._lib.ora_column(self._h, i, tok.ctypes.data, _ptr(rt), lay.ctypes.data if len(lay) else None,
                                  len(lay), _ptr(logits), am.ctypes.data if want_logits else None)
        return rc, logits, am

    def column(self, i: int, tokens, layers: Sequence[int], real_tok=None, want_logits: bool = True):
        rc, logits, am = self.column_rc(i, tokens, layers, real_tok, want_logits)
        _check(rc, "column")
        return logits, am


def recompute_rc(shape, weights, tokens, layer_on, real_tok=None, real: str = "f64"):
    """Non-cached brute force; tokens [B,C], layer_on [C,L] -> (rc, logits[B,V])."""
    lib = _lib(real)
    p = _Packed(shape, weights)
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    B, Cc = tok.shape
    lo = np.ascontiguousarray(layer_on, dtype=np.uint8)
    assert lo.shape == (Cc, shape.L)
    rt = None if real_tok is None else np.ascontiguousarray(real_tok, dtype=np.uint8)
    logits = np.zeros((B, shape.V), dtype=np.float64)
    rc = lib.ora_recompute(C.byref(p.shape), C.byref(p.weights), B, Cc, tok.ctypes.data, _ptr(rt),
                           lo.ctypes.data, logits.ctypes.data)
    return rc, logits


def recompute(shape, weights, tokens, layer_on, real_tok=None, real: str = "f64") -> np.ndarray:
    rc, logits = recompute_rc(shape, weights, tokens, layer_on, real_tok, real)
    _check(rc, "recompute")
    return logits


def op_layernorm(x, g, b, real: str = "f64") -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    g, b = _f32(g), _f32(b)
    out = np.zeros_like(x)
    _check(_lib(real).ora_op_layernorm(x.ctypes.data, g.ctypes.data, b.ctypes.data, x.shape[0], x.shape[1],
                                       out.ctypes.data), "op_layernorm")
    return out


def op_linear(W, bias, x, real: str = "f64") -> np.ndarray:
    W = _f32(W)
    bias = None if bias is None else _f32(bias)
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.zeros((x.shape[0], W.shape[0]), dtype=np.float64)
    _check(_lib(real).ora_op_linear(W.ctypes.data, _ptr(bias), x.ctypes.data, x.shape[0], W.shape[1], W.shape[0],
                                    out.ctypes.data), "op_linear")
    return out


def op_attention(q, K, V, H: int, valid=None, real: str = "f64") -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    d = q.shape[0]
    va = None if valid is None else np.ascontiguousarray(valid, dtype=np.uint8)
    out = np.zeros(d, dtype=np.float64)
    _check(_lib(real).ora_op_attention(q.ctypes.data, K.ctypes.data, V.ctypes.data, _ptr(va), K.shape[0], H, d // H,
                                       out.ctypes.data), "op_attention")
    return out


def generate(shape, weights, prompts, P: int, N: int, n_min: int, n_max: int, warmup: int = 0, mask=None,
             tape=None, steps: Optional[int] = None, real: str = "f64"):
    """Prefill at full depth, then decode with the SkipDecode layer sets.

    prompts [B,P]; mask [B,P] (1 = real) or None; tape [T,B] teacher-forced
    decode inputs or None for greedy free-running.  Returns a dict with the
    per-step logits ([steps+1, B, V]: entry 0 comes from the last prompt
    column), the tokens fed, the layer sets and the per-layer cache lengths.
    """
    prompts = np.ascontiguousarray(prompts, dtype=np.int32)
    B = prompts.shape[0]
    T = N - P
    steps = T if steps is None else steps
    dec = Decoder(shape, weights, B, N, real)
    all_layers = list(range(shape.L))
    logits = am = None
    for i in range(P):
        rt = None if mask is None else mask[:, i]
        logits, am = dec.column(i, prompts[:, i], all_layers, rt, want_logits=(i == P - 1))
    out_logits = [logits]
    fed, sets = [], []
    for k in range(steps):
        i = P + k
        tok = am if tape is None else np.asarray(tape[k], dtype=np.int32)
        lay = active_layers(i, P, N, n_min, n_max, warmup, shape.L, real)
        logits, am = dec.column(i, tok, lay)
        out_logits.append(logits)
        fed.append(np.array(tok))
        sets.append(lay)
    res = {"logits": np.stack(out_logits), "fed": np.array(fed), "layers": sets,
           "kv_len": [dec.kv_len(l) for l in range(shape.L)]}
    dec.close()
    return res


def op_sample(logits, temperature: float, top_p: float, u: float, real: str = "f64"):
    """Temperature + top-p sampling of one token; returns (token, boundary margin, running-sum margin)."""
    z = np.ascontiguousarray(logits, dtype=np.float64)
    m = np.zeros(2, dtype=np.float64)
    tok = _check(_lib(real).ora_op_sample(z.ctypes.data, z.shape[0], temperature, top_p, u, m.ctypes.data), "op_sample")
    return tok, float(m[0]), float(m[1])
