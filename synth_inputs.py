"""Seeded synthetic inputs for the SkipDecode decode path.

This module only *draws inputs* (weights, prompts, padding lengths, token
tapes) and rounds them to the storage precision.  It contains none of the
method's arithmetic (no schedule, no decoder maths) and is the single piece
shared by the CPU oracle's tests and the HIP path's tests / benchmark: both
sides receive the very same buffers, so the generator is never a parity
variable.

Recipe (stands in for the paper's OPT-1.3B / OPT-6.7B checkpoints and its
E2E / Reddit-TLDR / CNN-DM prompts, Section 3, which are not available here):
  * every matrix, embedding table and bias  ~ N(0, 0.02)
  * LayerNorm gain = 1 + N(0, 0.02), LayerNorm bias ~ N(0, 0.02)
    (non-trivial biases/gains so that a dropped bias or affine term shows up)
  * prompt tokens uniform over [0, vocab)
  * ragged batches: per-row real prompt length uniform in [lo, hi], left-padded
Each tensor is drawn from its own counter-based Philox stream keyed by
(seed, tensor id), so a tensor's values do not depend on which other tensors
were drawn before it.
"""
from __future__ import annotations

import dataclasses
import os
from typing import Dict, List, Optional

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    L: int          # num_decoder_layers
    d: int          # d_model
    H: int          # attention heads
    f: int          # FFN width
    V: int          # vocabulary
    max_pos: int    # rows of the learned position table

    @property
    def dh(self) -> int:
        return self.d // self.H


# The five workload shapes of the benchmark contract (model part only).
TINY = ModelShape(L=4, d=256, H=4, f=1024, V=1000, max_pos=64)
OPT_1_3B = ModelShape(L=24, d=2048, H=32, f=8192, V=50272, max_pos=2048 + 1024)
OPT_6_7B = ModelShape(L=32, d=4096, H=32, f=16384, V=50272, max_pos=2048 + 1024)

_PER_LAYER = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
              "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
_GLOBAL = ("tok_emb", "pos_emb", "lnf_g", "lnf_b")


_CHUNK = 1 << 22          # elements per generator stream
_POOL = None


def _pool():
    global _POOL
    if _POOL is None:
        import concurrent.futures
        _POOL = concurrent.futures.ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1)))
    return _POOL


def _stream(seed: int, tensor_id: int, chunk: int = 0) -> np.random.Generator:
    """Counter-based Philox stream keyed by (seed, tensor id, chunk index)."""
    return np.random.Generator(np.random.Philox(key=[int(seed), (int(tensor_id) << 32) | int(chunk)]))


def _normal(seed: int, tid: int, shape, std: float = 0.02, mean: float = 0.0) -> np.ndarray:
    """N(mean, std) fp32 tensor.  The flat tensor is cut into chunks of 2^22 elements, chunk c drawn from its own
    Philox stream (seed, tid, c), so the values do not depend on the number of worker threads."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)

    def fill(c):
        view = out[c * _CHUNK:(c + 1) * _CHUNK]
        _stream(seed, tid, c).standard_normal(size=view.shape, dtype=np.float32, out=view)
        view *= np.float32(std)
        if mean != 0.0:
            view += np.float32(mean)

    nchunks = (n + _CHUNK - 1) // _CHUNK
    if nchunks <= 1:
        fill(0)
    else:
        list(_pool().map(fill, range(nchunks)))
    return out.reshape(shape)


def layer_tensor_shapes(s: ModelShape) -> Dict[str, tuple]:
    return {
        "ln1_g": (s.d,), "ln1_b": (s.d,),
        "wqkv": (3 * s.d, s.d), "bqkv": (3 * s.d,),     # rows: [q | k | v], each d
        "wo": (s.d, s.d), "bo": (s.d,),
        "ln2_g": (s.d,), "ln2_b": (s.d,),
        "w1": (s.f, s.d), "b1": (s.f,),
        "w2": (s.d, s.f), "b2": (s.d,),
    }


def make_weights(s: ModelShape, seed: int = 0, layers: Optional[int] = None) -> Dict[str, object]:
    """fp32 weights.  Per-layer entries are lists of `layers` arrays
    (default s.L).  All matrices are [out_features, in_features] row-major."""
    nl = s.L if layers is None else layers
    w: Dict[str, object] = {
        "tok_emb": _normal(seed, 1, (s.V, s.d)),
        "pos_emb": _normal(seed, 2, (s.max_pos, s.d)),
        "lnf_g": _normal(seed, 3, (s.d,), mean=1.0),
        "lnf_b": _normal(seed, 4, (s.d,)),
    }
    shapes = layer_tensor_shapes(s)
    for j, name in enumerate(_PER_LAYER):
        lst: List[np.ndarray] = []
        for l in range(nl):
            tid = 1000 + 100 * l + j
            mean = 1.0 if name in ("ln1_g", "ln2_g") else 0.0
            lst.append(_normal(seed, tid, shapes[name], mean=mean))
        w[name] = lst
    return w


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even) and return them
    again as fp32 (a new array).  Used to hand the CPU oracle exactly the weight
    values the bf16 device path stores."""
    out = np.array(a, dtype=np.float32, order="C", copy=True)
    flat = out.reshape(-1).view(np.uint32)

    def rnd(c):
        u = flat[c * _CHUNK:(c + 1) * _CHUNK]
        lsb = (u >> np.uint32(16)) & np.uint32(1)
        lsb += np.uint32(0x7FFF)
        u += lsb                      # finite inputs cannot wrap around
        u &= np.uint32(0xFFFF0000)

    nchunks = (flat.size + _CHUNK - 1) // _CHUNK
    if nchunks <= 1:
        rnd(0)
    else:
        list(_pool().map(rnd, range(nchunks)))
    return out


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already bf16-representable fp32 values (uint16)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def weights_to_bf16_values(w: Dict[str, object]) -> Dict[str, object]:
    out: Dict[str, object] = {}
    for k, v in w.items():
        if isinstance(v, list):
            out[k] = [round_to_bf16(x) for x in v]
        else:
            out[k] = round_to_bf16(v)
    return out


def make_prompts(B: int, P: int, V: int, seed: int = 1) -> np.ndarray:
    """[B, P] int32 tokens uniform over the vocabulary."""
    g = _stream(seed, 7001)
    return g.integers(0, V, size=(B, P), dtype=np.int32)


def make_token_tape(B: int, T: int, V: int, seed: int = 1) -> np.ndarray:
    """[T, B] int32 pre-drawn decode inputs (teacher forcing for timed runs)."""
    g = _stream(seed, 7002)
    return g.integers(0, V, size=(T, B), dtype=np.int32)


def make_ragged_mask(B: int, P: int, lo: int, hi: int, seed: int = 2) -> np.ndarray:
    """[B, P] uint8 left-padding mask: row b has a real length drawn uniformly
    from [lo, hi]; its last `len` columns are 1, the leading ones 0."""
    g = _stream(seed, 7003)
    lens = g.integers(lo, hi + 1, size=(B,))
    m = np.zeros((B, P), dtype=np.uint8)
    for b in range(B):
        m[b, P - int(lens[b]):] = 1
    return m
