"""Seeded synthetic inputs for the partially-linear FFN hot path.

This module only *generates data*: weights, calibration tokens and test tokens
with the shapes and value distributions of the workloads the library is
measured on.  It holds none of the method's arithmetic (no activation, no
fitting, no folding, no quantised predictor); both the CPU checker and the GPU
library are fed the arrays produced here.

All floating-point tensors are returned as numpy float32 arrays whose values
are exactly representable in the requested storage dtype ("f32" or "bf16"),
so widening them to fp64 on one side and narrowing them to bf16 on the other
is lossless.

Workload recipes (all synthetic, seeded; they stand in for a GELU FFN with
hidden size 4x the model width, the shape of the 7B-class models the method was
evaluated on):

  tiny    d=64,   h=256,   fp32, W ~ N(0, 0.02^2), 512 calibration tokens,
          32 test tokens, in-range target t=0.90.
  tiny_hard  as tiny but W1 ~ N(0, 0.2^2) so that pre-activations reach the
          curved part of GELU.
  decode  d=4096, h=16384, bf16, W ~ N(0, 0.02^2) with heavy-tail structure:
          1% of the input columns of W1 and 1% of the neurons' W2 columns are
          scaled by 8 before rounding to bf16.  4096 calibration tokens and
          1024 test tokens ~ N(0,1).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20250110


def _round_chunk_bf16(u: np.ndarray) -> None:
    """In place on the uint32 bit patterns: nearest bfloat16, ties to even."""
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += lsb
    u += np.uint32(0x7FFF)
    u &= np.uint32(0xFFFF0000)
    if nan.any():
        u[nan] |= np.uint32(0x7FC00000)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result is
    float32 holding bf16-representable values."""
    out = np.array(x, dtype=np.float32, order="C", copy=True)
    u = out.reshape(-1).view(np.uint32)
    n = u.shape[0]
    step = 1 << 22
    if n <= step:
        _round_chunk_bf16(u)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(lambda i: _round_chunk_bf16(u[i:i + step]), range(0, n, step)))
    return out


def _rng(seed: int, stream: int, chunk: int = 0) -> np.random.Generator:
    # Philox is counter based: (seed, stream, chunk) selects an independent sequence.
    return np.random.Generator(np.random.Philox(key=[seed, (stream << 32) | chunk]))


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x)
    raise ValueError(f"unknown storage dtype {dtype!r}")


_CHUNK = 1 << 22          # elements per independently keyed chunk
_POOL_THREADS = 8


def normal(seed: int, stream: int, shape, std: float = 1.0, dtype: str = "f32") -> np.ndarray:
    """N(0, std^2) samples of the given shape in the given storage dtype.  The
    flat array is filled in fixed-size chunks, chunk i from the Philox sequence
    keyed (seed, stream, i), so the values do not depend on how many threads
    fill them."""
    n = int(np.prod(shape))
    flat = np.empty(n, np.float32)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def fill(i):
        lo, hi = i * _CHUNK, min(n, (i + 1) * _CHUNK)
        _rng(seed, stream, i).standard_normal(size=hi - lo, dtype=np.float32, out=flat[lo:hi])
        if std != 1.0:
            flat[lo:hi] *= np.float32(std)

    if nchunks <= 1:
        for i in range(nchunks):
            fill(i)
    else:
        with ThreadPoolExecutor(max_workers=_POOL_THREADS) as ex:
            list(ex.map(fill, range(nchunks)))
    return _store(flat.reshape(shape), dtype)


@dataclass
class FFNLayer:
    """One synthetic FFN layer: y = W2 . act(W1 x + b1) + b2."""
    d: int
    h: int
    dtype: str            # "f32" | "bf16"
    W1: np.ndarray        # h x d
    W2: np.ndarray        # d x h
    b1: np.ndarray | None = None   # h
    b2: np.ndarray | None = None   # d
    heavy_inputs: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    heavy_neurons: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))


def make_layer(d: int, h: int, dtype: str, seed: int, *, w1_std: float = 0.02,
               w2_std: float = 0.02, heavy_frac: float = 0.0, heavy_scale: float = 8.0,
               with_bias: bool = False, bias_std: float = 0.05) -> FFNLayer:
    """Weights ~ N(0, std^2).  If heavy_frac > 0, that fraction of W1's input
    columns and of the neurons' W2 columns is multiplied by heavy_scale before
    the values are rounded to the storage dtype."""
    W1 = normal(seed, 1, (h, d), w1_std, "f32")
    W2 = normal(seed, 2, (d, h), w2_std, "f32")
    hin = np.zeros(0, np.int64)
    hne = np.zeros(0, np.int64)
    if heavy_frac > 0.0:
        g = _rng(seed, 3)
        n_in = max(1, int(round(heavy_frac * d)))
        n_ne = max(1, int(round(heavy_frac * h)))
        hin = np.sort(g.choice(d, size=n_in, replace=False))
        hne = np.sort(g.choice(h, size=n_ne, replace=False))
        W1[:, hin] *= np.float32(heavy_scale)
        W2[:, hne] *= np.float32(heavy_scale)
    b1 = b2 = None
    if with_bias:
        b1 = _store(normal(seed, 6, (h,), bias_std), dtype)
        b2 = _store(normal(seed, 7, (d,), bias_std), dtype)
    return FFNLayer(d=d, h=h, dtype=dtype, W1=_store(W1, dtype), W2=_store(W2, dtype),
                    b1=b1, b2=b2, heavy_inputs=hin, heavy_neurons=hne)


def make_tokens(n: int, d: int, dtype: str, seed: int, stream: int, std: float = 1.0) -> np.ndarray:
    """n token vectors ~ N(0, std^2), n x d."""
    return normal(seed, stream, (n, d), std, dtype)


STREAM_CAL = 4
STREAM_TEST = 5


@dataclass
class Workload:
    name: str
    layer: FFNLayer
    X_cal: np.ndarray     # n_cal x d
    X_test: np.ndarray    # n_test x d
    coverage: float       # in-range target t (fallback rate ~ 1 - t)
    act: str = "gelu_erf"


def workload_seed(config: int, layer: int = 0) -> int:
    return BASE_SEED + 1000 * config + layer


def tiny(hard: bool = False, with_bias: bool = False, n_cal: int = 512, n_test: int = 32,
         coverage: float = 0.90) -> Workload:
    seed = workload_seed(0, 1 if hard else 0)
    lay = make_layer(64, 256, "f32", seed, w1_std=0.2 if hard else 0.02, with_bias=with_bias)
    return Workload("tiny_hard" if hard else "tiny", lay,
                    make_tokens(n_cal, 64, "f32", seed, STREAM_CAL),
                    make_tokens(n_test, 64, "f32", seed, STREAM_TEST), coverage)


def decode(layer: int = 0, *, d: int = 4096, h: int = 16384, n_cal: int = 4096,
           n_test: int = 1024, coverage: float = 0.95, dtype: str = "bf16",
           config: int = 1) -> Workload:
    """The 7B-class decode layer (or a scaled-down copy with the same recipe)."""
    seed = workload_seed(config, layer)
    lay = make_layer(d, h, dtype, seed, heavy_frac=0.01, heavy_scale=8.0)
    return Workload(f"decode_d{d}_h{h}_L{layer}", lay,
                    make_tokens(n_cal, d, dtype, seed, STREAM_CAL),
                    make_tokens(n_test, d, dtype, seed, STREAM_TEST), coverage)
