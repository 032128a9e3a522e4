"""Seeded synthetic layers and calibration activations.

This module only draws random numbers, rounds them to a storage type and
describes the benchmark layer shapes.  It contains none of the quantization
method's arithmetic, so both the CPU oracle's tests and the GPU path's tests
may take their inputs from here without sharing any method code.

Storage conventions
-------------------
* ``"f32"`` tensors are ``numpy.float32`` arrays.
* ``"bf16"`` tensors are ``numpy.uint16`` arrays holding bfloat16 bit patterns
  (round-to-nearest-even from float32).  ``to_f64`` widens either kind exactly.

The stand-ins follow the shapes of LLaMA-2-7B linear layers and the
128 x 2048-token calibration set of the paper's experimental setup (Sec. 4.1
and the implementation-details appendix); the real calibration text and model
weights are not available, so weights are Gaussian with a few amplified
outlier input columns and activations are per-channel-scaled Gaussians or
heavy-tailed Student-t draws.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
import os

import numpy as np

BASE_SEED = 260119675
_CHUNK = 2048  # tokens per independently seeded block of X

_TENSOR_W = 1
_TENSOR_X = 2
_TENSOR_SCALE = 3
_TENSOR_OUTLIER = 4
_TENSOR_SKETCH = 5
_TENSOR_LOWRANK = 6
_TENSOR_CODEBOOK = 7


# ----------------------------------------------------------------------------
# storage helpers
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (uint16 bf16 bits or float32/64)."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def to_device(a: np.ndarray):
    """Stored numpy tensor (uint16 = bfloat16 bits, float32, float64, uint8) -> torch tensor on the
    current GPU holding the same bits (uint16 becomes torch.bfloat16)."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def store(a64: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return a64.astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a64.astype(np.float32))
    if dtype == "f64":
        return a64.astype(np.float64)
    raise ValueError(dtype)


def _rng(seed: int, layer: int, tensor: int, chunk: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([int(seed), int(layer), int(tensor), int(chunk)])
    return np.random.Generator(np.random.Philox(ss))


# ----------------------------------------------------------------------------
# layer / config descriptions
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerSpec:
    """One linear layer to quantize: W is m x n, activations are t x n."""
    name: str
    m: int
    n: int
    t: int
    dtype: str = "bf16"            # storage type of W and X
    w_sigma: float = 0.02
    outlier_frac: float = 0.005    # share of input columns of W that are amplified
    outlier_mul: float = 20.0
    x_kind: str = "lognormal"      # "lognormal" (per-channel scale) or "student_t"
    x_sigma: float = 1.5           # sigma of log per-channel scale
    x_nu: float = 3.0              # Student-t degrees of freedom
    layer_id: int = 0


@dataclass(frozen=True)
class Config:
    name: str
    layers: tuple
    bits: int
    group: int
    block: int
    damps: tuple = (0.01,)
    seed: int = BASE_SEED
    note: str = ""


_T = 128 * 2048

CONFIGS = {
    "C1": Config(
        "C1",
        (LayerSpec("lin512", 512, 512, 2048, dtype="f32", outlier_frac=0.01,
                   outlier_mul=10.0, x_sigma=1.0, layer_id=10),),
        bits=4, group=128, block=128, note="small fp32 layer"),
    "C2": Config(
        "C2",
        (LayerSpec("attn_proj", 4096, 4096, _T, layer_id=20),),
        bits=4, group=128, block=128, note="Llama-7B-shaped attention projection"),
    "C3": Config(
        "C3",
        (LayerSpec("up_proj", 11008, 4096, _T, x_kind="student_t", layer_id=30),
         LayerSpec("down_proj", 4096, 11008, _T, x_kind="student_t", layer_id=31)),
        bits=3, group=128, block=128, note="MLP pair, heavy-tailed activations"),
    "C4": Config(
        "C4",
        (LayerSpec("attn_proj", 4096, 4096, _T, layer_id=20),),
        bits=2, group=64, block=256, damps=(0.001, 0.01, 0.1),
        note="low-bit stress, damp sweep"),
    "C5": Config(
        "C5",
        tuple(
            [LayerSpec(nm, 4096, 4096, _T, layer_id=50 + i)
             for i, nm in enumerate(("q_proj", "k_proj", "v_proj", "o_proj"))]
            + [LayerSpec("gate_proj", 11008, 4096, _T, layer_id=54),
               LayerSpec("up_proj", 11008, 4096, _T, layer_id=55),
               LayerSpec("down_proj", 4096, 11008, _T, layer_id=56)]),
        bits=3, group=128, block=128, note="full decoder block, 7 linears"),
}


def scaled(spec: LayerSpec, m: int | None = None, n: int | None = None,
           t: int | None = None) -> LayerSpec:
    """Same distributions, different sizes (for parity cases and CPU samples)."""
    return LayerSpec(spec.name, m or spec.m, n or spec.n, t or spec.t, spec.dtype,
                     spec.w_sigma, spec.outlier_frac, spec.outlier_mul, spec.x_kind,
                     spec.x_sigma, spec.x_nu, spec.layer_id)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
def gen_weight(spec: LayerSpec, seed: int = BASE_SEED) -> np.ndarray:
    """W (m x n) in storage form: N(0, w_sigma^2), a few input columns amplified."""
    rng = _rng(seed, spec.layer_id, _TENSOR_W)
    w = rng.standard_normal((spec.m, spec.n), dtype=np.float32).astype(np.float64)
    w *= spec.w_sigma
    n_out = int(round(spec.outlier_frac * spec.n))
    if n_out > 0:
        cols = _rng(seed, spec.layer_id, _TENSOR_OUTLIER).choice(spec.n, n_out, replace=False)
        w[:, cols] *= spec.outlier_mul
    return store(w, spec.dtype)


def gen_weight_with_low_rank_part(spec: LayerSpec, seed: int = BASE_SEED, rank: int = 8,
                                  strength: float = 6.0) -> np.ndarray:
    """gen_weight plus a few strong directions: sum_k c_k a_k b_k^T with unit-norm Gaussian
    a_k, b_k and c_k = strength * w_sigma * sqrt(max(m, n)) / (k + 1), i.e. `strength` times
    the largest singular value of the Gaussian part for k = 0, then decaying.  Trained
    weights have such leading directions; pure Gaussian noise gives a low-rank step
    nothing to find."""
    w = to_f64(gen_weight(spec, seed))
    rng = _rng(seed, spec.layer_id, _TENSOR_LOWRANK)
    for k in range(rank):
        a = rng.standard_normal(spec.m)
        b = rng.standard_normal(spec.n)
        c = strength * spec.w_sigma * np.sqrt(max(spec.m, spec.n)) / (k + 1)
        w += c * np.outer(a / np.linalg.norm(a), b / np.linalg.norm(b))
    return store(w, spec.dtype)


def gen_sketch_vectors(spec: LayerSpec, r: int, seed: int = BASE_SEED) -> np.ndarray:
    """r x n float32 standard normal draws: the random vectors a sketching method asks for,
    drawn here so that every implementation under test sees the same ones."""
    rng = _rng(seed, spec.layer_id, _TENSOR_SKETCH)
    return rng.standard_normal((r, spec.n), dtype=np.float32)


def gen_codebook(W64: np.ndarray, entries: int, dim: int, spec: LayerSpec, seed: int = BASE_SEED) -> np.ndarray:
    """entries x dim float32 codebook drawn at random for a vector quantizer: distinct pieces of
    `dim` consecutive columns (starting at a multiple of dim) of the given weight matrix, picked
    uniformly -- a random, untrained codebook in the weights' own units."""
    rng = _rng(seed, spec.layer_id, _TENSOR_CODEBOOK)
    m, n = W64.shape
    pieces = np.ascontiguousarray(W64[:, : (n // dim) * dim]).reshape(-1, dim)
    pick = rng.choice(pieces.shape[0], size=min(entries, pieces.shape[0]), replace=False)
    cb = pieces[pick].astype(np.float32)
    if cb.shape[0] < entries:   # a layer smaller than the codebook: fill up with Gaussian entries of the same spread
        extra = rng.standard_normal((entries - cb.shape[0], dim)) * float(np.std(pieces))
        cb = np.vstack([cb, extra.astype(np.float32)])
    return cb


def channel_scales(spec: LayerSpec, seed: int = BASE_SEED) -> np.ndarray:
    if spec.x_kind != "lognormal":
        return np.ones(spec.n)
    g = _rng(seed, spec.layer_id, _TENSOR_SCALE).standard_normal(spec.n)
    return np.exp(spec.x_sigma * g)


def _gen_x_chunk(spec: LayerSpec, seed: int, c: int, rows: int, s: np.ndarray) -> np.ndarray:
    rng = _rng(seed, spec.layer_id, _TENSOR_X, c)
    if spec.x_kind == "lognormal":
        z = rng.standard_normal((_CHUNK, spec.n), dtype=np.float32)
        z *= s.astype(np.float32)
    elif spec.x_kind == "student_t":
        z = rng.standard_t(spec.x_nu, size=(_CHUNK, spec.n)).astype(np.float32)
    else:
        raise ValueError(spec.x_kind)
    z = z[:rows]
    if spec.dtype == "bf16":
        return f32_to_bf16_bits(z)
    return np.ascontiguousarray(z, dtype=np.float32)


def gen_activations(spec: LayerSpec, seed: int = BASE_SEED, t0: int = 0,
                    t1: int | None = None, workers: int | None = None) -> np.ndarray:
    """Rows [t0, t1) of the calibration input X (tokens x channels), storage form.

    Every block of 2048 tokens has its own counter-based stream, so any token
    range can be produced independently and in parallel; t0 must be a multiple
    of 2048.
    """
    t1 = spec.t if t1 is None else t1
    assert t0 % _CHUNK == 0 and 0 <= t0 <= t1
    s = channel_scales(spec, seed)
    out_dtype = np.uint16 if spec.dtype == "bf16" else np.float32
    out = np.empty((t1 - t0, spec.n), dtype=out_dtype)
    chunks = list(range(t0 // _CHUNK, (t1 + _CHUNK - 1) // _CHUNK))

    def work(c):
        lo = c * _CHUNK
        rows = min(_CHUNK, t1 - lo)
        out[lo - t0: lo - t0 + rows] = _gen_x_chunk(spec, seed, c, rows, s)

    workers = workers or min(16, os.cpu_count() or 1)
    if len(chunks) <= 1 or workers <= 1:
        for c in chunks:
            work(c)
    else:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(work, chunks))
    return out
