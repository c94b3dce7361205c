"""Seeded synthetic inputs for the block-sparse FFN prefill path.

This module only draws random tensors and rounds them to bf16.  It holds none
of the method's arithmetic (no pooling, scoring, selection or FFN maths), so
both the CPU oracle's tests and the GPU tests may feed from it.

Every tensor is reproducible on its own: it is drawn from a Philox stream whose
key is (master seed, tensor id), so no tensor depends on the order in which the
others were generated.

Layouts (row-major, one contiguous row of ``d_model`` values per hidden unit):

* ``x``        [T][d_model]          token hidden states
* ``w_gate``   [d_ffn][d_model]      gate projection, neuron-major
* ``w_up``     [d_ffn][d_model]      up projection, neuron-major
* ``w_down``   [d_ffn][d_model]      down projection, neuron-major (row j is
                                     the d_model-vector neuron j adds to y)
* ``w1``       [d_model][r]          predictor first layer
* ``w2``       [r][d_ffn]            predictor second layer
* ``wc1``      [rc][d_model]         compensator first layer, unit-major
* ``wc2``      [rc][d_model]         compensator second layer, unit-major

All tensors are kept as uint16 bf16 bit patterns; ``bf16_to_f32`` gives the
exact values they stand for.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

MASTER_SEED = 20260200397

# tensor ids that salt the Philox key
_TID = {
    "x_n": 1, "x_m": 2, "w_gate": 3, "w_up": 4, "w_down": 5,
    "w1": 6, "w2": 7, "wc1": 8, "wc2": 9, "q_pred": 10, "schedule": 11,
}
_LAYER_STRIDE = 64  # tensor ids of layer l are offset by l * _LAYER_STRIDE


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (round-to-nearest-even), as uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact float32 value of each bf16 bit pattern."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK_ELEMS = 1 << 22   # elements per independently keyed chunk of a large tensor


def _normal_bf16(seed: int, tid: int, shape, scale, chunked=None) -> np.ndarray:
    """bf16 bits of N(0,1) samples times `scale` (a scalar, or one float64 factor
    per column).  Large 2-D tensors are drawn and rounded in row chunks, each from
    its own Philox key (seed, tid * 2^20 + chunk + 1), in parallel; the result
    does not depend on the number of threads."""
    shape = tuple(int(v) for v in (shape if isinstance(shape, (tuple, list)) else (shape,)))

    def make(gen, shp):
        v = gen.standard_normal(shp, dtype=np.float32)
        if np.ndim(scale) == 0:
            v *= np.float32(scale)
        else:
            v = (v.astype(np.float64) * scale).astype(np.float32)
        return f32_to_bf16_bits(v)

    if chunked is None:
        chunked = len(shape) == 2 and int(np.prod(shape)) > _CHUNK_ELEMS
    if not chunked:
        return make(np.random.Generator(np.random.Philox(key=[seed, tid])), shape)
    rows_per = max(1, _CHUNK_ELEMS // shape[1])
    out = np.empty(shape, dtype=np.uint16)
    starts = list(range(0, shape[0], rows_per))

    def fill(ci):
        r0 = starts[ci]
        r1 = min(shape[0], r0 + rows_per)
        gen = np.random.Generator(np.random.Philox(key=[seed, tid * (1 << 20) + ci + 1]))
        out[r0:r1] = make(gen, (r1 - r0, shape[1]))

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(fill, range(len(starts))))
    return out


def _normal(seed: int, tid: int, shape) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=[seed, tid]))
    return gen.standard_normal(shape, dtype=np.float32)


def _uniform(seed: int, tid: int, shape) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=[seed, tid]))
    return gen.random(shape, dtype=np.float64)


def normal_bf16(seed: int, tid: int, shape, std: float) -> np.ndarray:
    """bf16 bits of N(0, std^2) samples."""
    return _normal_bf16(seed, tid, shape, float(std))


@dataclass(frozen=True)
class Shape:
    """One workload's sizes."""
    name: str
    d_model: int
    d_ffn: int
    n_tokens: int
    block: int
    r_pred: int
    r_comp: int
    sparsity: float = 0.5
    n_layers: int = 1

    @property
    def n_blocks(self) -> int:
        return -(-self.n_tokens // self.block)


# The five benchmark configurations (shapes only).
CONFIGS: Dict[str, Shape] = {
    "c0": Shape("c0-tiny", 256, 688, 256, 64, 32, 16),
    "c1": Shape("c1-llama3.2-1b", 2048, 8192, 4096, 128, 64, 32),
    "c2": Shape("c2-llama3.1-8b", 4096, 14336, 8192, 128, 128, 64),
    "c3": Shape("c3-llama3.1-8b-sweep", 4096, 14336, 4096, 64, 128, 64),
    "c4": Shape("c4-qwen2.5-7b-stack", 3584, 18944, 16384, 128, 128, 64, 0.5, 28),
}
C3_BLOCKS = (64, 256)
C3_SPARSITIES = (0.0, 0.25, 0.5, 0.75)


@dataclass
class LayerTensors:
    """bf16 bit patterns of one layer's weights (layouts in the module doc)."""
    w_gate: np.ndarray
    w_up: np.ndarray
    w_down: np.ndarray
    w1: np.ndarray
    w2: np.ndarray
    wc1: np.ndarray
    wc2: np.ndarray
    q_pred: Optional[np.ndarray] = None


def make_hidden(shape: Shape, seed: int = MASTER_SEED,
                n_tokens: Optional[int] = None) -> np.ndarray:
    """x[t][c] = bf16(n[t][c] * exp(0.5 * m[c])), n and m iid N(0,1).

    Heavy-tailed per-channel scales, as LLM hidden states have outlier
    channels.  ``n_tokens`` may cut the prompt short (rows are drawn in order,
    so a prefix of a longer prompt is the same bytes).
    """
    t = shape.n_tokens if n_tokens is None else n_tokens
    m = _normal(seed, _TID["x_m"], (shape.d_model,)).astype(np.float64)
    scale = np.exp(0.5 * m)
    # chunk boundaries depend on d_model only, so a shorter prompt is a prefix of the full one
    rows_per = max(1, _CHUNK_ELEMS // shape.d_model)
    chunked = shape.n_tokens * shape.d_model > _CHUNK_ELEMS
    t_gen = min(shape.n_tokens, -(-t // rows_per) * rows_per) if chunked else shape.n_tokens
    return _normal_bf16(seed, _TID["x_n"], (t_gen, shape.d_model), scale, chunked)[:t]


def make_layer(shape: Shape, layer: int = 0, seed: int = MASTER_SEED,
               with_q_pred: bool = False) -> LayerTensors:
    """Random-init weights of one layer: FFN N(0,0.02), predictor N(0,0.05),
    compensator N(0,0.02); the second parameter is the standard deviation."""
    o = layer * _LAYER_STRIDE
    dm, df, r, rc = shape.d_model, shape.d_ffn, shape.r_pred, shape.r_comp
    lt = LayerTensors(
        w_gate=normal_bf16(seed, o + _TID["w_gate"], (df, dm), 0.02),
        w_up=normal_bf16(seed, o + _TID["w_up"], (df, dm), 0.02),
        w_down=normal_bf16(seed, o + _TID["w_down"], (df, dm), 0.02),
        w1=normal_bf16(seed, o + _TID["w1"], (dm, r), 0.05),
        w2=normal_bf16(seed, o + _TID["w2"], (r, df), 0.05),
        wc1=normal_bf16(seed, o + _TID["wc1"], (rc, dm), 0.02),
        wc2=normal_bf16(seed, o + _TID["wc2"], (rc, dm), 0.02),
    )
    if with_q_pred:
        lt.q_pred = normal_bf16(seed, o + _TID["q_pred"], (dm,), 1.0)
    return lt


def layer_sparsities(n_layers: int, seed: int = MASTER_SEED,
                     lo: float = 0.3, hi: float = 0.7,
                     mean: float = 0.5) -> np.ndarray:
    """Per-layer sparsity draw for the layer-stack workload: uniform in
    [lo, hi], then shifted by a constant so the mean is exactly ``mean``
    (additive renormalisation), then clipped to [0, 1]."""
    s = lo + (hi - lo) * _uniform(seed, _TID["schedule"], (n_layers,))
    s = s + (mean - s.mean())
    return np.clip(s, 0.0, 1.0)


def integer_valued_case(d_model: int, d_ffn: int, n_tokens: int, r: int,
                        seed: int = 7) -> Dict[str, np.ndarray]:
    """Small-integer tensors (exact in bf16, fp32 and fp64) for tie tests:
    every sum the predictor forms is an exact integer, so equal scores are
    exactly equal on any machine.  Values in {-2..2}."""
    gen = np.random.Generator(np.random.Philox(key=[seed, 99]))
    def ints(shape):
        return f32_to_bf16_bits(gen.integers(-2, 3, size=shape).astype(np.float32))
    return {"x": ints((n_tokens, d_model)), "w1": ints((d_model, r)),
            "w2": ints((r, d_ffn))}
