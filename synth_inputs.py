"""Seeded synthetic inputs for the Book-Keeping clipped-gradient path.

This module is shared by the CPU oracle's tests, the GPU parity tests and the
benchmark.  It holds only workload descriptions and random input generation:
none of the method's arithmetic (norms, clipping, weighted sums, noise) lives
here.

The workloads stand in for the linear layers of GPT-shaped transformer blocks
(paper section 3, forward rule s_l = a_l W_l + b_l with a_l in R^{B x T x d},
s_l in R^{B x T x p}).  The paper measures efficiency from tensor dimensions
alone (appendix "Experiment settings"), so no dataset or weights are needed:
activations are N(0,1) and output gradients are small zero-mean Gaussians.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"
F16 = "f16"

CLIP_STANDARD = 0
CLIP_AUTOMATIC = 1


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # F32, BF16 or F16 storage of a and g
    B: int                          # samples in the micro-batch
    T: int                          # tokens per sample
    layers: Tuple[Tuple[int, int], ...]   # (d_in, d_out) per linear layer
    g_std: float                    # standard deviation of output gradients
    g_layer_scale: bool             # multiply layer l's g by s_l ~ U[0.5, 2)
    clip_mode: int
    R: float
    sigma: float
    stability: float = 0.01
    data_seed: int = 0
    noise_seed: int = 1
    noise_step: int = 0
    shard_count: int = 1            # noise goes to 1/shard_count of the flat gradient
    shard_rank: int = 0
    a_std: float = 1.0              # standard deviation of activations

    @property
    def L(self) -> int:
        return len(self.layers)

    @property
    def psi(self) -> int:
        return sum(d * p for d, p in self.layers)

    def layer_offsets(self) -> List[int]:
        """Start of each layer's [d, p] block in the flattened gradient."""
        offs, acc = [], 0
        for d, p in self.layers:
            offs.append(acc)
            acc += d * p
        return offs

    def noise_range(self) -> Tuple[int, int]:
        """(global element offset, count) of the rank's contiguous shard."""
        n = self.psi // self.shard_count
        return self.shard_rank * n, n


def _gpt_block(d: int) -> Tuple[Tuple[int, int], ...]:
    return ((d, 3 * d), (d, d), (d, 4 * d), (4 * d, d))


WORKLOADS = {
    "cfg0": Workload("cfg0", F32, 4, 8, ((16, 16),), 1.0, False,
                     CLIP_STANDARD, 1.0, 0.5),
    "cfg1": Workload("cfg1", BF16, 16, 256, _gpt_block(768) * 12, 1e-2, True,
                     CLIP_AUTOMATIC, 1.0, 1.0),
    "cfg2": Workload("cfg2", BF16, 8, 512, _gpt_block(1280) * 36, 1e-2, True,
                     CLIP_STANDARD, 1.0, 0.8),
    "cfg3": Workload("cfg3", BF16, 2, 4096, ((768, 768),) * 4, 1e-2, False,
                     CLIP_AUTOMATIC, 1.0, 1.0),
    "cfg4": Workload("cfg4", BF16, 4, 2048, _gpt_block(12288), 10.0 ** -2.5, False,
                     CLIP_STANDARD, 1.0, 1.0, shard_count=8, shard_rank=0),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, layer: int, which: int, sample: int) -> np.random.Generator:
    return np.random.default_rng([seed, layer, which, sample])


def layer_g_scale(w: Workload, layer: int) -> float:
    """Per-layer multiplier s_l of the output gradients (1 when the workload has none)."""
    if not w.g_layer_scale:
        return 1.0
    return float(np.random.default_rng([w.data_seed, layer, 2]).uniform(0.5, 2.0))


def gen_tensor(w: Workload, layer: int, which: int, g_extra_scale: float = 1.0) -> np.ndarray:
    """One layer's activation (which=0, [B,T,d]) or output gradient (which=1, [B,T,p]).

    Returns float32 for F32 workloads, uint16 bfloat16 bit patterns for BF16 workloads and
    numpy float16 (IEEE binary16, rounded to nearest even, subnormals kept) for F16 workloads.  Every (layer, tensor, sample) has its own random stream, so the
    values do not depend on how many threads generate them.
    """
    d, p = w.layers[layer]
    width = d if which == 0 else p
    std = w.a_std if which == 0 else w.g_std * layer_g_scale(w, layer) * g_extra_scale
    out = np.empty((w.B, w.T, width), dtype={F32: np.float32, BF16: np.uint16, F16: np.float16}[w.dtype])

    def one(i: int) -> None:
        x = _rng(w.data_seed, layer, which, i).standard_normal((w.T, width), dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[i] = f32_to_bf16_bits(x) if w.dtype == BF16 else x      # assignment rounds to float16 for F16

    if w.B * w.T * width < (1 << 20):
        for i in range(w.B):
            one(i)
    else:
        with ThreadPoolExecutor(max_workers=min(8, w.B)) as ex:
            list(ex.map(one, range(w.B)))
    return out


def gen_layer(w: Workload, layer: int, g_extra_scale: float = 1.0):
    return gen_tensor(w, layer, 0), gen_tensor(w, layer, 1, g_extra_scale)


def to_f64(x: np.ndarray) -> np.ndarray:
    """Exact widening of stored inputs (float32, float16, or bfloat16 bits) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def small_workload(name: str, dtype: str, B: int, T: int, layers, **kw) -> Workload:
    """Ad-hoc workload for parity tests on ragged shapes."""
    base = dict(g_std=1.0 if dtype == F32 else 1e-2, g_layer_scale=False,
                clip_mode=CLIP_STANDARD, R=1.0, sigma=1.0)
    base.update(kw)
    return Workload(name, dtype, B, T, tuple(tuple(x) for x in layers), **base)
