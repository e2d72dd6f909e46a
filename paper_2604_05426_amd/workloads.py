"""Seeded synthetic inputs for the multi-LoRA layer.

This module only draws random numbers and rounds them to the input dtype; it holds
none of the layer's arithmetic and imports neither the HIP binding nor the CPU oracle,
so both sides can be fed the same bits.

The shapes stand in for the paper's fine-tuning workloads (Llama-8B / 70B projection
shapes, 4-32 co-resident adapters, ranks 4-128, a few hundred to a few thousand tokens
per adapter, scale alpha / r), which need datasets and model weights that are not
available; the layer's cost depends only on these shapes.

Recipe (one numpy Generator(PCG64(seed)) per workload, draws in this order):
ranks, token counts, alphas (only where the config draws them), then X, W, A_0..,
B_0.., dY as float32 standard normals times sigma:  X, dY ~ N(0,1);  W, B_i ~ N(0, 0.02^2);
A_i ~ N(0, 1/k).  For bf16 workloads each array is then rounded once to bf16
(round-to-nearest-even) and kept as float32 holding the rounded value exactly.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result is float32 with the low
    16 mantissa bits zero."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)) << np.uint32(16)
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are exactly representable in bf16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


@dataclass
class Workload:
    name: str
    dtype: str                 # "f32" or "bf16"
    T: int
    k: int
    n: int
    ranks: List[int]
    scales: List[float]
    offsets: List[int]         # N+1 entries
    X: np.ndarray              # float32, exactly the values of the input dtype
    W: np.ndarray
    A: List[np.ndarray]
    B: List[np.ndarray]
    dY: np.ndarray
    seed: int = 0

    @property
    def N(self) -> int:
        return len(self.ranks)

    @property
    def seg_lens(self) -> List[int]:
        return [self.offsets[i + 1] - self.offsets[i] for i in range(self.N)]

    @property
    def R1(self) -> int:
        return int(sum(t * r for t, r in zip(self.seg_lens, self.ranks)))


def _draw(rng: np.random.Generator, shape, sigma: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return round_to_bf16(a) if dtype == "bf16" else a


def make_workload(name: str, dtype: str, k: int, n: int, ranks: Sequence[int],
                  seg_lens: Sequence[int], scales: Sequence[float], seed: int,
                  rng: Optional[np.random.Generator] = None,
                  b_sigma: float = 0.02) -> Workload:
    """Tensors for a given segmentation (the generator continues from ``rng`` when the
    caller already drew ranks / lengths from it)."""
    if rng is None:
        rng = np.random.Generator(np.random.PCG64(seed))
    ranks = [int(r) for r in ranks]
    seg_lens = [int(t) for t in seg_lens]
    off = [0]
    for t in seg_lens:
        off.append(off[-1] + t)
    T = off[-1]
    X = _draw(rng, (T, k), 1.0, dtype)
    W = _draw(rng, (k, n), 0.02, dtype)
    A = [_draw(rng, (k, r), 1.0 / np.sqrt(k), dtype) for r in ranks]
    B = [_draw(rng, (r, n), b_sigma, dtype) for r in ranks]
    dY = _draw(rng, (T, n), 1.0, dtype)
    return Workload(name=name, dtype=dtype, T=T, k=k, n=n, ranks=ranks,
                    scales=[float(s) for s in scales], offsets=off, X=X, W=W, A=A, B=B,
                    dY=dY, seed=seed)


# (name, input width, output width) of the seven LoRA'd projections of one Llama-3.1-8B block (paper App. B: LoRA on
# all linear layers of attention and MLP; hidden 4096, 8 KV heads of 128, MLP width 14336)
LLAMA8B_BLOCK = [("q_proj", 4096, 4096), ("k_proj", 4096, 1024), ("v_proj", 4096, 1024), ("o_proj", 4096, 4096),
                 ("gate_proj", 4096, 14336), ("up_proj", 4096, 14336), ("down_proj", 14336, 4096)]


def block_workloads(dtype: str, shapes: Sequence, ranks: Sequence[int], seg_lens: Sequence[int],
                    scales: Sequence[float], seed: int, b_sigma: float = 0.02) -> List[Workload]:
    """One Workload per (name, k, n) in ``shapes``, all over the same segmentation (each adapter has one rank and
    one scale for every projection it is attached to); layer l draws from seed + l."""
    return [make_workload(name, dtype, k, n, ranks, seg_lens, scales, seed + l, b_sigma=b_sigma)
            for l, (name, k, n) in enumerate(shapes)]


CONFIG_NAMES = ["tiny_fp32", "llama8b_qproj", "hetero_lengths", "llama8b_mlp_up", "llama70b_mlp"]


def config_shape(index: int):
    """(dtype, k, n, ranks, seg_lens, scales, seed, rng) of benchmark config ``index`` (0-based).
    Only the small integer draws happen here; tensors are drawn by ``config``."""
    seed = index
    rng = np.random.Generator(np.random.PCG64(seed))
    if index == 0:    # tiny fp32 layer, 4 adapters x 64 tokens, scale 2 (alpha = 2r)
        ranks, lens = [4, 8, 8, 16], [64] * 4
        return "f32", 256, 256, ranks, lens, [2.0] * 4, seed, rng
    if index == 1:    # Llama-8B q_proj, 8 adapters x 2048 tokens, scale 16/r
        ranks = [8, 8, 16, 16, 32, 32, 64, 64]
        return "bf16", 4096, 4096, ranks, [2048] * 8, [16.0 / r for r in ranks], seed, rng
    if index == 2:    # heterogeneous lengths: 16 adapters, ranks, lengths, alphas drawn
        ranks = [int(r) for r in rng.choice([4, 8, 16, 32, 64, 128], size=16)]
        lens = [int(t) for t in rng.integers(128, 4097, size=16)]
        alphas = [float(a) for a in rng.choice([8, 16, 32], size=16)]
        return "bf16", 4096, 4096, ranks, lens, [a / r for a, r in zip(alphas, ranks)], seed, rng
    if index == 3:    # Llama-8B MLP up/gate, 32 adapters x 1024 tokens
        ranks = [[8, 16, 32, 64][i % 4] for i in range(32)]
        return "bf16", 4096, 14336, ranks, [1024] * 32, [16.0 / r for r in ranks], seed, rng
    if index == 4:    # Llama-70B MLP, 16 adapters x 2048 tokens
        ranks = [[16, 32, 64, 128][i % 4] for i in range(16)]
        return "bf16", 8192, 28672, ranks, [2048] * 16, [16.0 / r for r in ranks], seed, rng
    raise IndexError(index)


def config(index: int) -> Workload:
    """Benchmark config ``index`` (0-based) with all tensors drawn."""
    dtype, k, n, ranks, lens, scales, seed, rng = config_shape(index)
    return make_workload(CONFIG_NAMES[index], dtype, k, n, ranks, lens, scales, seed, rng=rng)


def small_case(seed: int, dtype: str = "bf16", k: int = 512, n: int = 768,
               ranks: Sequence[int] = (4, 16, 0, 33, 128, 8),
               seg_lens: Sequence[int] = (129, 1, 70, 257, 300, 0),
               scales: Optional[Sequence[float]] = None, b_sigma: float = 0.02) -> Workload:
    """A ragged case the oracle finishes in seconds: several tiles, ragged tails,
    an empty segment, a rank-0 segment, ranks that are not multiples of 8."""
    if scales is None:
        scales = [2.0, 0.5, 1.0, 16.0 / 33.0, 0.125, 3.0][: len(ranks)]
        scales = list(scales) + [1.0] * (len(ranks) - len(scales))
    return make_workload(f"small_seed{seed}", dtype, k, n, ranks, seg_lens, scales, seed,
                         b_sigma=b_sigma)
