"""Seeded synthetic workloads: layer layouts and random q/k/v tensors.

This module holds no attention arithmetic.  It is the one piece shared by the GPU
library's tests/benchmark and the CPU oracle's tests: both sides receive the same
bytes from here.  Tensors are N(0,1) draws from a seeded `torch.Generator`, cast to
the workload's dtype (arXiv 2409.15012 trains 24-layer models with sliding window
s = 1024, a few standard layers and 2-3-way cache sharing among sliding layers:
Section 3 and Section 6; the shapes below stand in for that long-context setting).
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch

FULL = 0
SLIDING = 1

# (kind, window, cache_id) per layer
LayerTuple = Tuple[int, int, int]


def layout_tiny(window: int = 64) -> List[LayerTuple]:
    """4 layers: full (cache 0), sliding (cache 1), sliding sharing 1, full sharing 0."""
    return [(FULL, 0, 0), (SLIDING, window, 1), (SLIDING, window, 1), (FULL, 0, 0)]


def layout_mix24(window: int = 1024) -> List[LayerTuple]:
    """24 layers: 0 and 12 full with private caches; 1-11 and 13-23 sliding in
    sharing groups {1-4, 5-8, 9-11} and {13-16, 17-20, 21-23}."""
    layers: List[LayerTuple] = []
    cid = 0
    for half in range(2):
        layers.append((FULL, 0, cid))
        cid += 1
        for size in (4, 4, 3):
            layers.extend([(SLIDING, window, cid)] * size)
            cid += 1
    return layers


def layout_full24() -> List[LayerTuple]:
    """Standard 24-layer stack: every layer full attention with its own cache."""
    return [(FULL, 0, i) for i in range(24)]


def layout_variant(name: str, n_layers: int = 24, window: int = 1024) -> List[LayerTuple]:
    """A few layouts in the spirit of the variants Section 5.1 and the appendix name
    (their exact per-layer maps are drawn in figures only, so these are stand-ins):
    'ma'        one standard cache at layer 0, read again by every 6th layer; sliding elsewhere, pairs share
    'ma_offset' same with the first standard layer moved to layer 2
    'ma_pairs'  two standard caches (layers 0 and 12), each read by one more standard layer
    'sliding'   every layer sliding with its own ring
    """
    layers: List[LayerTuple] = []
    if name == "sliding":
        return [(SLIDING, window, i) for i in range(n_layers)]
    if name in ("ma", "ma_offset"):
        first = 0 if name == "ma" else 2
        full_at = {first + 6 * t for t in range(4) if first + 6 * t < n_layers}
        next_id, run = 1, 0
        for li in range(n_layers):
            if li in full_at:
                layers.append((FULL, 0, 0))
                run = 0
            else:
                if run % 2 == 0:
                    next_id += 1
                layers.append((SLIDING, window, next_id))
                run += 1
        return layers
    if name == "ma_pairs":
        full_map = {0: 0, 6: 0, 12: 1, 18: 1}
        next_id, run = 1, 0
        for li in range(n_layers):
            if li in full_map:
                layers.append((FULL, 0, full_map[li]))
                run = 0
            else:
                if run % 3 == 0:
                    next_id += 1
                layers.append((SLIDING, window, next_id))
                run += 1
        return layers
    raise ValueError(name)


@dataclass
class Workload:
    name: str
    dtype: str  # "f32" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    layers: List[LayerTuple]
    context: int  # tokens per sequence (uniform) or upper bound (ragged)
    seed: int
    ragged_lo: int = 0  # >0: per-sequence lengths uniform in [ragged_lo, context]
    prefill_len: int = 0
    decode_steps: int = 0
    seq_lens: List[int] = field(default_factory=list)

    def __post_init__(self):
        if not self.seq_lens:
            if self.ragged_lo:
                g = torch.Generator().manual_seed(self.seed + 7919)
                self.seq_lens = torch.randint(self.ragged_lo, self.context + 1, (self.batch,), generator=g).tolist()
            else:
                self.seq_lens = [self.context] * self.batch

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def writer_layers(self) -> List[int]:
        seen, out = set(), []
        for li, (_, _, cid) in enumerate(self.layers):
            if cid not in seen:
                seen.add(cid)
                out.append(li)
        return out


def config(i: int) -> Workload:
    """The five synthetic configurations (index as in the baseline description)."""
    if i == 0:
        return Workload("tiny_fp32", "f32", 1, 4, 4, 64, layout_tiny(64), 256, 1234, prefill_len=256, decode_steps=16)
    if i == 1:
        return Workload("mix24_b8_ctx4096", "bf16", 8, 32, 8, 128, layout_mix24(1024), 4096, 1235, decode_steps=1)
    if i == 2:
        return Workload("mix24_b32_ctx32768", "bf16", 32, 32, 8, 128, layout_mix24(1024), 32768, 1236, decode_steps=1)
    if i == 3:
        return Workload("mix24_prefill_s32768", "bf16", 1, 32, 8, 128, layout_mix24(1024), 32768, 1237, prefill_len=32768)
    if i == 4:
        return Workload("mix24_vs_full24_ragged_b64", "bf16", 64, 32, 8, 128, layout_mix24(1024), 65536, 1238,
                        ragged_lo=1024, decode_steps=1)
    raise ValueError("config index 0..4")


def randn(seed: int, shape: Sequence[int], dtype: torch.dtype, device: str = "cpu") -> torch.Tensor:
    """N(0,1) tensor from a seed, drawn in fp32 on `device` and cast to `dtype`.

    The CPU and GPU generators are different streams: a test picks one device for a
    tensor and hands the same bytes to both sides.
    """
    g = torch.Generator(device=device).manual_seed(int(seed))
    return torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32).to(dtype)


def layer_seed(base: int, layer: int, what: str, step: int = 0) -> int:
    """Distinct seed per (layer, tensor role, step)."""
    role = {"q": 1, "k": 2, "v": 3}[what]
    return base * 1000003 + layer * 1009 + role * 101 + step * 7 + 13
