"""The five benchmark configurations (shapes only).

Shapes are the linear layers of LLaMA-7B / LLaMA-70B decoders; they stand in for the
LLaMA-2 checkpoints the paper evaluates (Sec. 5, "Models and datasets"), whose weights are
not available offline.  N = output features (rows of the index matrix), K = input
features.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple


@dataclass(frozen=True)
class LayerSpec:
    name: str
    N: int
    K: int
    count: int = 1  # how many identical-shape matrices the decoder layer holds


@dataclass(frozen=True)
class Config:
    index: int
    label: str
    bits: int
    Ms: Tuple[int, ...]
    layers: Tuple[LayerSpec, ...]

    def matrices(self) -> List[Tuple[int, LayerSpec]]:
        """(matrix_id, spec) for every distinct matrix of the set, in launch order."""
        out = []
        mid = 0
        for spec in self.layers:
            for _ in range(spec.count):
                out.append((mid, spec))
                mid += 1
        return out

    def index_bytes(self) -> int:
        return sum(s.N * s.K * self.bits // 8 * s.count for s in self.layers)

    def weights(self) -> int:
        return sum(s.N * s.K * s.count for s in self.layers)


_LLAMA7B = (
    LayerSpec("qkvo", 4096, 4096, 4),
    LayerSpec("gate_up", 11008, 4096, 2),
    LayerSpec("down", 4096, 11008, 1),
)
_LLAMA70B_MLP = (
    LayerSpec("gate_up", 28672, 8192, 2),
    LayerSpec("down", 8192, 28672, 1),
)

CONFIGS: Tuple[Config, ...] = (
    Config(0, "single 4096x4096, 2-bit, M=1", 2, (1,), (LayerSpec("linear", 4096, 4096, 1),)),
    Config(1, "LLaMA-7B linear set, 3-bit, M=1", 3, (1,), _LLAMA7B),
    Config(2, "LLaMA-7B linear set, 2-bit, M=16", 2, (16,), _LLAMA7B),
    Config(3, "LLaMA-7B linear set, 3-bit, M=2048 (prefill)", 3, (2048,), _LLAMA7B),
    Config(4, "LLaMA-70B MLP, 2-bit, M=1 and M=8", 2, (1, 8), _LLAMA70B_MLP),
)


def get_config(i: int) -> Config:
    return CONFIGS[i]
