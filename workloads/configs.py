"""The five synthetic video-shaped workloads the build is measured and tested on.

Each stands in for an attention block of a video DiT in sparse training
(paper Sec. "Evaluation": latent grids ordered frames x height x width, head
dimension 128, predictor rank 16, 80-98 % sparsity); none of the paper's
datasets or weights is used.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional, Tuple


@dataclass(frozen=True)
class WorkloadConfig:
    index: int                 # position in the benchmark's config list
    name: str
    B: int
    H: int                     # heads held by this GPU
    grid: Tuple[int, int, int]  # latent frames, height, width; L is the product
    d: int                     # head dimension
    r: int                     # predictor rank (the paper's d_lr)
    k: Optional[int]           # KV kept per query, same for every head; None = per-head draw
    k_choices: Tuple[int, ...]  # when k is None: the set each head's k is drawn from
    dtype: str                 # "f32" or "bf16": storage type of Q,K,V,W and outputs
    basis_rank: int            # rank of the Gaussian basis shared by Q and K
    scale: float               # softmax scale applied to q.k

    @property
    def L(self) -> int:
        f, h, w = self.grid
        return f * h * w


def _cfg(index, name, H, grid, d, r, k, dtype, basis_rank, scale_num, k_choices=()):
    return WorkloadConfig(index=index, name=name, B=1, H=H, grid=grid, d=d, r=r, k=k,
                          k_choices=tuple(k_choices), dtype=dtype, basis_rank=basis_rank,
                          scale=scale_num / math.sqrt(d))


CONFIGS = (
    _cfg(0, "tiny_f32_L1k", 2, (8, 8, 16), 64, 16, 128, "f32", 32, 1.0),
    _cfg(1, "bf16_L32k_H24", 24, (16, 32, 64), 128, 16, 2048, "bf16", 64, 2.0),
    _cfg(2, "bf16_L128k_H6", 6, (32, 64, 64), 128, 16, 8192, "bf16", 64, 2.0),
    _cfg(3, "bf16_L64k_H24_hetero_k", 24, (16, 64, 64), 128, 32, None, "bf16", 64, 2.0,
         k_choices=(512, 1024, 2048, 4096, 8192, 16384)),
    _cfg(4, "bf16_L512k_H2", 2, (64, 64, 128), 128, 32, 16384, "bf16", 128, 2.0),
)


def get_config(index: int) -> WorkloadConfig:
    return CONFIGS[index]
