"""The five workload shapes.

They take the shapes of the paper's visual-AR workloads (App. B "Models" and
"Static Tree Structures": LlamaGen-style 16384-code dim-8 codebooks on 32x32 /
64x64 token grids, a Lumina-mGPT-style 8192 image codes inside a 65536-wide
logit row on a 48x48 grid, trees of 26 and ~58 drafted nodes).  Index 1..5.
"""
from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class Config:
    idx: int
    name: str
    V: int                 # image vocabulary (codebook size)
    ldv: int               # logit row stride (>= vocab_offset + V)
    vocab_offset: int      # column of image token 0 inside a logit row
    D: int                 # codebook embedding dim
    k: int                 # neighbourhood size |B_k|
    lam: float             # multiplicative bound factor lambda
    N: int                 # drafted nodes; rows M = N + 1 (row 0 = root)
    branching: Tuple[int, ...]
    H: int
    Dh: int
    S: int                 # cached context length
    kv_dtype: str          # "f32" | "bf16"
    B: int
    sigma: float           # std of the logits

    @property
    def M(self) -> int:
        return self.N + 1

    @property
    def depth(self) -> int:
        return len(self.branching)

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


_XXL_BRANCH = (6, 3, 2, 2, 1, 1)

CONFIGS = {
    1: Config(1, "tiny", 1024, 1024, 0, 8, 16, 2.0, 15, (4, 2, 1, 1),
              4, 64, 256, "f32", 1, 1.5),
    2: Config(2, "llamagen-l-like", 16384, 16384, 0, 8, 100, 2.0, 26, (4, 2, 2, 1, 1),
              16, 64, 1024, "bf16", 1, 2.0),
    3: Config(3, "llamagen-xxl-like", 16384, 16384, 0, 8, 1000, 3.0, 60, _XXL_BRANCH,
              24, 64, 1024, "bf16", 4, 2.0),
    4: Config(4, "lumina-mgpt-like", 8192, 65536, 4, 256, 1000, 2.0, 60, _XXL_BRANCH,
              32, 128, 2400, "bf16", 1, 2.0),
    5: Config(5, "stress", 16384, 16384, 0, 8, 1000, 3.0, 128, (8, 4, 2, 2, 1, 1, 1, 1),
              24, 64, 4096, "bf16", 16, 2.0),
}


def get_config(idx: int) -> Config:
    return CONFIGS[int(idx)]
