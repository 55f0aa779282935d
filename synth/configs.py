"""The five workloads: shapes, seeds, mask tail, head grouping and split plans."""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Tuple

BASE_SEED = 251112056


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    H: int
    d: int
    Sq: int
    Skv: int
    kv_valid_len: int
    unit_rms: bool
    latent_grid: Tuple[int, int, int]
    text_tokens: int = 0
    heads_per_group: int = 0                      # >0: run through the head-chunk scheduler
    query_ranges: Tuple[Tuple[int, int], ...] = field(default_factory=tuple)   # (offset, length)
    key_chunks: Tuple[Tuple[int, int], ...] = field(default_factory=tuple)     # (offset, length)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def flops(self) -> int:
        return 4 * self.Sq * self.Skv * self.d * self.H * self.B


def _split_pct(S, pcts):
    """Contiguous ranges: floor(p*S) each, the last takes the remainder."""
    out, off = [], 0
    for i, p in enumerate(pcts):
        n = S - off if i == len(pcts) - 1 else int(math.floor(p * S))
        out.append((off, n))
        off += n
    return tuple(out)


_S720 = 33 * 45 * 80 + 256       # 119 056
_S544 = 33 * 34 * 60 + 256       # 67 576

CONFIGS = {
    1: Workload("c1_tiny", 1, 1, 2, 64, 1024, 1024, 1024, False, (4, 16, 16)),
    2: Workload("c2_lowres_clip", 2, 1, 24, 128, 9600, 9600, 9600, True, (8, 30, 40)),
    3: Workload("c3_544x960_group", 3, 1, 3, 128, _S544, _S544, _S544 - 100, True, (33, 34, 60), 256),
    4: Workload("c4_720p_headchunk", 4, 1, 24, 128, _S720, _S720, _S720, True, (33, 45, 80), 256,
                heads_per_group=3),
    5: Workload("c5_720p_split_merge", 5, 1, 6, 128, _S720, _S720, _S720, True, (33, 45, 80), 256,
                query_ranges=_split_pct(_S720, (0.40, 0.35, 0.25)),
                key_chunks=tuple((i * (_S720 // 4), _S720 // 4) for i in range(4))),
}


def get_config(i: int) -> Workload:
    return CONFIGS[int(i)]
