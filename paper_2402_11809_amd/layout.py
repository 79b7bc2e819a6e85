"""Host-side description of a step block: which rows are mask rows and which group they
belong to (Eq. 2 of the paper restricted to the rows that are not cached yet)."""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class BlockLayoutSpec:
    is_mask: np.ndarray  # uint8 [L]
    group: np.ndarray    # int32 [L]

    @property
    def n_rows(self) -> int:
        return int(self.is_mask.shape[0])

    @property
    def n_groups(self) -> int:
        return int(self.group.max()) + 1


def grouped_layout(n_groups: int, masks_per_group: int) -> BlockLayoutSpec:
    """n_groups groups, each one non-mask row followed by masks_per_group mask rows."""
    is_mask, group = [], []
    for g in range(n_groups):
        is_mask += [0] + [1] * masks_per_group
        group += [g] * (1 + masks_per_group)
    return BlockLayoutSpec(np.asarray(is_mask, dtype=np.uint8), np.asarray(group, dtype=np.int32))


def paper_layout(k: int) -> BlockLayoutSpec:
    """[x_l, M^k, c_1, M^k, ..., c_k, M^k]: (k+1)^2 rows."""
    return grouped_layout(k + 1, k)


def first_step_layout(k: int) -> BlockLayoutSpec:
    """[x_l, M^k]: the first iteration has no candidates to verify yet."""
    return grouped_layout(1, k)


def prefill_layout(n: int) -> BlockLayoutSpec:
    """n committed tokens, no masks: Eq. 3 degenerates to the causal mask."""
    return grouped_layout(n, 0)
