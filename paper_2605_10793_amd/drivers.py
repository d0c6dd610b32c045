"""Loops over the calibration entry points (orchestration only: every step runs in the library's kernels).

online        Alg. 1 as the paper runs it: every mini-batch is rotated, accumulated and followed at once by its
              Procrustes update; nothing is stored.
offline_iid   the comparison variant of Sec. 4.4 (Table 2): the activations are stored first (here: a device tensor)
              and every update draws its rows i.i.d. from the store, with the same number of rows per update and the
              same number of updates as the online loop.
"""
from __future__ import annotations

from typing import Callable, Iterable, List, Optional

import numpy as np

from . import inputs


def online(cal, batches: Iterable, on_update: Optional[Callable] = None) -> int:
    """step_batch + update_rotation per batch (device tensors).  Returns the number of updates."""
    n = 0
    for X in batches:
        cal.step_batch(X)
        _, st = cal.update_rotation()
        if on_update:
            on_update(n, st)
        n += 1
    return n


def offline_iid(cal, pool, rows_per_update: int, n_updates: int, seed: int, on_batch: Optional[Callable] = None,
                on_update: Optional[Callable] = None) -> List[np.ndarray]:
    """Every update steps `rows_per_update` rows drawn i.i.d. (with replacement) from the stored rows `pool` (2-D
    device tensor).  on_batch(u, idx) runs between the step and its update, on_update(u, stats) after it.
    Returns the row indices drawn for each update."""
    import torch
    drawn = []
    for u in range(n_updates):
        idx = inputs.iid_row_indices(seed, u, pool.shape[0], rows_per_update)
        X = pool.index_select(0, torch.from_numpy(idx).to(pool.device))      # gather: plumbing, not the method
        cal.step_batch(X)
        if on_batch:
            on_batch(u, idx)
        _, st = cal.update_rotation()
        if on_update:
            on_update(u, st)
        drawn.append(idx)
    return drawn
