"""CPU oracle for the KV-cache write step.  TEST INFRASTRUCTURE ONLY.

The step that precedes paged attention: the keys and values of the new tokens are stored into the
paged cache (the PagedAttention layout the paper cites), token t at slot slot_mapping[t] =
block * block_size + offset.  The paper is silent on the step; the reading taken is a pure copy,
a negative slot meaning "padding token, store nothing".  Plain loops, no arithmetic: the result is
bit-exact by definition.
"""
from __future__ import annotations

import numpy as np


def kv_cache_write(k_cache: np.ndarray, v_cache: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, slot_mapping) -> None:
    """k_cache, v_cache: [num_blocks, block_size, Hkv, D], modified in place; k_new, v_new: [T, Hkv, D]."""
    block_size = k_cache.shape[1]
    for t, slot in enumerate(np.asarray(slot_mapping).tolist()):
        if slot < 0:
            continue
        block, offset = divmod(int(slot), block_size)
        for h in range(k_new.shape[1]):
            k_cache[block, offset, h, :] = k_new[t, h, :]
            v_cache[block, offset, h, :] = v_new[t, h, :]
