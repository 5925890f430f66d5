"""One decode step's growth of the KV history, by its definition (test infrastructure only).

Each decode step appends one token's key and value to every request (Section
2.1); the history is stored in 16-token blocks (Section 3).  Written out:

  extend:  a request whose length is a multiple of K gets the next block of the
           free list (requests in batch order) in column length / K; every
           length grows by one.
  append:  request i's new K/V rows go to block tables[i][(L_i - 1) // K], slot
           (L_i - 1) % K, for every KV head, where L_i already counts the token.

Nothing to pin beyond the statement itself: the tests check the first against the
table-building oracle run on the grown token sequences (a grown request's blocks
are its old ones plus a private one), the second by reading the token back
through the gather used by the attention oracle.
"""
from __future__ import annotations

import numpy as np


def extend(tables: np.ndarray, seq_lens: np.ndarray, free: list, K: int = 16):
    """In place; `free` is the remaining free list (consumed from the front).  Returns the blocks added."""
    added = 0
    for i in range(len(seq_lens)):
        L = int(seq_lens[i])
        if L % K == 0:
            if L // K >= tables.shape[1]:
                raise ValueError("table row has no column left")
            if not free:
                raise MemoryError("KV pool exhausted")
            tables[i, L // K] = free.pop(0)
            added += 1
        seq_lens[i] = L + 1
    return added


def append(k_cache: np.ndarray, v_cache: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
           tables: np.ndarray, seq_lens: np.ndarray, K: int = 16):
    """In place on caches [num_blocks, Hkv, K, d]; k_new, v_new are [B, Hkv, d]."""
    for i in range(len(seq_lens)):
        L = int(seq_lens[i])
        if L <= 0:
            continue
        b = int(tables[i, (L - 1) // K])
        k_cache[b, :, (L - 1) % K, :] = k_new[i]
        v_cache[b, :, (L - 1) % K, :] = v_new[i]
