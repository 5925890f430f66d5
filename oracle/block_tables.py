"""Block tables by the plain definition of prefix aliasing (test infrastructure only).

The paper's engines store KV in 16-token blocks and reuse a block across
requests when the block's tokens *and everything before them* agree (Section
2.2, hash-identified block reuse; Section 4.2: two requests agree at level l
iff they share their first l*K tokens).  Written out without any hash:

  request i, column c aliases request j, column c   iff
      c is a full chunk of both and tokens_i[0 : K(c+1)] == tokens_j[0 : K(c+1)].
  A trailing partial chunk is never shared (decode appends into it).

Block ids are fixed by a deterministic allocator: walk requests in batch order
and columns left to right; a column whose whole prefix was already given a
block reuses that block, any other column takes the next id of the free list.
The free list is 0,1,2,... or, for perm_seed != 0, that list shuffled by a
Fisher-Yates pass driven by the generator s += GAMMA; r = mix(s) (constants as
in the hash specification): for k = N-1 down to 1: j = r mod (k+1); swap(k, j).
"""
from __future__ import annotations

import numpy as np

_MASK = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15


def _mix(x: int) -> int:
    x &= _MASK
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _MASK
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _MASK
    x ^= x >> 31
    return x


def free_list(num_blocks: int, perm_seed: int):
    order = list(range(num_blocks))
    if perm_seed != 0:
        s = perm_seed & _MASK
        for k in range(num_blocks - 1, 0, -1):
            s = (s + _GAMMA) & _MASK
            j = _mix(s) % (k + 1)
            order[k], order[j] = order[j], order[k]
    return order


def build_block_tables(seqs, num_blocks: int, perm_seed: int = 0, max_blocks_per_seq=None, K: int = 16):
    """Tables [B, max_blocks] (int32, -1 padded), seq_lens [B], refcount [num_blocks].

    `seqs` is a list of int32 token arrays.  Raises MemoryError when the pool
    has too few blocks.
    """
    B = len(seqs)
    lens = np.array([len(s) for s in seqs], dtype=np.int32)
    need = max((-(-int(L) // K) for L in lens), default=0)
    width = need if max_blocks_per_seq is None else max_blocks_per_seq
    if need > width:
        raise ValueError("max_blocks_per_seq too small")
    tables = np.full((B, width), -1, dtype=np.int32)
    refcount = np.zeros(num_blocks, dtype=np.int32)
    free = free_list(num_blocks, perm_seed)
    nxt = 0
    owner = {}                       # bytes of a whole block-aligned prefix -> block id
    for i, s in enumerate(seqs):
        s = np.ascontiguousarray(s, dtype=np.int32)
        T = len(s)
        for c in range(-(-T // K)):
            full = (c + 1) * K <= T
            key = s[:(c + 1) * K].tobytes() if full else None
            if full and key in owner:
                b = owner[key]
            else:
                if nxt >= num_blocks:
                    raise MemoryError("KV pool exhausted")
                b = free[nxt]
                nxt += 1
                if full:
                    owner[key] = b
            tables[i, c] = b
            refcount[b] += 1
    return tables, lens, refcount
