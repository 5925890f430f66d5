"""Seeded synthetic inputs for paged decode attention over prefix-aliased KV.

This module only *draws inputs*: token streams with a prescribed sharing
structure, query vectors and KV pool contents.  It holds none of the method's
arithmetic (no hashing, no block-table construction, no attention), so both the
CPU oracle's tests and the HIP path's tests/bench can feed from it without
sharing any code of the method itself.

Shapes follow the workloads the paper motivates (Section 3: a Llama-3-8B-shaped
layer, 16-token KV blocks, batches whose requests share one long prefix or fall
into several prefix groups, and a no-sharing control), with random token ids
standing in for the paper's dataset prompts: only lengths and the sharing
structure reach this path.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np

BLOCK = 16                 # tokens per KV block (Section 3, experimental setup)
VOCAB = 32000              # token ids are uniform in [0, VOCAB)
SEED_BASE = 20260506 * 10  # per-config seed = SEED_BASE + config index
BF16_NAN = np.uint16(0x7FC0)


# --------------------------------------------------------------------------
# bf16 <-> fp32 on raw bits (round to nearest even), used only to *draw* bf16
# inputs and to hand exact values to whoever consumes them.
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Spec:
    """One synthetic batch shape.

    groups: one (n_requests, prefix_len) pair per prefix group; requests of a
    group start with the same prefix_len tokens.  prefix_len == 0 means the
    requests share nothing.  suffix: inclusive range of unique-suffix lengths.
    interleave: batch order cycles through the groups (arrival order) instead
    of listing each group contiguously.
    """
    name: str
    index: int
    dtype: str                       # "f32" | "bf16"
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    groups: Tuple[Tuple[int, int], ...]
    suffix: Tuple[int, int]
    interleave: bool = False
    pool_factor: float = 1.0         # pool size = ceil(pool_factor * live blocks)
    perm_seed: int = 0               # 0: blocks handed out 0,1,2,...; else seeded shuffle
    q_gain: float = 1.0              # multiplies q ("peaked" softmax variants)

    @property
    def batch(self) -> int:
        return sum(n for n, _ in self.groups)

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index


# The five batch shapes the measurement is quoted on.
CONFIGS = {
    # fp32 parity shape: 4 requests share 256 tokens, 64 private tokens each.
    "c1": Spec("c1", 1, "f32", 8, 2, 64, ((4, 256),), (64, 64)),
    # Llama-3-8B-shaped layer, one homogeneous batch.
    "c2": Spec("c2", 2, "bf16", 32, 8, 128, ((64, 4096),), (128, 1024)),
    # eight prefix groups mixed into one batch in arrival order.
    "c3": Spec("c3", 3, "bf16", 32, 8, 128, tuple((32, 4096) for _ in range(8)), (128, 1024),
               interleave=True),
    # long shared context, physical blocks scattered in an over-sized pool.
    "c4": Spec("c4", 4, "bf16", 32, 8, 128, ((32, 32768),), (512, 512),
               pool_factor=1.5, perm_seed=0xFEA7FEA7),
    # no sharing: independent contexts (status-quo first-come-first-served batch).
    "c5": Spec("c5", 5, "bf16", 64, 8, 128, ((512, 0),), (512, 4096)),
}


def scaled(spec: Spec, batch_div: int = 1, len_div: int = 1, name: Optional[str] = None) -> Spec:
    """A smaller batch of the same structure (for CPU-time-bounded parity cases).

    Lengths are divided and then nudged off multiples of the block size so that
    ragged tails stay in the mix.
    """
    groups = tuple((max(1, n // batch_div), (p // len_div) // BLOCK * BLOCK) for n, p in spec.groups)
    lo, hi = spec.suffix
    lo2, hi2 = max(1, lo // len_div), max(1, hi // len_div)
    if lo2 == hi2 and lo != hi:
        hi2 = lo2 + BLOCK + 3
    elif lo2 == hi2 and lo2 % BLOCK == 0:
        lo2 = hi2 = lo2 + 5
    return replace(spec, name=name or f"{spec.name}_small", groups=groups, suffix=(lo2, hi2))


@dataclass
class Workload:
    spec: Spec
    tokens: np.ndarray          # int32, all requests back to back
    tok_offsets: np.ndarray     # int64 [B+1]
    group_of: np.ndarray        # int32 [B] prefix group of each request (-1: none)
    q: np.ndarray               # [B, Hq, d] float32, or uint16 bf16 bits
    k_cache: np.ndarray         # [num_blocks, Hkv, 16, d] float32 or uint16 bits
    v_cache: np.ndarray
    num_blocks: int
    perm_seed: int
    max_blocks_per_seq: int

    def request_tokens(self, i: int) -> np.ndarray:
        return self.tokens[self.tok_offsets[i]:self.tok_offsets[i + 1]]

    @property
    def seq_lens(self) -> np.ndarray:
        return np.diff(self.tok_offsets).astype(np.int32)


def draw_tokens(spec: Spec, rng: np.random.Generator):
    """Token streams with the group structure of `spec` (batch order included)."""
    per_group: List[List[np.ndarray]] = []
    for n, plen in spec.groups:
        prefix = rng.integers(0, VOCAB, size=plen, dtype=np.int32)
        reqs = []
        for _ in range(n):
            slen = int(rng.integers(spec.suffix[0], spec.suffix[1] + 1))
            suffix = rng.integers(0, VOCAB, size=slen, dtype=np.int32)
            reqs.append(np.concatenate([prefix, suffix]))
        per_group.append(reqs)
    order: List[Tuple[int, int]] = []
    if spec.interleave:
        most = max(len(g) for g in per_group)
        for r in range(most):
            for gi, g in enumerate(per_group):
                if r < len(g):
                    order.append((gi, r))
    else:
        for gi, g in enumerate(per_group):
            order.extend((gi, r) for r in range(len(g)))
    seqs = [per_group[gi][r] for gi, r in order]
    group_of = np.array([gi if spec.groups[gi][1] > 0 else -1 for gi, _ in order], dtype=np.int32)
    return seqs, group_of


def _draw_normal_bits(rng, shape, dtype, chunk_rows=2048):
    """standard_normal(float32) of `shape`; bf16 configs are rounded to bf16 bits."""
    if dtype == "f32":
        return rng.standard_normal(size=shape, dtype=np.float32)
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(shape[0], -1)
    for r0 in range(0, shape[0], chunk_rows):
        r1 = min(shape[0], r0 + chunk_rows)
        x = rng.standard_normal(size=(r1 - r0, flat.shape[1]), dtype=np.float32)
        flat[r0:r1] = f32_to_bf16_bits(x)
    return out


def generate(spec: Spec, with_kv: bool = True) -> Workload:
    """Draw one batch: tokens, q and the whole KV pool (per *physical* block).

    The KV pool is drawn for every physical block, so whichever block table a
    builder produces, the data under it is defined.  Poisoning of dead slots is
    a separate step (`poison_dead_slots`) because it needs the tables.
    """
    rng = np.random.Generator(np.random.PCG64(spec.seed))
    seqs, group_of = draw_tokens(spec, rng)
    lens = np.array([len(s) for s in seqs], dtype=np.int64)
    tok_offsets = np.zeros(len(seqs) + 1, dtype=np.int64)
    np.cumsum(lens, out=tok_offsets[1:])
    tokens = np.concatenate(seqs).astype(np.int32) if seqs else np.zeros(0, np.int32)

    # live blocks if every group prefix is stored once
    live = 0
    for gi, (n, p) in enumerate(spec.groups):
        live += p // BLOCK
    for i, s in enumerate(seqs):
        p = spec.groups[group_of[i]][1] if group_of[i] >= 0 else 0
        live += -(-(len(s) - (p // BLOCK) * BLOCK) // BLOCK)
    num_blocks = int(np.ceil(spec.pool_factor * live))
    max_nb = int(-(-lens.max() // BLOCK)) if len(seqs) else 0

    B, Hq, Hkv, d = spec.batch, spec.num_q_heads, spec.num_kv_heads, spec.head_dim
    q = rng.standard_normal(size=(B, Hq, d), dtype=np.float32) * np.float32(spec.q_gain)
    if spec.dtype == "bf16":
        q = f32_to_bf16_bits(q)
    if with_kv:
        k_cache = _draw_normal_bits(rng, (num_blocks, Hkv, BLOCK, d), spec.dtype)
        v_cache = _draw_normal_bits(rng, (num_blocks, Hkv, BLOCK, d), spec.dtype)
    else:
        k_cache = v_cache = None
    return Workload(spec, tokens, tok_offsets, group_of, q, k_cache, v_cache,
                    num_blocks, spec.perm_seed, max_nb)


def poison_dead_slots(wl: Workload, block_tables: np.ndarray, seq_lens: np.ndarray) -> None:
    """Overwrite every KV slot no request may read with NaN, in place.

    Dead = blocks no table row references within its length, and the slots past
    seq_len in a request's last (partial) block when no other request owns them.
    A reader that over-reads or forgets the length mask then produces NaN.
    """
    nbk = wl.k_cache.shape[0]
    live_upto = np.zeros(nbk, dtype=np.int32)   # number of leading live slots per block
    for i in range(block_tables.shape[0]):
        L = int(seq_lens[i])
        nb = -(-L // BLOCK)
        if nb == 0:
            continue
        row = block_tables[i, :nb]
        fill = np.full(nb, BLOCK, dtype=np.int32)
        fill[-1] = L - (nb - 1) * BLOCK
        np.maximum.at(live_upto, row, fill)
    nan = BF16_NAN if wl.k_cache.dtype == np.uint16 else np.float32(np.nan)
    slot = np.arange(BLOCK, dtype=np.int32)
    dead = slot[None, :] >= live_upto[:, None]          # [num_blocks, 16]
    for cache in (wl.k_cache, wl.v_cache):
        view = cache.transpose(0, 2, 1, 3)              # [num_blocks, 16, Hkv, d]
        view[dead] = nan


def as_f64(x: np.ndarray) -> np.ndarray:
    """Exact upcast of a drawn array (float32 values or bf16 bits) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)
