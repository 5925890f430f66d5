"""Decode attention by its definition, in float64 (test infrastructure only).

Section 2.1 of the paper: Attention(Q, K, V) = softmax(Q K^T / sqrt(d)) V, and
in decode the current token's query attends to every cached key/value.  Here
each request has one query token; its cached keys/values are found through a
block table over 16-token physical blocks (Section 3, experimental setup).

Layout taken as input (values, not bits):
  q            [B, Hq, d]
  k_cache      [num_blocks, Hkv, block, d]     (same for v_cache)
  block_tables [B, >= ceil(L_i / block)] int   (entries past that are ignored)
  seq_lens     [B] int    number of cached tokens request i attends to
Query head h reads KV head h // (Hq // Hkv).  A request with seq_len 0 yields
a zero row.  No blocking, no running maximum across pieces: gather, score,
softmax, weighted sum.
"""
from __future__ import annotations

import math

import numpy as np


def gather_kv(cache: np.ndarray, table_row: np.ndarray, seq_len: int) -> np.ndarray:
    """Cached vectors of one request, in token order: [Hkv, seq_len, d] float64."""
    block = cache.shape[2]
    nb = -(-seq_len // block)
    picked = cache[np.asarray(table_row[:nb], dtype=np.int64)]        # [nb, Hkv, block, d]
    per_head = np.transpose(picked, (1, 0, 2, 3)).reshape(cache.shape[1], nb * block, cache.shape[3])
    return per_head[:, :seq_len, :].astype(np.float64)


def decode_attention(q, k_cache, v_cache, block_tables, seq_lens, scale=None, requests=None):
    """out[i, h, :] = sum_t softmax_t(q[i,h] . k_t * scale) v_t   (float64).

    scale defaults to 1/sqrt(d).  `requests` restricts the computation to some
    batch rows (the others are returned as NaN) so that large batches can be
    spot-checked.
    """
    q = np.asarray(q, dtype=np.float64)
    B, Hq, d = q.shape
    Hkv = k_cache.shape[1]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    rows = range(B) if requests is None else requests
    for i in rows:
        L = int(seq_lens[i])
        if L == 0:
            out[i] = 0.0
            continue
        K = gather_kv(k_cache, block_tables[i], L)                    # [Hkv, L, d]
        V = gather_kv(v_cache, block_tables[i], L)
        qi = q[i].reshape(Hkv, G, d)
        s = np.matmul(qi, np.transpose(K, (0, 2, 1))) * scale         # [Hkv, G, L]
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[i] = np.matmul(p, V).reshape(Hq, d)
    return out
