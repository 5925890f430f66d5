"""Chunked cumulative prefix hashes (test infrastructure only).

Follows the chunk-parallel formulation of the paper's prefix hash computation
(Appendix "Prefix Hash Computation", Algorithm 2): every chunk of K tokens is
hashed on its own into a leaf value, and the leaves are chained, h_c =
Hash(h_{c-1} || leaf_c) with h_0 a fixed constant, so that h_c depends on
exactly the first c*K tokens.  A trailing partial chunk also gets a hash.

The paper leaves Hash and the initial constant open.  They are fixed here
(all arithmetic modulo 2**64):

  mix(x):  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9;
           x ^= x >> 27; x *= 0x94D049BB133111EB;
           x ^= x >> 31                          (the splitmix64 finaliser)
  GAMMA  = 0x9E3779B97F4A7C15
  leaf of a chunk with n tokens t_1..t_n (each an int32 read as unsigned 32 bit):
           a = mix(GAMMA ^ n);  a = mix(a ^ t_j) for j = 1..n;  leaf = a
  chain:   h_0 = 0x243F6A8885A308D3;  h_c = mix(mix(h_{c-1} + GAMMA) ^ leaf_c)

Written with Python integers, one step per line of the specification.
"""
from __future__ import annotations

MASK = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15
H0 = 0x243F6A8885A308D3


def mix(x: int) -> int:
    x &= MASK
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & MASK
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & MASK
    x ^= x >> 31
    return x


def leaf_hash(chunk) -> int:
    a = mix(GAMMA ^ len(chunk))
    for t in chunk:
        a = mix(a ^ (int(t) & 0xFFFFFFFF))
    return a


def chunk_hashes(tokens, K: int = 16):
    """Cumulative prefix hashes h_1..h_C of one token sequence, C = ceil(T/K)."""
    T = len(tokens)
    C = -(-T // K)
    leaves = [leaf_hash(tokens[c * K:min((c + 1) * K, T)]) for c in range(C)]   # independent per chunk
    H = []
    h = H0
    for c in range(C):                                                         # sequential chaining
        h = mix(mix((h + GAMMA) & MASK) ^ leaves[c])
        H.append(h)
    return H


# ---------------------------------------------------------------------------
# The sequential formulation (Appendix "Prefix Hash Computation", Algorithm 1):
# one incremental xxHash-64 state is fed the tokens one by one and its digest is
# taken at every chunk boundary and at the end.  The digest of a streaming state
# equals the one-shot hash of the bytes fed so far, so h_c = XXH64(first
# min(c*K, T) tokens) -- written here exactly so, one full hash per prefix.
# Tokens are fed as 4-byte little-endian integers (the paper does not say; this
# is what feeding an int32 array to a byte-oriented hash amounts to).
#
# XXH64 follows its published specification (five odd 64-bit primes, four lanes
# over 32-byte stripes, tail in 8/4/1-byte steps, avalanche); the tests pin it
# against the xxhash module byte for byte.

P1, P2, P3 = 0x9E3779B185EBCA87, 0xC2B2AE3D27D4EB4F, 0x165667B19E3779F9
P4, P5 = 0x85EBCA77C2B2AE63, 0x27D4EB2F165667C5


def _rotl(x: int, r: int) -> int:
    return ((x << r) | (x >> (64 - r))) & MASK


def _round(acc: int, lane: int) -> int:
    return (_rotl((acc + lane * P2) & MASK, 31) * P1) & MASK


def _merge(h: int, v: int) -> int:
    return ((h ^ _round(0, v)) * P1 + P4) & MASK


def xxh64(data: bytes, seed: int = 0) -> int:
    n = len(data)
    p = 0
    if n >= 32:
        v = [(seed + P1 + P2) & MASK, (seed + P2) & MASK, seed & MASK, (seed - P1) & MASK]
        while p + 32 <= n:
            for i in range(4):
                v[i] = _round(v[i], int.from_bytes(data[p + 8 * i:p + 8 * i + 8], "little"))
            p += 32
        h = (_rotl(v[0], 1) + _rotl(v[1], 7) + _rotl(v[2], 12) + _rotl(v[3], 18)) & MASK
        for i in range(4):
            h = _merge(h, v[i])
    else:
        h = (seed + P5) & MASK
    h = (h + n) & MASK
    while p + 8 <= n:
        h ^= _round(0, int.from_bytes(data[p:p + 8], "little"))
        h = (_rotl(h, 27) * P1 + P4) & MASK
        p += 8
    if p + 4 <= n:
        h ^= (int.from_bytes(data[p:p + 4], "little") * P1) & MASK
        h = (_rotl(h, 23) * P2 + P3) & MASK
        p += 4
    while p < n:
        h ^= (data[p] * P5) & MASK
        h = (_rotl(h, 11) * P1) & MASK
        p += 1
    h ^= h >> 33
    h = (h * P2) & MASK
    h ^= h >> 29
    h = (h * P3) & MASK
    h ^= h >> 32
    return h


def chunk_hashes_xxh64(tokens, K: int = 16, seed: int = 0):
    """Algorithm 1's hash vector: h_c = XXH64 of the first min(c*K, T) tokens."""
    T = len(tokens)
    raw = b"".join((int(t) & 0xFFFFFFFF).to_bytes(4, "little") for t in tokens)
    return [xxh64(raw[:4 * min(c * K, T)], seed) for c in range(1, -(-T // K) + 1)]
