"""Chunked cumulative prefix hashes (test infrastructure only).

Follows the chunk-parallel formulation of the paper's prefix hash computation
(Appendix "Prefix Hash Computation", Algorithm 2): every chunk of K tokens is
hashed on its own into a leaf value, and the leaves are chained, h_c =
Hash(h_{c-1} || leaf_c) with h_0 a fixed constant, so that h_c depends on
exactly the first c*K tokens.  A trailing partial chunk also gets a hash.

The paper leaves Hash and the initial constant open.  This build fixes them
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
