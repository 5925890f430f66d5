"""The sequential prefix-hash formulation (Algorithm 1): the oracle's XXH64 against the xxhash module.

The module is a third party's implementation of the same published hash: one-shot digests for every
length around the stripe and tail boundaries, several seeds, and the streaming use Algorithm 1 makes
of it (feed token by token, digest at every chunk boundary and at the end).
"""
import random
import struct

import numpy as np
import pytest

from oracle.hashing import chunk_hashes_xxh64, xxh64

xxhash = pytest.importorskip("xxhash")


def test_known_digests_of_the_module():
    assert xxh64(b"") == 0xEF46DB3751D8E999
    assert xxh64(b"abc") == 0x44BC2CF5AD770999


@pytest.mark.parametrize("seed", [0, 1, 0x9E3779B97F4A7C15, (1 << 64) - 1])
def test_one_shot_matches_for_every_length(seed):
    rng = random.Random(seed & 0xFFFF)
    for n in list(range(0, 140)) + [255, 256, 257, 1000, 4099]:
        data = bytes(rng.getrandbits(8) for _ in range(n))
        assert xxh64(data, seed) == xxhash.xxh64(data, seed=seed).intdigest(), n


@pytest.mark.parametrize("T,K", [(0, 16), (1, 16), (15, 16), (16, 16), (17, 16), (100, 16), (333, 16), (64, 4), (37, 5)])
def test_algorithm_1_streaming(T, K):
    rng = np.random.default_rng(T * 131 + K)
    tokens = rng.integers(-2 ** 31, 2 ** 31, size=T, dtype=np.int64).astype(np.int32)
    state = xxhash.xxh64(seed=7)
    want = []
    for i, t in enumerate(tokens, start=1):
        state.update(struct.pack("<i", int(t)))
        if i % K == 0 or i == T:
            want.append(state.intdigest())
    assert chunk_hashes_xxh64(tokens, K, seed=7) == want
    assert len(want) == -(-T // K)


def test_prefix_consistency():
    rng = np.random.default_rng(2)
    a = rng.integers(0, 50000, size=100, dtype=np.int32)
    b = a.copy()
    b[70] += 1                                   # differs inside chunk 5 (tokens 64..79)
    ha, hb = chunk_hashes_xxh64(a), chunk_hashes_xxh64(b)
    assert ha[:4] == hb[:4] and all(x != y for x, y in zip(ha[4:], hb[4:]))
