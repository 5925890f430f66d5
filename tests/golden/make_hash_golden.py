"""Writes tests/golden/hash_vectors.json from the oracle alone.

Run from the repository root:  python tests/golden/make_hash_golden.py
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle.hashing import chunk_hashes  # noqa: E402

CASES = {
    "a_to_f_K2": ([65, 66, 67, 68, 69, 70], 2),
    "single_token": ([7], 16),
    "one_full_chunk": (list(range(16)), 16),
    "full_plus_one": (list(range(17)), 16),
    "negative_token_ids": ([-1, -2, 3], 16),
    "forty_tokens": ([(i * 7919) % 32000 for i in range(40)], 16),
}

if __name__ == "__main__":
    out = {name: {"tokens": toks, "K": K, "hashes": [f"0x{h:016x}" for h in chunk_hashes(toks, K)]}
           for name, (toks, K) in CASES.items()}
    with open(os.path.join(HERE, "hash_vectors.json"), "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
