"""Pins for the block-table and chunk-hash oracles (no GPU)."""
import json
import os

import numpy as np
import pytest

import workloads as W
from oracle.block_tables import build_block_tables, free_list
from oracle.hashing import chunk_hashes

GOLD = os.path.join(os.path.dirname(__file__), "golden")
FACTS = json.load(open(os.path.join(GOLD, "paper_facts.json")))


# ---------------------------------------------------------------- hashes
def test_paper_example_three_cumulative_hashes():
    ex = FACTS["hash_vector_example"]
    H = chunk_hashes(ex["tokens"], ex["K"])
    assert len(H) == ex["num_hashes"]
    # hash c is cumulative over the first covers_tokens[c] tokens and nothing after them
    for c, n in enumerate(ex["covers_tokens"]):
        assert chunk_hashes(ex["tokens"][:n], ex["K"])[c] == H[c]
        other_tail = ex["tokens"][:n] + [999] * (len(ex["tokens"]) - n)
        assert chunk_hashes(other_tail, ex["K"])[c] == H[c]
        if n > 0:
            changed = list(ex["tokens"])
            changed[n - 1] += 1
            assert chunk_hashes(changed, ex["K"])[c] != H[c]


@pytest.mark.parametrize("T,K,C", FACTS["hash_count"]["cases"])
def test_hash_count_is_ceil_T_over_K(T, K, C):
    assert len(chunk_hashes(list(range(T)), K)) == C


def _second_implementation(tokens, K=16):
    """The written hash specification again, vectorised over chunks with numpy
    uint64 arithmetic (independent of the oracle's Python-integer version)."""
    def mix(x):
        x = x ^ (x >> np.uint64(30))
        x = x * np.uint64(0xBF58476D1CE4E5B9)
        x = x ^ (x >> np.uint64(27))
        x = x * np.uint64(0x94D049BB133111EB)
        return x ^ (x >> np.uint64(31))
    gamma = np.uint64(0x9E3779B97F4A7C15)
    t = np.asarray(tokens, dtype=np.int32).view(np.uint32).astype(np.uint64)
    T = len(t)
    C = -(-T // K)
    pad = np.zeros(C * K, dtype=np.uint64)
    pad[:T] = t
    pad = pad.reshape(C, K)
    n = np.minimum(K, T - K * np.arange(C)).astype(np.uint64)
    with np.errstate(over="ignore"):
        a = mix(gamma ^ n)
        for j in range(K):
            a = np.where(j < n, mix(a ^ pad[:, j]), a)
        out = []
        h = np.uint64(0x243F6A8885A308D3)
        for c in range(C):
            h = mix(mix(h + gamma) ^ a[c])
            out.append(int(h))
    return out


@pytest.mark.parametrize("T", [1, 15, 16, 17, 48, 333])
def test_two_independent_implementations_agree(T):
    rng = np.random.default_rng(T)
    toks = rng.integers(-5, 32000, size=T, dtype=np.int32)
    assert chunk_hashes(toks) == _second_implementation(toks)


def test_prefix_consistency_both_directions():
    """h_c equal iff the first c*K tokens are equal, on random and adversarial streams."""
    rng = np.random.default_rng(42)
    base = rng.integers(0, 32000, size=96, dtype=np.int32)
    variants = [base.copy() for _ in range(8)]
    variants[1][15] += 1                      # last token of chunk 0
    variants[2][16] += 1                      # first token of chunk 1
    variants[3][[20, 21]] = variants[3][[21, 20]]     # swapped neighbours inside chunk 1
    v4 = variants[4].copy()
    variants[4][16:32], variants[4][32:48] = v4[32:48].copy(), v4[16:32].copy()   # swapped chunks 1, 2
    variants[5][95] += 1                      # very last token
    variants[6] = base[:40].copy()            # shorter: two full chunks + partial
    variants[7] = np.concatenate([base[:32], rng.integers(0, 32000, size=64, dtype=np.int32)])
    for _ in range(6):
        variants.append(rng.integers(0, 3, size=int(rng.integers(1, 70)), dtype=np.int32))  # tiny alphabet
    H = [chunk_hashes(v) for v in variants]
    for a in range(len(variants)):
        for b in range(a + 1, len(variants)):
            for c in range(min(len(variants[a]), len(variants[b])) // 16):
                same_prefix = np.array_equal(variants[a][:16 * (c + 1)], variants[b][:16 * (c + 1)])
                assert (H[a][c] == H[b][c]) == same_prefix, (a, b, c)


def test_partial_chunk_hash_differs_from_padded_full_chunk():
    toks = list(range(20))
    padded = toks + [0] * 12
    assert chunk_hashes(toks)[1] != chunk_hashes(padded)[1]
    assert chunk_hashes(toks)[0] == chunk_hashes(padded)[0]


def test_hash_golden_file_regression():
    gold = json.load(open(os.path.join(GOLD, "hash_vectors.json")))
    for name, case in gold.items():
        got = [f"0x{h:016x}" for h in chunk_hashes(case["tokens"], case["K"])]
        assert got == case["hashes"], name


def test_hashes_are_well_spread_no_collisions_at_workload_scale():
    wl = W.generate(W.CONFIGS["c2"], with_kv=False)
    seen = {}
    for i in range(wl.spec.batch):
        toks = wl.request_tokens(i)
        for c, h in enumerate(chunk_hashes(toks)):
            key = toks[:16 * (c + 1)].tobytes()
            assert seen.setdefault((c, h), key) == key


# ---------------------------------------------------------------- free list
@pytest.mark.parametrize("n,seed", [(1, 5), (2, 5), (97, 1), (4608, 0xFEA7FEA7)])
def test_free_list_is_a_permutation(n, seed):
    fl = free_list(n, seed)
    assert sorted(fl) == list(range(n))
    assert free_list(n, 0) == list(range(n))
    if n > 50:
        assert fl != list(range(n))
        assert fl != free_list(n, seed + 1)


# ---------------------------------------------------------------- tables
def _small_batch(seed, n=9):
    rng = np.random.default_rng(seed)
    stems = [rng.integers(0, 50, size=int(rng.integers(0, 70)), dtype=np.int32) for _ in range(3)]
    seqs = []
    for _ in range(n):
        stem = stems[int(rng.integers(0, 3))]
        cut = int(rng.integers(0, len(stem) + 1))
        tail = rng.integers(0, 50, size=int(rng.integers(1, 40)), dtype=np.int32)
        seqs.append(np.concatenate([stem[:cut], tail]))
    seqs.append(seqs[0].copy())          # an exact duplicate request
    return seqs


@pytest.mark.parametrize("seed", range(6))
def test_aliasing_iff_equal_full_prefix_all_pairs(seed):
    seqs = _small_batch(seed)
    bt, lens, rc = build_block_tables(seqs, 400)
    for i in range(len(seqs)):
        nb_i = -(-len(seqs[i]) // 16)
        assert (bt[i, :nb_i] >= 0).all() and (bt[i, nb_i:] == -1).all()
        assert len(set(bt[i, :nb_i].tolist())) == nb_i           # no id twice in one row
        for j in range(i + 1, len(seqs)):
            nb_j = -(-len(seqs[j]) // 16)
            for ci in range(nb_i):
                for cj in range(nb_j):
                    full = (ci + 1) * 16 <= len(seqs[i]) and (cj + 1) * 16 <= len(seqs[j])
                    same = (ci == cj and full and
                            np.array_equal(seqs[i][:16 * (ci + 1)], seqs[j][:16 * (ci + 1)]))
                    assert (bt[i, ci] == bt[j, cj]) == same, (i, j, ci, cj)
    assert rc.sum() == sum(-(-len(s) // 16) for s in seqs)
    assert (np.bincount(bt[bt >= 0], minlength=400) == rc).all()


@pytest.mark.parametrize("seed", range(3))
def test_ids_are_handed_out_in_free_list_order_and_permutation_commutes(seed):
    seqs = _small_batch(seed)
    bt0, _, _ = build_block_tables(seqs, 300, perm_seed=0)
    first_use = list(dict.fromkeys(bt0[bt0 >= 0].tolist()))     # row-major first occurrences
    assert first_use == list(range(len(first_use)))
    pseed = 1234 + seed
    fl = np.array(free_list(300, pseed))
    btp, _, _ = build_block_tables(seqs, 300, perm_seed=pseed)
    assert np.array_equal(btp, np.where(bt0 >= 0, fl[np.clip(bt0, 0, None)], -1))


def test_pool_exhaustion_and_width_errors():
    seqs = [np.arange(40, dtype=np.int32)]
    with pytest.raises(MemoryError):
        build_block_tables(seqs, 2)
    with pytest.raises(ValueError):
        build_block_tables(seqs, 10, max_blocks_per_seq=2)
    bt, _, _ = build_block_tables(seqs, 3, max_blocks_per_seq=5)
    assert bt.tolist() == [[0, 1, 2, -1, -1]]


def _tables_for(name):
    wl = W.generate(W.CONFIGS[name], with_kv=False)
    seqs = [wl.request_tokens(i) for i in range(wl.spec.batch)]
    bt, lens, rc = build_block_tables(seqs, wl.num_blocks, wl.perm_seed)
    return wl, bt, lens, rc


def test_structure_c1_sixteen_shared_columns_four_private():
    wl, bt, lens, rc = _tables_for("c1")
    assert (bt[:, :16] == bt[0, :16]).all()
    assert len(set(bt[:, 16:].ravel().tolist())) == 16
    assert len(set(bt.ravel().tolist())) == 32 and (lens == 320).all()
    assert (rc[bt[0, :16]] == 4).all()


def test_structure_c2_one_group_256_shared_columns():
    wl, bt, lens, rc = _tables_for("c2")
    assert (bt[:, :256] == bt[0, :256]).all()
    priv = bt[:, 256:]
    ids = priv[priv >= 0]
    assert len(set(ids.tolist())) == len(ids)                   # all suffix blocks distinct
    assert (rc > 0).sum() == 256 + len(ids) == wl.num_blocks
    assert rc.sum() == sum(-(-int(L) // 16) for L in lens)


def test_structure_c3_eight_disjoint_groups_interleaved():
    wl, bt, lens, rc = _tables_for("c3")
    assert wl.group_of[:16].tolist() == list(range(8)) * 2      # arrival order cycles the groups
    heads = {}
    for i in range(256):
        heads.setdefault(int(wl.group_of[i]), set()).add(tuple(bt[i, :256].tolist()))
    assert all(len(v) == 1 for v in heads.values()) and len(heads) == 8
    runs = [set(next(iter(v))) for v in heads.values()]
    for a in range(8):
        for b in range(a + 1, 8):
            assert not (runs[a] & runs[b])
    assert (rc > 0).sum() == wl.num_blocks


def test_structure_c4_permuted_pool_one_and_a_half_times_live():
    wl, bt, lens, rc = _tables_for("c4")
    assert wl.num_blocks == 4608 and (rc > 0).sum() == 3072
    assert (bt[:, :2048] == bt[0, :2048]).all() and (lens == 32768 + 512).all()
    assert bt[0, :8].tolist() != list(range(8))                 # placement is scattered
    fl = free_list(4608, wl.perm_seed)
    assert bt[0, :2048].tolist() == fl[:2048]


def test_structure_c5_no_aliasing_at_all():
    wl, bt, lens, rc = _tables_for("c5")
    ids = bt[bt >= 0]
    assert len(set(ids.tolist())) == len(ids) == wl.num_blocks
    assert rc.max() == 1 and lens.min() >= 512 and lens.max() <= 4096


# ---------------------------------------------------------------- bytes per token
def test_kv_bytes_per_token_matches_paper_footprint():
    f = FACTS["kv_footprint"]
    per_token_layer = 2 * f["kv_heads"] * f["head_dim"] * f["bytes_per_element"]
    assert per_token_layer == 4096
    total = per_token_layer * f["layers"] * f["tokens"]
    assert abs(total / 2 ** 30 - f["reported_gb"]) < 0.05       # 1.31e9 B = 1.22 GiB
    assert f["block_tokens"] == W.BLOCK
