"""Pins for the float64 attention oracle (no GPU).

Each test checks the oracle against something other than itself: scalar brute
force written independently here, closed forms of softmax attention, a dense
library attention on a contiguous table, and invariants that any correct
paged-attention result must satisfy.
"""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle.attention import decode_attention


def _rand_case(seed, B, Hq, Hkv, d, lens, block=16, extra_blocks=3, shared_first=0):
    """Random caches and a table whose rows use distinct blocks, except that the
    first `shared_first` columns of every row alias the same physical blocks."""
    rng = np.random.default_rng(seed)
    nbs = [-(-L // block) for L in lens]
    total = sum(nbs) + extra_blocks
    ids = rng.permutation(total)
    width = max(nbs + [1])
    bt = np.full((B, width), -1, dtype=np.int32)
    p = 0
    for i, nb in enumerate(nbs):
        bt[i, :nb] = ids[p:p + nb]
        p += nb
    for i in range(1, B):
        s = min(shared_first, lens[i] // block, lens[0] // block)
        bt[i, :s] = bt[0, :s]
    k = rng.standard_normal((total, Hkv, block, d))
    v = rng.standard_normal((total, Hkv, block, d))
    q = rng.standard_normal((B, Hq, d))
    return q, k, v, bt, np.array(lens, dtype=np.int32)


def _brute_force(q, k, v, bt, lens, scale):
    """Scalar loops straight from softmax(q k / sqrt(d)) v; own indexing."""
    B, Hq, d = q.shape
    Hkv, block = k.shape[1], k.shape[2]
    G = Hq // Hkv
    out = [[[0.0] * d for _ in range(Hq)] for _ in range(B)]
    for i in range(B):
        for h in range(Hq):
            g = h // G
            scores = []
            for t in range(int(lens[i])):
                blk = int(bt[i][t // block])
                slot = t % block
                acc = 0.0
                for e in range(d):
                    acc += float(q[i, h, e]) * float(k[blk, g, slot, e])
                scores.append(acc * scale)
            if not scores:
                continue
            mx = max(scores)
            w = [math.exp(s - mx) for s in scores]
            z = sum(w)
            for t in range(int(lens[i])):
                blk = int(bt[i][t // block])
                slot = t % block
                for e in range(d):
                    out[i][h][e] += (w[t] / z) * float(v[blk, g, slot, e])
    return np.array(out)


@pytest.mark.parametrize("seed,B,Hq,Hkv,d,lens,shared", [
    (1, 3, 4, 2, 8, [40, 17, 1], 1),
    (2, 2, 6, 3, 4, [16, 33], 0),
    (3, 3, 2, 2, 5, [5, 0, 31], 0),
    (4, 2, 8, 1, 3, [32, 39], 2),
])
def test_brute_force_tiny(seed, B, Hq, Hkv, d, lens, shared):
    q, k, v, bt, L = _rand_case(seed, B, Hq, Hkv, d, lens, shared_first=shared)
    got = decode_attention(q, k, v, bt, L)
    want = _brute_force(q, k, v, bt, L, 1.0 / math.sqrt(d))
    assert np.abs(got - want).max() < 1e-12


def test_custom_scale_brute_force():
    q, k, v, bt, L = _rand_case(11, 2, 4, 2, 6, [21, 9])
    got = decode_attention(q, k, v, bt, L, scale=0.37)
    want = _brute_force(q, k, v, bt, L, 0.37)
    assert np.abs(got - want).max() < 1e-12


def test_single_token_returns_its_value():
    q, k, v, bt, L = _rand_case(5, 2, 4, 2, 8, [1, 1])
    out = decode_attention(q, k, v, bt, L)
    for i in range(2):
        for h in range(4):
            assert np.allclose(out[i, h], v[bt[i, 0], h // 2, 0], atol=1e-15)


def test_equal_keys_give_mean_of_values():
    q, k, v, bt, L = _rand_case(6, 2, 4, 2, 8, [37, 20])
    k[:] = k[0, 0, 0]            # every key identical -> uniform softmax
    out = decode_attention(q, k, v, bt, L)
    for i in range(2):
        nb = -(-L[i] // 16)
        for h in range(4):
            rows = v[bt[i, :nb], h // 2].reshape(-1, 8)[:L[i]]
            assert np.allclose(out[i, h], rows.mean(axis=0), atol=1e-13)


def test_constant_values_are_reproduced():
    q, k, v, bt, L = _rand_case(7, 2, 4, 2, 8, [50, 3])
    c = np.linspace(-1, 1, 8)
    v[:] = c
    out = decode_attention(q, k, v, bt, L)
    assert np.allclose(out, c, atol=1e-13)


def test_dominating_key_selects_its_value():
    q, k, v, bt, L = _rand_case(8, 1, 2, 1, 8, [45])
    t_star = 29
    blk, slot = bt[0, t_star // 16], t_star % 16
    out = decode_attention(q, k, v, bt, L)
    for h in range(2):
        k2 = k.copy()
        k2[blk, 0, slot] = q[0, h] * 200.0     # score ~ 200 |q|^2 / sqrt(d): dwarfs the rest
        out2 = decode_attention(q, k2, v, bt, L)
        assert np.allclose(out2[0, h], v[blk, 0, slot], atol=1e-9)
    assert not np.allclose(out[0, 0], v[blk, 0, slot], atol=1e-3)


def test_dense_library_attention_on_contiguous_table():
    """Identity table + equal lengths reduces to dense attention (third opinion)."""
    rng = np.random.default_rng(9)
    B, Hq, Hkv, d, L = 3, 8, 2, 16, 64
    nb = L // 16
    k = rng.standard_normal((B * nb, Hkv, 16, d))
    v = rng.standard_normal((B * nb, Hkv, 16, d))
    q = rng.standard_normal((B, Hq, d))
    bt = np.arange(B * nb, dtype=np.int32).reshape(B, nb)
    out = decode_attention(q, k, v, bt, np.full(B, L, dtype=np.int32))
    # dense [B, Hq, 1, d] x [B, Hq, L, d], kv heads repeated for the query groups
    kd = torch.from_numpy(k).reshape(B, nb, Hkv, 16, d).permute(0, 2, 1, 3, 4).reshape(B, Hkv, L, d)
    vd = torch.from_numpy(v).reshape(B, nb, Hkv, 16, d).permute(0, 2, 1, 3, 4).reshape(B, Hkv, L, d)
    kd = kd.repeat_interleave(Hq // Hkv, dim=1)
    vd = vd.repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, :, None, :], kd, vd)
    assert np.abs(out - ref[:, :, 0, :].numpy()).max() < 1e-12


def test_identical_histories_give_identical_rows():
    q, k, v, bt, L = _rand_case(10, 3, 4, 2, 8, [40, 40, 23])
    bt[1] = bt[0]                 # same physical history
    q[1] = q[0]
    out = decode_attention(q, k, v, bt, L)
    assert np.array_equal(out[0], out[1])
    # same history stored twice in different blocks
    nb = 3
    k[bt[2, :2]] = k[bt[0, :2]]
    v[bt[2, :2]] = v[bt[0, :2]]
    k[bt[2, 2]] = 0
    v[bt[2, 2]] = 0
    L2 = np.array([32, 32, 32], dtype=np.int32)
    q[2] = q[0]
    out = decode_attention(q, k, v, bt, L2)
    assert np.array_equal(out[0], out[2])


def test_physical_placement_does_not_matter():
    q, k, v, bt, L = _rand_case(12, 3, 4, 2, 8, [40, 17, 33], shared_first=1)
    out = decode_attention(q, k, v, bt, L)
    rng = np.random.default_rng(0)
    perm = rng.permutation(k.shape[0])          # block b moves to perm[b]
    k2 = np.empty_like(k)
    v2 = np.empty_like(v)
    k2[perm] = k
    v2[perm] = v
    bt2 = np.where(bt >= 0, perm[np.clip(bt, 0, None)], -1).astype(np.int32)
    out2 = decode_attention(q, k2, v2, bt2, L)
    assert np.array_equal(out, out2)


def test_columns_past_length_are_ignored():
    q, k, v, bt, L = _rand_case(13, 2, 4, 2, 8, [20, 35])
    out = decode_attention(q, k, v, bt, L)
    bt2 = bt.copy()
    bt2[0, 2:] = 0                # garbage in ignored columns
    k2 = k.copy()
    k2[bt[0, 1], :, 4:] = np.nan  # slots past seq_len in the last block
    out2 = decode_attention(q, k2, v, bt2, L)
    assert np.array_equal(out[0], out2[0])


def test_split_and_merge_identity():
    """Attention over a sequence equals the log-sum-exp merge of its two halves."""
    q, k, v, bt, L = _rand_case(14, 1, 2, 1, 8, [48])
    d = 8
    full = decode_attention(q, k, v, bt, L)
    # first 32 tokens via the oracle, last 16 via a one-block table
    a = decode_attention(q, k, v, bt[:, :2], np.array([32], dtype=np.int32))
    b = decode_attention(q, k, v, bt[:, 2:3], np.array([16], dtype=np.int32))
    for h in range(2):
        ka = k[bt[0, :2], 0].reshape(-1, d)
        kb = k[bt[0, 2], 0]
        lse_a = np.log(np.exp(ka @ q[0, h] / math.sqrt(d)).sum())
        lse_b = np.log(np.exp(kb @ q[0, h] / math.sqrt(d)).sum())
        wa = 1.0 / (1.0 + math.exp(lse_b - lse_a))
        merged = wa * a[0, h] + (1 - wa) * b[0, h]
        assert np.abs(merged - full[0, h]).max() < 1e-12


def test_zero_length_row_is_zero_and_subset_selection():
    q, k, v, bt, L = _rand_case(15, 3, 4, 2, 8, [0, 18, 7])
    out = decode_attention(q, k, v, bt, L)
    assert np.array_equal(out[0], np.zeros((4, 8)))
    part = decode_attention(q, k, v, bt, L, requests=[2])
    assert np.array_equal(part[2], out[2]) and np.isnan(part[1]).all()


def test_oracle_on_generated_workload_with_poison():
    """c1 drawn by the shared generator: dead slots poisoned, output finite."""
    from oracle.block_tables import build_block_tables
    wl = W.generate(W.CONFIGS["c1"])
    seqs = [wl.request_tokens(i) for i in range(wl.spec.batch)]
    bt, lens, _ = build_block_tables(seqs, wl.num_blocks)
    clean = decode_attention(wl.q, wl.k_cache, wl.v_cache, bt, lens)
    W.poison_dead_slots(wl, bt, lens)
    out = decode_attention(wl.q, wl.k_cache, wl.v_cache, bt, lens)
    assert np.isfinite(out).all() and np.array_equal(out, clean)


def test_bf16_bit_helpers_match_torch_rounding():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(4096).astype(np.float32)
    x[:4] = [1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -(1.0 + 2 ** -8), 0.0]     # exact ties
    bits = W.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), t.view(torch.int16).numpy())
    assert np.array_equal(W.bf16_bits_to_f32(bits), t.float().numpy())
