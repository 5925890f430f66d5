"""Growing the KV history step by step: host bookkeeping on the CPU, the append kernel and a
short decode loop (extend -> append -> attention) on the GPU, against the oracle."""
import numpy as np
import pytest

import workloads as W
from oracle import append as oappend
from oracle.attention import decode_attention, gather_kv
from oracle.block_tables import build_block_tables, free_list


def start(spec, extra_cols=4):
    wl = W.generate(spec)
    seqs = [wl.request_tokens(i) for i in range(spec.batch)]
    width = wl.max_blocks_per_seq + extra_cols
    bt, lens, _ = build_block_tables(seqs, wl.num_blocks + 8 * spec.batch, wl.perm_seed, width)
    used = set(bt[bt >= 0].tolist())
    free = [b for b in free_list(wl.num_blocks + 8 * spec.batch, wl.perm_seed) if b not in used]
    return wl, seqs, bt, lens, free


def test_oracle_extend_agrees_with_tables_built_from_the_grown_sequences():
    spec = W.scaled(W.CONFIGS["c2"], batch_div=8, len_div=8)
    wl, seqs, bt, lens, free = start(spec)
    rng = np.random.default_rng(3)
    for step in range(40):
        oappend.extend(bt, lens, free)
        seqs = [np.concatenate([s, rng.integers(0, W.VOCAB, 1, dtype=np.int32)]) for s in seqs]
    # same sharing structure as tables built from scratch on the grown sequences: equal columns alias equally
    bt2, lens2, _ = build_block_tables(seqs, wl.num_blocks + 8 * spec.batch, wl.perm_seed, bt.shape[1])
    assert np.array_equal(lens, lens2)
    B = len(seqs)
    for i in range(B):
        for j in range(i):
            same = (bt[i] == bt[j]) & (bt[i] >= 0)
            same2 = (bt2[i] == bt2[j]) & (bt2[i] >= 0)
            assert np.array_equal(same, same2)
    assert ((bt >= 0) == (bt2 >= 0)).all()


def test_library_extend_follows_the_oracle_and_rolls_back():
    import paper_2605_06046_amd as fea
    spec = W.scaled(W.CONFIGS["c3"], batch_div=8, len_div=8)
    wl, seqs, bt, lens, free = start(spec)
    nb_total = wl.num_blocks + 8 * spec.batch
    pool = fea.fea_kv_alloc(nb_total, 16, wl.perm_seed)
    lbt, llens, _, _ = fea.fea_build_block_tables(pool, wl.tokens, wl.tok_offsets, bt.shape[1])
    assert np.array_equal(lbt, bt)
    for step in range(50):
        want = oappend.extend(bt, lens, free)
        got = fea.fea_kv_extend(pool, lbt, llens)
        assert got == want and np.array_equal(lbt, bt) and np.array_equal(llens, lens)
    _, free_now, _, rc = fea.fea_kv_stats(pool)
    assert free_now == len(free)
    assert rc.sum() == (bt >= 0).sum()
    # a pool too small for the step: nothing changes
    small = fea.fea_kv_alloc(int((bt >= 0).sum()), 16, 0)
    tiny_bt = np.full((2, 2), -1, dtype=np.int32); tiny_lens = np.zeros(2, dtype=np.int32)
    assert fea.fea_kv_extend(small, tiny_bt, tiny_lens) == 2
    full = fea.fea_kv_alloc(1, 16, 0)
    keep_bt, keep_lens = tiny_bt.copy(), np.array([16, 32], dtype=np.int32)
    before = (keep_bt.copy(), keep_lens.copy())
    with pytest.raises(fea.FeaError) as ei:
        fea.fea_kv_extend(full, keep_bt, keep_lens)      # column 2 does not exist
    assert ei.value.code == -3 and np.array_equal(keep_bt, before[0]) and np.array_equal(keep_lens, before[1])
    two = np.array([0, 0], dtype=np.int32)
    with pytest.raises(fea.FeaError) as ei:
        fea.fea_kv_extend(full, tiny_bt.copy(), two)     # two blocks needed, one free
    assert ei.value.code == -2 and (two == 0).all()
    # released rows give their appended blocks back
    for i in range(lbt.shape[0]):
        fea.fea_release(pool, lbt[i][lbt[i] >= 0])
    assert fea.fea_kv_stats(pool)[1] == nb_total


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["c1", "c2", "c5"])
def test_decode_loop_on_the_device(name):
    import torch
    import paper_2605_06046_amd as fea
    from gpu_harness import assert_close, to_device, values
    small = {"c1": None, "c2": dict(batch_div=8, len_div=8), "c5": dict(batch_div=16, len_div=4)}[name]
    spec = W.CONFIGS[name] if small is None else W.scaled(W.CONFIGS[name], **small)
    wl = W.generate(spec)
    steps = 36
    extra = 8 * spec.batch
    nb_total = wl.num_blocks + extra
    pool = fea.fea_kv_alloc(nb_total, 16, wl.perm_seed)
    width = wl.max_blocks_per_seq + 4
    bt, lens, _, _ = fea.fea_build_block_tables(pool, wl.tokens, wl.tok_offsets, width)
    # caches with room for the blocks to come; host copies are the oracle's
    def grow(c):
        out = np.zeros((nb_total,) + c.shape[1:], dtype=c.dtype)
        out[:c.shape[0]] = c
        return out
    hk, hv = grow(wl.k_cache), grow(wl.v_cache)
    W.poison_dead_slots(dataclass_replace(wl, k_cache=hk, v_cache=hv, num_blocks=nb_total), bt, lens)
    dk, dv = to_device(hk), to_device(hv)
    dtype = fea.FEA_DTYPE_BF16 if spec.dtype == "bf16" else fea.FEA_DTYPE_F32
    p = fea.AttnParams(spec.num_q_heads, spec.num_kv_heads, spec.head_dim, dtype)
    ws = torch.zeros(fea.fea_decode_workspace_bytes(p, spec.batch, width), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(11)
    shape_new = (spec.batch, spec.num_kv_heads, spec.head_dim)
    for step in range(steps):
        fea.fea_kv_extend(pool, bt, lens)
        kn = rng.standard_normal(shape_new, dtype=np.float32)
        vn = rng.standard_normal(shape_new, dtype=np.float32)
        qn = rng.standard_normal((spec.batch, spec.num_q_heads, spec.head_dim), dtype=np.float32)
        if spec.dtype == "bf16":
            kn, vn, qn = W.f32_to_bf16_bits(kn), W.f32_to_bf16_bits(vn), W.f32_to_bf16_bits(qn)
        oappend.append(hk, hv, kn, vn, bt, lens)
        dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
        fea.fea_kv_append(p, to_device(kn), to_device(vn), dk, dv, dbt, dl)
        if step % 7 == 6 or step == steps - 1:
            dq = to_device(qn)
            out = torch.empty_like(dq)
            fea.fea_decode_attention(p, dq, dk, dv, dbt, dl, out, ws)
            torch.cuda.synchronize()
            want = decode_attention(values(qn), values(hk), values(hv), bt, lens)
            got = out.float().cpu().numpy().astype(np.float64)
            assert_close(got, want, spec.dtype, what=f"{name} step {step}")
    torch.cuda.synchronize()
    back_k = dk.cpu().view(torch.int16).numpy().view(hk.dtype) if spec.dtype == "bf16" else dk.cpu().numpy()
    back_v = dv.cpu().view(torch.int16).numpy().view(hv.dtype) if spec.dtype == "bf16" else dv.cpu().numpy()
    live = np.zeros(nb_total, dtype=bool); live[bt[bt >= 0]] = True
    # every live slot holds exactly what the oracle wrote (bit for bit); NaN poison compares as bytes
    assert np.array_equal(back_k.view(np.uint8)[live], hk.view(np.uint8)[live])
    assert np.array_equal(back_v.view(np.uint8)[live], hv.view(np.uint8)[live])


def dataclass_replace(obj, **kw):
    import dataclasses
    return dataclasses.replace(obj, **kw)
