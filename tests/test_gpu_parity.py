"""GPU parity: the HIP path (through the C ABI) against the float64 oracle."""
import dataclasses

import numpy as np
import pytest

import workloads as W
from oracle.block_tables import build_block_tables
from gpu_harness import assert_close, library_tables, oracle_for, run_hip, run_workload, values
from oracle.attention import decode_attention

pytestmark = pytest.mark.gpu


def _check_tables(wl, bt, lens):
    seqs = [wl.request_tokens(i) for i in range(wl.spec.batch)]
    obt, olens, _ = build_block_tables(seqs, wl.num_blocks, wl.perm_seed, wl.max_blocks_per_seq)
    assert np.array_equal(bt, obt) and np.array_equal(lens, olens)


def test_c1_fp32_full():
    wl = W.generate(W.CONFIGS["c1"])
    out, bt, lens, info = run_workload(wl)
    _check_tables(wl, bt, lens)
    print("c1", info, assert_close(out, oracle_for(wl, bt, lens), "f32", what="c1"))
    assert info["groups"] == 1 and info["grouped_requests"] == 4 and info["shared_blocks"] == 16


SMALL = {
    "c2": dict(batch_div=8, len_div=8),      # 8 requests, 512-token prefix, suffix 16..128
    "c3": dict(batch_div=8, len_div=8),      # 8 groups x 4
    "c4": dict(batch_div=4, len_div=16),     # 8 requests, 2048-token prefix, permuted pool
    "c5": dict(batch_div=16, len_div=4),     # 32 independent requests, 128..1024 tokens
}


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_scaled_configs_elementwise(name):
    wl = W.generate(W.scaled(W.CONFIGS[name], **SMALL[name]))
    out, bt, lens, info = run_workload(wl)
    _check_tables(wl, bt, lens)
    assert (lens % 16 != 0).any()                      # ragged tails present
    print(name, info, assert_close(out, oracle_for(wl, bt, lens), "bf16", what=name))
    if name != "c5":
        assert info["groups"] >= 1
    else:
        assert info["groups"] == 0


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_peaked_softmax_variant(name):
    """q scaled x8: the softmax concentrates and outputs are O(1)."""
    spec = dataclasses.replace(W.scaled(W.CONFIGS[name], **SMALL[name]), q_gain=8.0)
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    want = oracle_for(wl, bt, lens)
    assert np.abs(want).max() > 0.5
    assert_close(out, want, "bf16", what=name + " peaked")


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_full_size_configs_every_row(name):
    """The full-size batches in the launch configuration the benchmark times: every output row of
    every request against the oracle (tables bit-exact first)."""
    wl = W.generate(W.CONFIGS[name])
    out, bt, lens, info = run_workload(wl)
    _check_tables(wl, bt, lens)
    assert info["overflow"] == 0 and info["variant"] == 1
    want = oracle_for(wl, bt, lens)
    print(name, info, assert_close(out, want, "bf16", what=name + " full size, all rows"))
    # row by row as well: no single request may hide behind the batch-wide relative error
    err = np.abs(out - want).reshape(wl.spec.batch, -1).max(axis=1)
    rl2 = (np.linalg.norm((out - want).reshape(wl.spec.batch, -1), axis=1)
           / np.maximum(np.linalg.norm(want.reshape(wl.spec.batch, -1), axis=1), 1e-30))
    assert err.max() <= 2e-2 and rl2.max() <= 6e-3, (int(err.argmax()), float(err.max()), int(rl2.argmax()), float(rl2.max()))


def _random_tables(seed, B, Hkv, d, dtype, lens, num_blocks, mode):
    rng = np.random.default_rng(seed)
    width = max(1, max(-(-L // 16) for L in lens) + 2)
    bt = np.full((B, width), -1, dtype=np.int32)
    for i, L in enumerate(lens):
        nb = -(-L // 16)
        if mode == "random":                         # ids drawn with replacement: repeats inside rows and across
            bt[i, :nb] = rng.integers(0, num_blocks, size=nb)
        elif mode == "same_first_then_random":       # equal first block, then unrelated
            bt[i, :nb] = rng.integers(0, num_blocks, size=nb)
            if nb:
                bt[i, 0] = 3
        elif mode == "nested":                       # runs of different depth shared with row 0
            base = (np.arange(nb) * 7 + 1) % num_blocks
            bt[i, :nb] = base
            cut = int(rng.integers(0, nb + 1))
            bt[i, cut:nb] = rng.integers(0, num_blocks, size=nb - cut)
        elif mode == "all_same_block":
            bt[i, :nb] = 5
        elif mode == "identical_rows":
            bt[i, :nb] = (np.arange(nb) * 3 + 2) % num_blocks
    k = rng.standard_normal((num_blocks, Hkv, 16, d), dtype=np.float32)
    v = rng.standard_normal((num_blocks, Hkv, 16, d), dtype=np.float32)
    if dtype == "bf16":
        k, v = W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)
    return bt, k, v


@pytest.mark.parametrize("mode", ["random", "same_first_then_random", "nested", "all_same_block", "identical_rows"])
@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 8, 2, 64), ("bf16", 32, 8, 128), ("bf16", 16, 2, 128), ("bf16", 16, 4, 64), ("bf16", 8, 2, 256)])
@pytest.mark.parametrize("lens", [[0, 1, 15, 16, 17, 160, 161, 500, 512, 33, 160, 160, 700, 2, 48, 31],
                                  [0, 160, 161, 500, 512, 100, 160, 160, 700, 48, 64, 49, 1000]])
def test_any_block_table_is_handled(mode, dtype, Hq, Hkv, d, lens):
    B = len(lens)
    seed = {"random": 101, "same_first_then_random": 202, "nested": 303, "all_same_block": 404, "identical_rows": 505}[mode]
    bt, k, v = _random_tables(seed, B, Hkv, d, dtype, lens, 40, mode)
    rng = np.random.default_rng(5)
    q = rng.standard_normal((B, Hq, d), dtype=np.float32)
    if dtype == "bf16":
        q = W.f32_to_bf16_bits(q)
    L = np.array(lens, dtype=np.int32)
    out, info = run_hip(q, k, v, bt, L, Hq, Hkv, d, dtype)
    want = decode_attention(values(q), values(k), values(v), bt, L)
    assert_close(out, want, dtype, what=mode)
    assert (out[0] == 0).all()                        # zero-length request


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 4, 4, 32), ("f32", 6, 2, 128), ("f32", 2, 1, 256),
                                            ("bf16", 12, 4, 64), ("bf16", 8, 8, 256), ("bf16", 24, 8, 128),
                                            ("bf16", 64, 8, 128), ("bf16", 8, 8, 128), ("bf16", 32, 2, 128),
                                            ("bf16", 28, 4, 128), ("bf16", 40, 8, 128), ("bf16", 12, 1, 128),
                                            ("bf16", 6, 1, 128), ("bf16", 34, 2, 128)])
def test_other_shapes(dtype, Hq, Hkv, d):
    spec = W.Spec("shape", 11, dtype, Hq, Hkv, d, ((5, 96), (3, 0)), (1, 200))
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert_close(out, oracle_for(wl, bt, lens), dtype, what=f"{dtype} {Hq}/{Hkv}/{d}")


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 8, 4, 64), ("f32", 6, 2, 128), ("bf16", 130, 2, 64), ("f32", 4, 2, 256),
                                            ("f32", 4, 4, 32)])
def test_vector_sweep_on_batches_that_fill_the_chip(dtype, Hq, Hkv, d):
    """The vector sweep has two instantiations: wide passes (up to 16 stacked query rows) for batches too small to
    fill the chip - every other small case here - and passes of 4 rows for the rest.  These batches are big enough
    for the second: two prefix groups (one of them wider than a row tile) and requests on their own."""
    B = 2048 // Hkv // 8 + 40
    spec = W.Spec("vec_big", 12, dtype, Hq, Hkv, d, ((B // 2, 256), (B // 4, 96), (B - B // 2 - B // 4, 0)), (150, 800))
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert B * Hkv * (1 + bt.shape[1] // 8) > 2048 and info["variant"] == 0 and info["groups"] == 2
    assert_close(out, oracle_for(wl, bt, lens), dtype, what=f"vector sweep {dtype} {Hq}/{Hkv}/{d}")


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_grouping_off_split_sizes_scale_and_determinism(name):
    spec = W.CONFIGS[name] if name == "c1" else W.scaled(W.CONFIGS[name], **SMALL[name])
    wl = W.generate(spec)
    bt, lens = library_tables(wl)
    W.poison_dead_slots(wl, bt, lens)
    s = wl.spec
    args = (wl.q, wl.k_cache, wl.v_cache, bt, lens, s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
    want = oracle_for(wl, bt, lens)
    base, info = run_hip(*args)
    again, _ = run_hip(*args)
    assert np.array_equal(base, again)                        # run-to-run bitwise identical
    off, info_off = run_hip(*args, max_group=1)
    assert info_off["groups"] == 0 and info["groups"] >= 1
    assert_close(off, want, s.dtype, what="grouping off")
    for sb in (1, 2, 6, 64):
        o, i2 = run_hip(*args, split_blocks=sb)
        assert i2["split_blocks"] == (sb + 1) // 2 * 2
        assert_close(o, want, s.dtype, what=f"split {sb}")
    scaled_out, _ = run_hip(*args, scale=0.05)
    want_s = decode_attention(values(wl.q), values(wl.k_cache), values(wl.v_cache), bt, lens, scale=0.05)
    assert_close(scaled_out, want_s, s.dtype, what="custom scale")


def test_plan_reuse_flag_and_errors():
    import torch
    from paper_2605_06046_amd import (AttnParams, FEA_DTYPE_BF16, FEA_FLAG_REUSE_PLAN, FeaError,
                                      fea_decode_attention, fea_decode_workspace_bytes)
    from gpu_harness import to_device
    wl = W.generate(W.scaled(W.CONFIGS["c2"], **SMALL["c2"]))
    bt, lens = library_tables(wl)
    s = wl.spec
    p = AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, FEA_DTYPE_BF16, fused_max=-1)
    dq, dk, dv = to_device(wl.q), to_device(wl.k_cache), to_device(wl.v_cache)
    dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
    ws = torch.empty(fea_decode_workspace_bytes(p, s.batch, bt.shape[1]), dtype=torch.uint8, device="cuda")
    o1, o2 = torch.empty_like(dq), torch.empty_like(dq)
    fea_decode_attention(p, dq, dk, dv, dbt, dl, o1, ws)
    p2 = AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, FEA_DTYPE_BF16, flags=FEA_FLAG_REUSE_PLAN, fused_max=-1)
    dq2 = to_device(W.f32_to_bf16_bits(W.bf16_bits_to_f32(wl.q) * np.float32(0.5)))
    fea_decode_attention(p2, dq2, dk, dv, dbt, dl, o2, ws)     # "next layer": new q, same tables
    torch.cuda.synchronize()
    want2 = decode_attention(W.bf16_bits_to_f32(wl.q) * 0.5, values(wl.k_cache), values(wl.v_cache), bt, lens)
    assert_close(o2.float().cpu().numpy().astype(np.float64), want2, "bf16", what="reused plan")
    with pytest.raises(FeaError) as ei:
        fea_decode_attention(p, dq, dk, dv, dbt, dl, o1, ws[:4096])
    assert ei.value.code == -3
    with pytest.raises(FeaError):
        fea_decode_attention(p, dq, dk, dv, dbt, dl, o1, ws[1:])          # misaligned workspace
    # B == 0 is a no-op
    fea_decode_attention(p, dq[:0], dk, dv, dbt[:0], dl[:0], o1[:0], ws)


def test_profiling_events_bracket_each_kernel():
    import torch
    from paper_2605_06046_amd import (AttnParams, FEA_DTYPE_BF16, fea_decode_attention,
                                      fea_decode_workspace_bytes, fea_profile_enable, fea_profile_read)
    from gpu_harness import to_device
    wl = W.generate(W.scaled(W.CONFIGS["c2"], **SMALL["c2"]))
    bt, lens = library_tables(wl)
    s = wl.spec
    p = AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, FEA_DTYPE_BF16, fused_max=-1)
    dq, dk, dv = to_device(wl.q), to_device(wl.k_cache), to_device(wl.v_cache)
    dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
    ws = torch.empty(fea_decode_workspace_bytes(p, s.batch, bt.shape[1]), dtype=torch.uint8, device="cuda")
    ref = torch.empty_like(dq)
    fea_decode_attention(p, dq, dk, dv, dbt, dl, ref, ws)
    for which in (-1, 0, 1, 2):
        out = torch.empty_like(dq)
        fea_profile_enable(3, which)
        for _ in range(3):
            fea_decode_attention(p, dq, dk, dv, dbt, dl, out, ws)
        torch.cuda.synchronize()
        for c in range(3):
            ms = fea_profile_read(c)
            for k in range(3):
                if which in (-1, k):
                    assert 0.0 < ms[k] < 50.0, (which, c, ms)
                else:
                    assert ms[k] == 0.0, (which, c, ms)
        fea_profile_enable(0, -1)
        assert torch.equal(out, ref)                     # measuring does not change the result


@pytest.mark.gpu
@pytest.mark.parametrize("B,prefix,Hq,Hkv", [(300, 320, 32, 8), (500, 96, 32, 8), (130, 512, 64, 8), (300, 3200, 32, 8),
                                          (100, 640, 28, 4), (70, 320, 40, 8)])
def test_wide_prefix_groups(B, prefix, Hq, Hkv):
    """One prefix group far wider than a workgroup's row tiles (the paper's large homogeneous
    batches, Experiment 5): every request's rows against the oracle."""
    spec = W.Spec("wide", 21, "bf16", Hq, Hkv, 128, ((B, prefix),), (1, 70), interleave=True)
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["groups"] == 1 and info["grouped_requests"] == B and info["overflow"] == 0
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what=f"wide group B={B}")


@pytest.mark.gpu
def test_device_chunk_hashes_match_the_oracle():
    """Algorithm 2 on the device, bit for bit against the oracle's hash vectors: ragged lengths,
    empty requests, a request longer than one staging tile, unaligned starts."""
    import torch
    from oracle.hashing import chunk_hashes
    from paper_2605_06046_amd import fea_chunk_hashes_device
    rng = np.random.default_rng(17)
    lens = [0, 1, 15, 16, 17, 31, 32, 33, 100, 0, 4673, 16 * 2048, 16 * 2048 + 1, 16 * 2048 * 2 + 5, 3]
    seqs = [rng.integers(-2 ** 31, 2 ** 31, size=n, dtype=np.int64).astype(np.int32) for n in lens]
    toks = np.concatenate(seqs)
    toff = np.zeros(len(seqs) + 1, dtype=np.int64)
    toff[1:] = np.cumsum(lens)
    hoff = np.zeros(len(seqs) + 1, dtype=np.int64)
    hoff[1:] = np.cumsum([-(-n // 16) for n in lens])
    sentinel = 0x5A5A5A5A5A5A5A5A
    hashes = torch.full((int(hoff[-1]) + 3,), sentinel, dtype=torch.int64, device="cuda")
    fea_chunk_hashes_device(torch.from_numpy(toks).cuda(), torch.from_numpy(toff).cuda(), torch.from_numpy(hoff).cuda(), hashes)
    torch.cuda.synchronize()
    got = hashes.cpu().numpy().view(np.uint64)
    for i, s in enumerate(seqs):
        assert got[hoff[i]:hoff[i + 1]].tolist() == chunk_hashes(s), i
    assert (got[hoff[-1]:] == sentinel).all()                  # nothing written past the last request
    # a row that would not fit is skipped, the others are still written
    short = torch.full((int(hoff[-2]),), sentinel, dtype=torch.int64, device="cuda")
    fea_chunk_hashes_device(torch.from_numpy(toks).cuda(), torch.from_numpy(toff).cuda(), torch.from_numpy(hoff).cuda(), short)
    torch.cuda.synchronize()
    got2 = short.cpu().numpy().view(np.uint64)
    assert np.array_equal(got2, got[:hoff[-2]])
    # the same values as the host function of the library
    from paper_2605_06046_amd import fea_chunk_hashes
    assert got[hoff[10]:hoff[11]].tolist() == fea_chunk_hashes(seqs[10]).tolist()


def _radix_workload(dtype, top, subs, singles, Hq=32, Hkv=8, d=128, seed=31):
    """Token streams with two sharing levels (the radix patterns of Section 3): every request starts
    with the same `top` tokens; subs = [(members, extra shared tokens), ...]; `singles` requests share
    only the top level.  Requests arrive interleaved.  Returns a Workload with drawn q/K/V."""
    rng = np.random.default_rng(seed)
    top_t = rng.integers(0, W.VOCAB, size=top, dtype=np.int32)
    seqs = []
    for m, extra in subs:
        sub_t = rng.integers(0, W.VOCAB, size=extra, dtype=np.int32)
        seqs += [np.concatenate([top_t, sub_t, rng.integers(0, W.VOCAB, size=int(rng.integers(1, 90)), dtype=np.int32)])
                 for _ in range(m)]
    seqs += [np.concatenate([top_t, rng.integers(0, W.VOCAB, size=int(rng.integers(1, 90)), dtype=np.int32)])
             for _ in range(singles)]
    order = rng.permutation(len(seqs))
    seqs = [seqs[j] for j in order]
    spec = W.Spec("radix", 41, dtype, Hq, Hkv, d, ((len(seqs), 0),), (1, 1))
    base = W.generate(spec)                       # for q and the K/V pool's value distribution
    toks = np.concatenate(seqs)
    offs = np.zeros(len(seqs) + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(s) for s in seqs])
    nblk = int(sum(-(-len(s) // 16) for s in seqs))
    rs = np.random.default_rng(seed + 1)
    shape = (nblk, Hkv, 16, d)
    k = rs.standard_normal(shape, dtype=np.float32)
    v = rs.standard_normal(shape, dtype=np.float32)
    if dtype == "bf16":
        k, v = W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)
    return dataclasses.replace(base, tokens=toks, tok_offsets=offs, k_cache=k, v_cache=v, num_blocks=nblk,
                               max_blocks_per_seq=max(-(-len(s) // 16) for s in seqs) + 1,
                               group_of=np.zeros(len(seqs), dtype=np.int32))


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("bf16", 32, 8, 128), ("f32", 8, 2, 64)])
def test_two_level_prefix_sharing(dtype, Hq, Hkv, d):
    """Nested prefixes: subgroups that go on sharing past the common run become groups of their own
    when that pays; whatever the planner decides, every row must match the oracle."""
    # 96 shared tokens (6 blocks); subgroups of 5 and 4 share 160 and 64 more; a pair shares 16 more
    # (too little to pay for sweeping the top level again); three requests share the top level only
    wl = _radix_workload(dtype, 96, [(5, 160), (4, 64), (2, 16)], 3, Hq, Hkv, d)
    out, bt, lens, info = run_workload(wl)
    assert_close(out, oracle_for(wl, bt, lens), dtype, what="two-level sharing")
    # in sweep cost (a tile with <= 16 / <= 32 query rows weighs 16 / 20): the five save 16*5*10 = 800 for a
    # run of 16 blocks at 20; the four save 16*4*4 = 256 for 10 blocks at 16; the pair would save 16*2*1 = 32
    # for 7 blocks at 16.  Two subgroups split off, the pair and the singles keep the top run.
    assert info["groups"] == 3 and info["grouped_requests"] == 14
    assert info["shared_blocks"] == 16 + 10 + 6
    # the same with a deep second level everywhere: all three subgroups split off, the singles keep the top run
    wl = _radix_workload(dtype, 64, [(6, 320), (3, 480), (2, 640)], 4, Hq, Hkv, d, seed=32)
    out, bt, lens, info = run_workload(wl)
    assert_close(out, oracle_for(wl, bt, lens), dtype, what="two-level sharing, deep")
    assert info["groups"] == 4 and info["grouped_requests"] == 15
    assert info["shared_blocks"] == (4 + 20) + (4 + 30) + (4 + 40) + 4


def test_captured_graph_replays_match_eager_calls():
    """The library neither allocates nor synchronises, so a decode step (append + attention) can be
    captured into a HIP graph.  Every replay, with the inputs changed in place between replays and
    eager work of the program in between, must give what the eager call gives on the same inputs."""
    import torch
    from paper_2605_06046_amd import (AttnParams, FEA_DTYPE_BF16, fea_decode_attention, fea_decode_workspace_bytes,
                                      fea_kv_append)
    from gpu_harness import to_device
    wl = W.generate(W.scaled(W.CONFIGS["c3"], 4, 8, name="c3_graph"))
    bt, lens = library_tables(wl)
    s = wl.spec
    params = AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, FEA_DTYPE_BF16, fused_max=-1)
    B, stride = bt.shape
    q, k, v = to_device(wl.q), to_device(wl.k_cache), to_device(wl.v_cache)
    dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
    ws = torch.empty(fea_decode_workspace_bytes(params, B, stride), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty_like(ws)
    out_g, out_e = torch.empty_like(q), torch.empty_like(q)
    g = torch.Generator(device="cuda"); g.manual_seed(3)
    k_new = torch.randn((B, s.num_kv_heads, s.head_dim), generator=g, device="cuda").to(torch.bfloat16)
    v_new = torch.randn((B, s.num_kv_heads, s.head_dim), generator=g, device="cuda").to(torch.bfloat16)

    def step(out, wsx, stream=None):
        fea_kv_append(params, k_new, v_new, k, v, dbt, dl, stream=stream)     # rewrites position L-1 of every request
        fea_decode_attention(params, q, k, v, dbt, dl, out, wsx, stream=stream)

    side = torch.cuda.Stream()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(out_g, ws, side)
        side.synchronize()
        with torch.cuda.graph(gr, stream=side):
            step(out_g, ws, side)
    torch.cuda.synchronize()
    for rep in range(4):
        # change the inputs in place: new query, new rows to append
        q.copy_(torch.randn(q.shape, generator=g, device="cuda").to(torch.bfloat16))
        k_new.copy_(torch.randn(k_new.shape, generator=g, device="cuda").to(torch.bfloat16))
        v_new.copy_(torch.randn(v_new.shape, generator=g, device="cuda").to(torch.bfloat16))
        out_g.fill_(float("nan"))
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        step(out_e, ws2)                       # eager, own workspace, same inputs (the append is idempotent)
        _ = (out_e.float() * 2).sum().item()   # unrelated eager work and a synchronisation between replays
        assert torch.equal(out_g, out_e), f"replay {rep} differs from the eager call"
    # and the last replay against the oracle
    kk, vv = k.float().cpu().numpy().astype(np.float64), v.float().cpu().numpy().astype(np.float64)
    want = decode_attention(q.float().cpu().numpy().astype(np.float64), kk, vv, bt, lens)
    assert_close(out_g.float().cpu().numpy().astype(np.float64), want, "bf16", what="graph replay")


def test_more_requests_than_the_grouping_limit():
    """Requests with index >= 2048 are never grouped (they sweep the prefix on their own); the rows of
    all 2100 requests must still match the oracle, grouped or not."""
    spec = W.Spec("many", 23, "bf16", 8, 2, 128, ((1400, 64), (700, 48)), (1, 40), interleave=True)
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["overflow"] == 0 and info["groups"] == 2 and info["grouped_requests"] == 2048
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what="B=2100")


def test_plan_only_then_reuse_equals_one_call():
    """FEA_FLAG_PLAN_ONLY leaves in the workspace exactly the plan a full call would make: planning on
    a side stream, then attending with FEA_FLAG_REUSE_PLAN, gives the full call's output bit for bit."""
    import torch
    from paper_2605_06046_amd import (AttnParams, FEA_DTYPE_BF16, FEA_FLAG_PLAN_ONLY, FEA_FLAG_REUSE_PLAN, FeaError,
                                      fea_decode_attention, fea_decode_workspace_bytes)
    from gpu_harness import to_device
    wl = W.generate(W.scaled(W.CONFIGS["c2"], 2, 4, name="c2_plan_only"))
    bt, lens = library_tables(wl)
    s = wl.spec
    mk = lambda flags: AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, FEA_DTYPE_BF16, flags=flags, fused_max=-1)
    q, k, v = to_device(wl.q), to_device(wl.k_cache), to_device(wl.v_cache)
    dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
    n = fea_decode_workspace_bytes(mk(0), *bt.shape)
    ws_a, ws_b = (torch.zeros(n, dtype=torch.uint8, device="cuda") for _ in range(2))
    out_a, out_b = torch.full_like(q, float("nan")), torch.full_like(q, float("nan"))
    fea_decode_attention(mk(0), q, k, v, dbt, dl, out_a, ws_a)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    fea_decode_attention(mk(FEA_FLAG_PLAN_ONLY), q, k, v, dbt, dl, out_b, ws_b, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    assert torch.isnan(out_b.float()).all()                      # planning alone writes no output
    fea_decode_attention(mk(FEA_FLAG_REUSE_PLAN), q, k, v, dbt, dl, out_b, ws_b)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b)
    with pytest.raises(FeaError):
        fea_decode_attention(mk(FEA_FLAG_PLAN_ONLY | FEA_FLAG_REUSE_PLAN), q, k, v, dbt, dl, out_b, ws_b)


def test_very_long_contexts():
    """Maximum sizes: two requests that share a 60 000-token prefix, and one request of 120 000
    tokens (thousands of table columns, the block-id windows refilled many times)."""
    pair = W.generate(W.Spec("long_pair", 24, "bf16", 32, 8, 128, ((2, 60000),), (17, 300)))
    out, bt, lens, info = run_workload(pair)
    assert info["groups"] == 1 and info["shared_blocks"] == 3750 and info["overflow"] == 0
    assert_close(out, oracle_for(pair, bt, lens), "bf16", what="60k shared prefix")
    lone = W.generate(W.Spec("long_one", 26, "bf16", 32, 8, 128, ((1, 0),), (120000, 120000)))
    out, bt, lens, info = run_workload(lone)
    assert bt.shape[1] >= 7500 and info["groups"] == 0 and info["overflow"] == 0
    assert_close(out, oracle_for(lone, bt, lens), "bf16", what="120k tokens, one request")


def test_many_small_groups():
    """Hundreds of prefix groups of two or three requests in arrival order: the group lists, the
    member offsets and the item emission by teams of waves all run at their widest."""
    groups = tuple((2 + (i % 2), 32 + 16 * (i % 5)) for i in range(500))
    spec = W.Spec("pairs", 25, "bf16", 16, 4, 128, groups, (1, 60), interleave=True)
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["groups"] == 500 and info["grouped_requests"] == spec.batch and info["overflow"] == 0
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what="500 small groups")


def test_three_level_prefix_sharing():
    """A system prompt (64 tokens) shared by 16 requests, four conversations of four sharing 160 more,
    and in each conversation two pairs sharing 320 more: the planner follows the sharing down level by
    level (every split pays by the tile weights), ending with eight pairs whose run is 4 + 10 + 20 blocks."""
    rng = np.random.default_rng(51)
    draw = lambda n: rng.integers(0, W.VOCAB, size=n, dtype=np.int32)
    top = draw(64)
    seqs = []
    for conv in range(4):
        mid = draw(160)
        for pair in range(2):
            deep = draw(320)
            for _ in range(2):
                seqs.append(np.concatenate([top, mid, deep, draw(int(rng.integers(1, 60)))]))
    order = rng.permutation(len(seqs))
    seqs = [seqs[j] for j in order]
    spec = W.Spec("three_levels", 43, "bf16", 32, 8, 128, ((len(seqs), 0),), (1, 1))
    base = W.generate(spec)
    offs = np.zeros(len(seqs) + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(x) for x in seqs])
    nblk = int(sum(-(-len(x) // 16) for x in seqs))
    rs = np.random.default_rng(52)
    k = W.f32_to_bf16_bits(rs.standard_normal((nblk, 8, 16, 128), dtype=np.float32))
    v = W.f32_to_bf16_bits(rs.standard_normal((nblk, 8, 16, 128), dtype=np.float32))
    wl = dataclasses.replace(base, tokens=np.concatenate(seqs), tok_offsets=offs, k_cache=k, v_cache=v, num_blocks=nblk,
                             max_blocks_per_seq=max(-(-len(x) // 16) for x in seqs) + 1,
                             group_of=np.zeros(len(seqs), dtype=np.int32))
    out, bt, lens, info = run_workload(wl)
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what="three sharing levels")
    assert info["groups"] == 8 and info["grouped_requests"] == 16 and info["shared_blocks"] == 8 * 34


@pytest.mark.parametrize("case", ["c2_small", "c3_small", "two_level", "nested_tables", "random_tables", "odd_stride"])
def test_runs_found_on_many_workgroups_give_the_same_plan(case):
    """Large tables have their leaders and common runs found by a kernel of many workgroups before the
    planner; forced on here for small ones: same plan (group counts, items, rows), bitwise the same output."""
    if case in ("c2_small", "c3_small"):
        wl = W.generate(W.scaled(W.CONFIGS[case[:2]], **SMALL[case[:2]]))
        bt, lens = library_tables(wl)
        q, k, v, s = wl.q, wl.k_cache, wl.v_cache, wl.spec
        shape = (s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
    elif case == "two_level":
        wl = _radix_workload("bf16", 96, [(5, 160), (4, 64), (2, 16)], 3)
        bt, lens = library_tables(wl)
        q, k, v, shape = wl.q, wl.k_cache, wl.v_cache, (32, 8, 128, "bf16")
    else:
        lens_l = [0, 160, 161, 500, 512, 100, 160, 160, 700, 48, 64, 49, 1000]
        mode = {"nested_tables": "nested", "random_tables": "same_first_then_random", "odd_stride": "nested"}[case]
        bt, k, v = _random_tables(7, len(lens_l), 8, 128, "bf16", lens_l, 40, mode)
        if case == "odd_stride":
            bt = np.ascontiguousarray(np.concatenate([bt, np.full((bt.shape[0], 3 - bt.shape[1] % 2), -1, np.int32)], axis=1))
            assert bt.shape[1] % 4 != 0
        lens = np.array(lens_l, dtype=np.int32)
        q = W.f32_to_bf16_bits(np.random.default_rng(5).standard_normal((len(lens_l), 32, 128), dtype=np.float32))
        shape = (32, 8, 128, "bf16")
    base, info = run_hip(q, k, v, bt, lens, *shape)
    forced, info2 = run_hip(q, k, v, bt, lens, *shape, run_kernel_min=-1)
    assert info2 == info
    assert np.array_equal(base, forced)
    assert_close(forced, decode_attention(values(q), values(k), values(v), bt, lens), "bf16", what=case)


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 4, 4, 32), ("f32", 6, 2, 128), ("f32", 2, 1, 256), ("bf16", 12, 4, 64),
                                            ("bf16", 8, 8, 256), ("bf16", 32, 8, 128), ("bf16", 64, 8, 128)])
def test_merge_with_several_rows_per_wave(dtype, Hq, Hkv, d):
    """Batches of very many rows are merged several rows to a wave; forced on here for small ones,
    including rows with many partials, rows of zero length and a ragged last wave."""
    spec = W.Spec("rows", 27, dtype, Hq, Hkv, d, ((5, 96), (3, 0), (1, 1200)), (1, 200))
    wl = W.generate(spec)
    want = None
    for forced in (1000000000, -1):                    # never / always several rows per wave
        out, bt, lens, info = run_workload(wl, split_blocks=2 if forced < 0 else 0, merge_rows_min=forced)   # many pieces per row
        want = oracle_for(wl, bt, lens) if want is None else want
        assert_close(out, want, dtype, what=f"merge rows {forced} {dtype} {Hq}/{Hkv}/{d}")


def _random_prefix_tree_batch(seed, dtype, Hq, Hkv, d):
    """A batch whose token streams come from a random prefix tree (depth up to 4, random fan-out and
    segment lengths, some requests ending exactly on a node, some empty or shorter than a block)."""
    rng = np.random.default_rng(seed)
    draw = lambda n: rng.integers(0, W.VOCAB, size=int(n), dtype=np.int32)
    seqs = []

    def grow(prefix, depth):
        for _ in range(int(rng.integers(2, 5))):
            seg = draw(rng.choice([16, 32, 48, 80, 160, 7, 100]))
            node = np.concatenate([prefix, seg])
            for _ in range(int(rng.integers(0, 5))):       # requests hanging off this node
                tail = draw(rng.choice([0, 1, 5, 16, 33, 70]))
                seqs.append(np.concatenate([node, tail]))
            if depth < 4 and rng.random() < 0.8:
                grow(node, depth + 1)

    grow(np.zeros(0, dtype=np.int32), 1)
    seqs += [np.zeros(0, dtype=np.int32), draw(3), draw(16)]
    order = rng.permutation(len(seqs))
    seqs = [seqs[j] for j in order][:220]
    spec = W.Spec("tree", 44, dtype, Hq, Hkv, d, ((len(seqs), 0),), (1, 1))
    base = W.generate(spec)
    offs = np.zeros(len(seqs) + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(x) for x in seqs])
    nblk = max(1, int(sum(-(-len(x) // 16) for x in seqs)))
    rs = np.random.default_rng(seed + 1000)
    k = rs.standard_normal((nblk, Hkv, 16, d), dtype=np.float32)
    v = rs.standard_normal((nblk, Hkv, 16, d), dtype=np.float32)
    if dtype == "bf16":
        k, v = W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)
    toks = np.concatenate(seqs) if sum(len(x) for x in seqs) else np.zeros(0, dtype=np.int32)
    return dataclasses.replace(base, tokens=toks, tok_offsets=offs, k_cache=k, v_cache=v, num_blocks=nblk,
                               max_blocks_per_seq=max(1, max(-(-len(x) // 16) for x in seqs)) + int(rng.integers(0, 4)),
                               group_of=np.zeros(len(seqs), dtype=np.int32))


@pytest.mark.parametrize("seed", range(10))
def test_random_prefix_trees(seed):
    """Random prefix trees through every path of the alias detection (nested runs, several levels,
    odd table strides, the many-workgroup run kernel forced on and off) against the oracle."""
    dtype, Hq, Hkv, d = [("bf16", 32, 8, 128), ("bf16", 28, 4, 128), ("bf16", 8, 8, 128), ("f32", 8, 2, 64),
                         ("bf16", 12, 2, 128)][seed % 5]
    wl = _random_prefix_tree_batch(100 + seed, dtype, Hq, Hkv, d)
    out, bt, lens, info = run_workload(wl)
    want = oracle_for(wl, bt, lens)
    assert info["overflow"] == 0
    assert_close(out, want, dtype, what=f"tree {seed}")
    out2, _, _, info2 = run_workload(wl, run_kernel_min=-1)
    assert info2 == info and np.array_equal(out, out2)


@pytest.mark.parametrize("B,Hq,Hkv", [(24, 32, 8), (32, 32, 8), (48, 32, 8), (64, 32, 8), (80, 32, 8), (20, 28, 4), (9, 64, 8)])
@pytest.mark.parametrize("scores", ["plain", "rising", "falling"])
def test_shared_runs_swept_by_teams_of_waves(B, Hq, Hkv, scores):
    """Prefix groups of 2, 3, 4 and 5 row tiles of 64 query rows (a last row tile that is not full, teams with
    a member that only fetches), whose shared run is swept by teams of waves, against the oracle - also with
    keys arranged so that the scores rise steeply along the shared prefix (every tile outgrows the reference
    exponent of its rows, which must then be raised and the sums rescaled) or fall (everything after the first
    tiles underflows)."""
    prefix = 2048
    spec = W.Spec("teams", 61, "bf16", Hq, Hkv, 128, ((B, prefix),), (1, 90))
    wl = W.generate(spec)
    bt, lens = library_tables(wl)
    if scores != "plain":
        d = 128
        k = W.bf16_bits_to_f32(wl.k_cache)
        t = np.arange(prefix, dtype=np.float32)
        ramp = (t if scores == "rising" else (prefix - 1 - t)) * np.float32(0.87) / np.float32(np.sqrt(d))
        shared = bt[0, :prefix // 16]                                   # the prefix blocks, in token order
        k[shared] = (k[shared].reshape(prefix // 16, Hkv, 16, d) * np.float32(0.05)
                     + ramp.reshape(prefix // 16, 1, 16, 1))
        wl.k_cache[:] = W.f32_to_bf16_bits(k)
        q = W.bf16_bits_to_f32(wl.q) * np.float32(0.1) + np.float32(1.0)    # every query points along the ramp
        wl.q[:] = W.f32_to_bf16_bits(q)
    W.poison_dead_slots(wl, bt, lens)
    s = wl.spec
    out, info = run_hip(wl.q, wl.k_cache, wl.v_cache, bt, lens, s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
    assert info["groups"] == 1 and info["grouped_requests"] == B and info["overflow"] == 0
    want = oracle_for(wl, bt, lens)
    assert_close(out, want, "bf16", what=f"teams B={B} {Hq}/{Hkv} {scores}")
    if scores == "rising":
        assert np.abs(want).max() > 0.5          # the softmax sits on the last prefix tokens: outputs are O(1)


@pytest.mark.parametrize("B,prefix", [(24, 2064), (32, 1968), (64, 2096), (96, 1040), (150, 784)])
def test_runs_of_odd_length_and_uneven_pieces_swept_by_teams(B, prefix):
    """Shared runs of an odd number of blocks, and of lengths that no number of pieces divides: a team takes an even
    number of columns, so the planner leaves a run's last odd column to the members' own sweeps (the plan reports
    one shared block less) and deals the tiles out evenly over the pieces."""
    spec = W.Spec("teams_odd", 63, "bf16", 32, 8, 128, ((B, prefix),), (1, 75))
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    blocks = prefix // 16
    assert info["groups"] == 1 and info["grouped_requests"] == B and info["overflow"] == 0
    assert info["shared_blocks"] == blocks - (blocks & 1)
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what=f"teams on a run of {blocks} blocks, B={B}")


def test_long_pieces_of_a_shared_run_swept_by_teams():
    """200 requests on a 16 384-token prefix: 13 row tiles per KV head take most of the waves, so the run is cut
    into few pieces of more than 128 columns each (the teams' block-id table holds up to 1024); sampled requests
    against the oracle, all rows finite."""
    spec = W.Spec("teams_long", 62, "bf16", 32, 8, 128, ((200, 16384),), (1, 70))
    wl = W.generate(spec)
    bt, lens = library_tables(wl)
    W.poison_dead_slots(wl, bt, lens)
    s = wl.spec
    out, info = run_hip(wl.q, wl.k_cache, wl.v_cache, bt, lens, s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
    assert info["groups"] == 1 and info["grouped_requests"] == 200 and info["overflow"] == 0
    assert info["items"] < 16 * 8 * 8 + 200 * 8 + 64        # at most 7 pieces of the 512-tile run: more than 64 tiles each
    assert np.isfinite(out).all()
    sample = [0, 1, 63, 64, 127, 128, 192, 199]
    want = oracle_for(wl, bt, lens, requests=sample)
    assert_close(out[sample], want[sample], "bf16", what="teams, pieces of more than 128 columns")


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
@pytest.mark.parametrize("heads", [(32, 8), (28, 4), (8, 8)])
def test_head_dim_64_on_the_matrix_core(name, heads):
    """bf16 caches with head_dim 64 take the matrix-core sweep too (2 KB blocks, two k-steps, four output products
    per 16 rows; shared runs with more than 64 rows go row tile by row tile, the team sequence being written for
    head_dim 128): the scaled batch shapes, a few query-group sizes, against the oracle."""
    spec = dataclasses.replace(W.scaled(W.CONFIGS[name], **SMALL[name]), head_dim=64, num_q_heads=heads[0],
                               num_kv_heads=heads[1], name=f"{name}_d64")
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["variant"] == 1 and info["overflow"] == 0
    print(name, heads, info, assert_close(out, oracle_for(wl, bt, lens), "bf16", what=f"{name} d=64 {heads}"))


def test_head_dim_64_wide_group_and_long_rows():
    """head_dim 64 with a prefix group of several row tiles (72 requests x 4 heads per KV head), items of 16, 32 and
    64 rows, ragged lengths, and scores that rise along the prefix (the reference exponents get raised)."""
    spec = W.Spec("d64_wide", 63, "bf16", 16, 4, 64, ((72, 1024), (9, 160), (3, 0)), (1, 90))
    wl = W.generate(spec)
    bt, lens = library_tables(wl)
    k = W.bf16_bits_to_f32(wl.k_cache)
    t = np.arange(1024, dtype=np.float32)
    shared = bt[0, :64]
    k[shared] = k[shared].reshape(64, 4, 16, 64) * np.float32(0.05) + (t * np.float32(0.9) / np.float32(8.0)).reshape(64, 1, 16, 1)
    wl.k_cache[:] = W.f32_to_bf16_bits(k)
    wl.q[:] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(wl.q) * np.float32(0.1) + np.float32(1.0))
    W.poison_dead_slots(wl, bt, lens)
    s = wl.spec
    out, info = run_hip(wl.q, wl.k_cache, wl.v_cache, bt, lens, s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
    assert info["variant"] == 1 and info["groups"] == 2
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what="d=64 wide group, rising scores")


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
@pytest.mark.parametrize("heads", [(16, 4), (14, 2), (4, 4)])
def test_head_dim_256_on_the_matrix_core(name, heads):
    """bf16 caches with head_dim 256 on the matrix-core sweep: 8 KB blocks, eight k-steps, sixteen output products
    per 16 rows, work items of at most 32 query rows, two waves per workgroup."""
    spec = dataclasses.replace(W.scaled(W.CONFIGS[name], **SMALL[name]), head_dim=256, num_q_heads=heads[0],
                               num_kv_heads=heads[1], name=f"{name}_d256")
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["variant"] == 1 and info["overflow"] == 0
    print(name, heads, info, assert_close(out, oracle_for(wl, bt, lens), "bf16", what=f"{name} d=256 {heads}"))


def test_head_dim_256_wide_group_and_rising_scores():
    spec = W.Spec("d256_wide", 64, "bf16", 8, 2, 256, ((40, 512), (9, 160), (3, 0)), (1, 90))
    wl = W.generate(spec)
    bt, lens = library_tables(wl)
    k = W.bf16_bits_to_f32(wl.k_cache)
    t = np.arange(512, dtype=np.float32)
    shared = bt[0, :32]
    k[shared] = k[shared].reshape(32, 2, 16, 256) * np.float32(0.05) + (t * np.float32(0.9) / np.float32(16.0)).reshape(32, 1, 16, 1)
    wl.k_cache[:] = W.f32_to_bf16_bits(k)
    wl.q[:] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(wl.q) * np.float32(0.1) + np.float32(1.0))
    W.poison_dead_slots(wl, bt, lens)
    s = wl.spec
    out, info = run_hip(wl.q, wl.k_cache, wl.v_cache, bt, lens, s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
    assert info["variant"] == 1 and info["groups"] == 2
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what="d=256 wide group, rising scores")


@pytest.mark.parametrize("Hq,Hkv,d", [(34, 2, 128), (32, 1, 128), (64, 1, 128), (60, 1, 64), (48, 2, 64), (20, 1, 256), (32, 1, 256),
                                      (40, 1, 128), (64, 2, 128)])
def test_wide_query_groups_on_the_matrix_core(Hq, Hkv, d):
    """Multi-query shapes: a request's query group of 17..64 heads per KV head (up to 32 at head_dim 256) is one
    work item of that many rows; prefix groups stack one or two requests per row tile, or none (64 heads)."""
    spec = W.Spec("mqa", 65, "bf16", Hq, Hkv, d, ((6, 320), (3, 96), (2, 0)), (1, 200))
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["variant"] == 1 and info["overflow"] == 0 and info["groups"] == 2
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what=f"query groups of {Hq // Hkv} heads, d={d}")


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_against_the_oracle(seed):
    """Seeded random draws over everything the interface accepts at once: cache type, head dim, head counts (query
    groups of 1 to 64 heads), prefix groups of random sizes and depths next to requests on their own, suffix
    ranges, arrival order, pool permutation - whichever kernels the shape selects."""
    rng = np.random.default_rng(9000 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    d = int(rng.choice([64, 128, 256] if dtype == "bf16" else [32, 64, 128, 256]))
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 24, 32] if d == 256 else [1, 2, 3, 4, 5, 7, 8, 12, 16, 24, 40, 64]))
    if dtype == "f32":
        G = min(G, 8)
    groups = []
    for _ in range(int(rng.integers(0, 4))):
        groups.append((int(rng.integers(2, 40)), int(rng.integers(1, 30)) * 16))
    groups += [(1, 0)] * int(rng.integers(0, 6))
    if not groups:
        groups = [(3, 0)]
    lo = int(rng.integers(1, 60))
    spec = W.Spec(f"rand{seed}", 100 + seed, dtype, G * Hkv, Hkv, d, tuple(groups), (lo, lo + int(rng.integers(0, 300))),
                  interleave=bool(rng.integers(0, 2)), pool_factor=1.0 + float(rng.random()),
                  perm_seed=int(rng.integers(0, 2)) * (seed + 1))
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl)
    assert info["overflow"] == 0
    print(seed, dtype, d, G * Hkv, Hkv, groups, info, assert_close(out, oracle_for(wl, bt, lens), dtype, what=f"random shape {seed}"))


# ---- batches small enough for one launch (no plan, no partial results) ----

def test_c1_takes_one_launch_by_default():
    wl = W.generate(W.CONFIGS["c1"])
    out, bt, lens, info = run_workload(wl, fused_max=0)
    assert info["variant"] == 2 and info["items"] == 0 and info["groups"] == 0 and info["overflow"] == 0
    print("c1 fused", assert_close(out, oracle_for(wl, bt, lens), "f32", what="c1 in one launch"))
    # the bound is on the row length and on the number of (request, KV head) pairs: the scaled c2 has longer rows
    wl = W.generate(W.scaled(W.CONFIGS["c2"], **SMALL["c2"]))
    out, bt, lens, info = run_workload(wl, fused_max=0)
    assert bt.shape[1] <= 64 or info["variant"] == 1
    out, bt, lens, info = run_workload(wl, fused_max=bt.shape[1])        # an explicit bound takes it
    assert info["variant"] == 2
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what="scaled c2 in one launch")
    out, bt, lens, info = run_workload(wl, fused_max=bt.shape[1] - 1)    # one entry short of the rows: planned
    assert info["variant"] == 1 and info["groups"] == 1


@pytest.mark.parametrize("mode", ["random", "same_first_then_random", "nested", "all_same_block", "identical_rows"])
@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 8, 2, 64), ("f32", 4, 4, 32), ("f32", 6, 2, 128), ("f32", 2, 1, 256),
                                            ("f32", 16, 2, 64), ("f32", 24, 2, 128), ("f32", 5, 1, 32), ("f32", 8, 1, 256),
                                            ("bf16", 32, 8, 128), ("bf16", 10, 2, 128), ("bf16", 16, 4, 64), ("bf16", 9, 1, 256)])
def test_any_block_table_in_one_launch(mode, dtype, Hq, Hkv, d):
    """Empty, one-token, block-edge and ragged histories; query groups of 1 to 12 heads (passes of four heads, of
    eight for wide groups over float32 caches, the last pass ragged); every cache type and head dim; tables that
    alias anywhere."""
    lens = [0, 1, 15, 16, 17, 160, 161, 500, 512, 33, 160, 160, 700, 2, 48, 31]
    B = len(lens)
    seed = {"random": 111, "same_first_then_random": 212, "nested": 313, "all_same_block": 414, "identical_rows": 515}[mode]
    bt, k, v = _random_tables(seed, B, Hkv, d, dtype, lens, 40, mode)
    rng = np.random.default_rng(6)
    q = rng.standard_normal((B, Hq, d), dtype=np.float32)
    if dtype == "bf16":
        q = W.f32_to_bf16_bits(q)
    L = np.array(lens, dtype=np.int32)
    out, info = run_hip(q, k, v, bt, L, Hq, Hkv, d, dtype, fused_max=bt.shape[1])
    assert info["variant"] == 2
    assert_close(out, decode_attention(values(q), values(k), values(v), bt, L), dtype, what=f"one launch, {mode}")
    assert (out[0] == 0).all()                        # zero-length request
    out_s, _ = run_hip(q, k, v, bt, L, Hq, Hkv, d, dtype, fused_max=bt.shape[1], scale=0.05)
    assert_close(out_s, decode_attention(values(q), values(k), values(v), bt, L, scale=0.05), dtype, what="one launch, custom scale")


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
@pytest.mark.parametrize("peaked", [False, True])
def test_scaled_configs_in_one_launch(name, peaked):
    """The one-launch kernel forced onto the scaled configurations (rows of up to 150 table entries, 8 to 32
    requests), with ordinary and with sharply peaked scores; twice, bit for bit."""
    spec = W.scaled(W.CONFIGS[name], **SMALL[name])
    wl = W.generate(dataclasses.replace(spec, q_gain=8.0) if peaked else spec)
    out, bt, lens, info = run_workload(wl, fused_max=1 << 20)
    assert info["variant"] == 2
    assert_close(out, oracle_for(wl, bt, lens), "bf16", what=f"{name} in one launch")
    again, _, _, _ = run_workload(wl, fused_max=1 << 20)
    assert np.array_equal(out, again)


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("bf16", 8, 2, 128), ("f32", 4, 1, 64), ("bf16", 64, 1, 64)])
def test_one_launch_on_rows_longer_than_its_table_buffer(dtype, Hq, Hkv, d):
    """The kernel keeps the first 512 entries of a request's table row in LDS and reads the rest from memory: histories
    of 8200 to 9500 tokens next to short ones, grouping flags that mean nothing to it, query groups of up to 64 heads
    (16 passes)."""
    spec = W.Spec("long_rows", 21, dtype, Hq, Hkv, d, ((2, 8192), (1, 0), (1, 0)), (5, 1300))
    wl = W.generate(spec)
    out, bt, lens, info = run_workload(wl, fused_max=1 << 20, max_group=1, split_blocks=6)
    assert bt.shape[1] > 512 and lens.max() > 8192 + 16 and info["variant"] == 2
    assert_close(out, oracle_for(wl, bt, lens), dtype, what=f"one launch, long rows {dtype} {Hq}/{Hkv}/{d}")


def test_calls_from_two_threads_on_streams_and_workspaces_of_their_own():
    """Nothing in a call is shared between callers but the read-only tuning (and, while it is on, the recording of
    kernel durations, which takes a lock): two threads, each with its stream, workspace and output, give what one does."""
    import threading
    import torch
    from paper_2605_06046_amd import (AttnParams, FEA_DTYPE_BF16, fea_decode_attention, fea_decode_workspace_bytes,
                                      fea_profile_enable, fea_profile_read)
    from gpu_harness import to_device
    wls = [W.generate(W.scaled(W.CONFIGS[n], **SMALL[n])) for n in ("c2", "c3")]
    jobs = []
    for wl in wls:
        bt, lens = library_tables(wl)
        s = wl.spec
        p = AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, FEA_DTYPE_BF16, fused_max=-1)
        q, k, v = to_device(wl.q), to_device(wl.k_cache), to_device(wl.v_cache)
        dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
        ws = torch.empty(fea_decode_workspace_bytes(p, s.batch, bt.shape[1]), dtype=torch.uint8, device="cuda")
        ref = torch.empty_like(q)
        fea_decode_attention(p, q, k, v, dbt, dl, ref, ws)
        jobs.append(dict(p=p, q=q, k=k, v=v, dbt=dbt, dl=dl, ws=ws, ref=ref, outs=[], stream=torch.cuda.Stream(), err=None))
    torch.cuda.synchronize()

    def work(j):
        try:
            for out in j["outs"]:
                fea_decode_attention(j["p"], j["q"], j["k"], j["v"], j["dbt"], j["dl"], out, j["ws"], stream=j["stream"])
            j["stream"].synchronize()
        except Exception as e:   # surfaces in the main thread
            j["err"] = e

    for recording in (False, True):
        if recording:
            fea_profile_enable(64, -1)
        try:
            for j in jobs:      # outputs made (and poisoned) here, so that the threads only make the library's calls
                j["outs"] = [torch.full_like(j["q"], float("nan")) for _ in range(25)]
            torch.cuda.synchronize()
            threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
            for t in threads:
                t.start()
            for t in threads:
                t.join()
            for j in jobs:
                assert j["err"] is None, j["err"]
                assert len(j["outs"]) == 25 and all(torch.equal(o, j["ref"]) for o in j["outs"])
            if recording:
                ms = [fea_profile_read(c) for c in range(50)]
                assert all(m[1] > 0 for m in ms)
        finally:
            if recording:
                fea_profile_enable(0, -1)
