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
    p = fea.AttnParams(spec.num_q_heads, spec.num_kv_heads, spec.head_dim, dtype, fused_max=-1)
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


class _Loop:
    """Device and host state of a decode loop on one batch: step() grows every request by one token
    (tables and lengths on the host, K/V rows through the append kernel; the oracle's caches follow)."""

    def __init__(self, spec, steps, seed=11, fused_max=-1):
        import torch
        self.fused_max = fused_max   # -1: plan, sweep and merge also where the library would take the batch in one launch
        import paper_2605_06046_amd as fea
        from gpu_harness import to_device
        self.fea, self.torch, self.to_device, self.spec = fea, torch, to_device, spec
        wl = W.generate(spec)
        nb_total = wl.num_blocks + (steps // 16 + 2) * spec.batch
        self.pool = fea.fea_kv_alloc(nb_total, 16, wl.perm_seed)
        self.width = wl.max_blocks_per_seq + steps // 16 + 2
        self.bt, self.lens, _, _ = fea.fea_build_block_tables(self.pool, wl.tokens, wl.tok_offsets, self.width)

        def grow(c):
            out = np.zeros((nb_total,) + c.shape[1:], dtype=c.dtype)
            out[:c.shape[0]] = c
            return out
        self.hk, self.hv = grow(wl.k_cache), grow(wl.v_cache)
        W.poison_dead_slots(dataclass_replace(wl, k_cache=self.hk, v_cache=self.hv, num_blocks=nb_total), self.bt, self.lens)
        self.dk, self.dv = to_device(self.hk), to_device(self.hv)
        self.dtype = fea.FEA_DTYPE_BF16 if spec.dtype == "bf16" else fea.FEA_DTYPE_F32
        self.p = self.params(0)
        self.ws = torch.zeros(fea.fea_decode_workspace_bytes(self.p, spec.batch, self.width), dtype=torch.uint8, device="cuda")
        self.rng = np.random.default_rng(seed)
        self.sync_tables()

    def params(self, flags):
        s = self.spec
        return self.fea.AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, self.dtype, flags=flags, fused_max=self.fused_max)

    def sync_tables(self):
        self.dbt, self.dl = self.torch.from_numpy(self.bt).cuda(), self.torch.from_numpy(self.lens).cuda()

    def draw(self, heads):
        x = self.rng.standard_normal((self.spec.batch, heads, self.spec.head_dim), dtype=np.float32)
        return W.f32_to_bf16_bits(x) if self.spec.dtype == "bf16" else x

    def step(self):
        self.fea.fea_kv_extend(self.pool, self.bt, self.lens)
        kn, vn = self.draw(self.spec.num_kv_heads), self.draw(self.spec.num_kv_heads)
        oappend.append(self.hk, self.hv, kn, vn, self.bt, self.lens)
        self.sync_tables()
        self.fea.fea_kv_append(self.p, self.to_device(kn), self.to_device(vn), self.dk, self.dv, self.dbt, self.dl)

    def attend(self, flags):
        """-> (query as drawn, device output) of one attention call with the given plan flags"""
        qn = self.draw(self.spec.num_q_heads)
        dq = self.to_device(qn)
        out = self.torch.full_like(dq, float("nan"))
        self.fea.fea_decode_attention(self.params(flags), dq, self.dk, self.dv, self.dbt, self.dl, out, self.ws)
        self.torch.cuda.synchronize()
        return qn, out

    def oracle(self, qn):
        from gpu_harness import values
        return decode_attention(values(qn), values(self.hk), values(self.hv), self.bt, self.lens)


LOOP_SPECS = {
    "c2": lambda: W.scaled(W.CONFIGS["c2"], batch_div=8, len_div=8),
    "c3": lambda: W.scaled(W.CONFIGS["c3"], batch_div=8, len_div=8),
    "c5": lambda: W.scaled(W.CONFIGS["c5"], batch_div=16, len_div=4),
    # 40 requests of one 2048-token prefix (row tiles swept by teams of waves), 3 more of another, 5 on their own,
    # suffixes of 1..40 tokens: many requests cross a block boundary on every step
    "teams_and_singles": lambda: W.Spec("loop_mix", 77, "bf16", 32, 8, 128, ((40, 2048), (3, 160), (1, 0), (1, 0), (1, 0), (1, 0), (1, 0)), (1, 40)),
    "f32_generic": lambda: W.Spec("loop_f32", 78, "f32", 8, 2, 64, ((6, 96), (1, 0), (1, 0)), (1, 33)),
}


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(LOOP_SPECS))
def test_one_plan_stretched_over_many_decode_steps(name):
    """FEA_FLAG_REFRESH_PLAN: the plan made at one decode step serves the following ones (every request one token
    longer per step, new table columns where a block filled up) - alias detection and work split are kept, the last
    piece of every request follows its length.  Every step attends; every third one, and each one after a new plan,
    is set against the oracle; the refreshed plan keeps the items of the plan it came from."""
    import paper_2605_06046_amd as fea
    from gpu_harness import assert_close
    steps = 40
    lp = _Loop(LOOP_SPECS[name](), steps)
    items = None
    for step in range(steps):
        lp.step()
        fresh = step in (0, 26)
        qn, out = lp.attend(0 if fresh else fea.FEA_FLAG_REFRESH_PLAN)
        info = fea.fea_decode_plan_info(lp.ws)
        assert info["overflow"] == 0
        if fresh:
            items = info["items"]
        assert info["items"] == items
        if fresh or step % 3 == 2 or step == steps - 1:
            assert_close(out.float().cpu().numpy().astype(np.float64), lp.oracle(qn), lp.spec.dtype, what=f"{name} step {step}")
    # the same plan used unrefreshed on the grown batch misses the new tokens: the refresh does change the result
    if name != "c5":
        qn, out_stale = lp.attend(fea.FEA_FLAG_REUSE_PLAN)
        lp.step(); lp.step()
        q2 = lp.draw(lp.spec.num_q_heads)
        dq = lp.to_device(q2)
        outs = []
        for flags in (fea.FEA_FLAG_REUSE_PLAN, fea.FEA_FLAG_REFRESH_PLAN):
            o = lp.torch.empty_like(dq)
            fea.fea_decode_attention(lp.params(flags), dq, lp.dk, lp.dv, lp.dbt, lp.dl, o, lp.ws)
            outs.append(o.float().cpu().numpy().astype(np.float64))
        assert_close(outs[1], lp.oracle(q2), lp.spec.dtype, what=f"{name} after two more steps")
        assert not np.allclose(outs[0], outs[1], rtol=0, atol=1e-6)


@pytest.mark.gpu
def test_refresh_reports_a_request_it_cannot_stretch():
    """Requests whose every block is shared have no piece of their own to stretch: once they have grown, a refreshed
    plan says so (overflow flag 2, NaN in every row) rather than leaving the new tokens out; a new plan is right."""
    import paper_2605_06046_amd as fea
    from gpu_harness import assert_close
    lp = _Loop(W.Spec("allshared", 5, "bf16", 8, 2, 128, ((4, 64),), (0, 0)), 4)
    qn, out = lp.attend(0)
    assert fea.fea_decode_plan_info(lp.ws)["overflow"] == 0
    assert_close(out.float().cpu().numpy().astype(np.float64), lp.oracle(qn), "bf16", what="all shared")
    qn, out = lp.attend(fea.FEA_FLAG_REFRESH_PLAN)          # nothing has grown: still fine
    assert fea.fea_decode_plan_info(lp.ws)["overflow"] == 0
    assert_close(out.float().cpu().numpy().astype(np.float64), lp.oracle(qn), "bf16", what="all shared, refreshed")
    lp.step()
    qn, out = lp.attend(fea.FEA_FLAG_REFRESH_PLAN)
    assert fea.fea_decode_plan_info(lp.ws)["overflow"] == 2
    assert lp.torch.isnan(out.float()).all()
    qn, out = lp.attend(0)
    assert fea.fea_decode_plan_info(lp.ws)["overflow"] == 0
    assert_close(out.float().cpu().numpy().astype(np.float64), lp.oracle(qn), "bf16", what="all shared, planned anew")
    lp.step()
    qn, out = lp.attend(fea.FEA_FLAG_REFRESH_PLAN)          # now every request has a block of its own
    assert fea.fea_decode_plan_info(lp.ws)["overflow"] == 0
    assert_close(out.float().cpu().numpy().astype(np.float64), lp.oracle(qn), "bf16", what="all shared, grown twice")


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["f32_generic", "allshared", "c2_tiny"])
def test_small_batches_in_one_launch_over_decode_steps(name):
    """Batches within the one-launch bound need no plan: whatever plan flag the loop passes, every step is right and
    the workspace says that no plan was used (variant 2).  FEA_FLAG_PLAN_ONLY still makes the plan."""
    import paper_2605_06046_amd as fea
    from gpu_harness import assert_close
    spec = {"f32_generic": LOOP_SPECS["f32_generic"],
            "allshared": lambda: W.Spec("allshared", 5, "bf16", 8, 2, 128, ((4, 64),), (0, 0)),
            "c2_tiny": lambda: W.scaled(W.CONFIGS["c2"], batch_div=16, len_div=16)}[name]()
    steps = 20
    lp = _Loop(spec, steps, fused_max=0)
    for step in range(steps):
        lp.step()
        flags = (0, fea.FEA_FLAG_REFRESH_PLAN, fea.FEA_FLAG_REUSE_PLAN)[step % 3]
        qn, out = lp.attend(flags)
        info = fea.fea_decode_plan_info(lp.ws)
        assert info["variant"] == 2 and info["items"] == 0 and info["groups"] == 0 and info["overflow"] == 0
        assert_close(out.float().cpu().numpy().astype(np.float64), lp.oracle(qn), lp.spec.dtype, what=f"{name} step {step}")
    lp.attend(fea.FEA_FLAG_PLAN_ONLY)
    info = fea.fea_decode_plan_info(lp.ws)
    assert info["variant"] in (0, 1) and info["items"] > 0 and info["groups"] >= 1


def dataclass_replace(obj, **kw):
    import dataclasses
    return dataclasses.replace(obj, **kw)
