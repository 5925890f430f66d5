"""fea_decode_attention_static (the entry point that allocates nothing) against
fea_decode_attention on the same inputs: bit for bit, two calls in a row, the second on
a smaller batch (the built-in workspace still holds the first call's plan and partials)."""
import numpy as np
import pytest

import workloads as W
from gpu_harness import assert_close, library_tables, oracle_for, to_device

pytestmark = pytest.mark.gpu


def _both(wl, bt, lens, fused_max=-1):
    import torch
    import paper_2605_06046_amd as fea
    s = wl.spec
    p = fea.AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim,
                       fea.FEA_DTYPE_BF16 if s.dtype == "bf16" else fea.FEA_DTYPE_F32, fused_max=fused_max)
    q, k, v = to_device(wl.q), to_device(wl.k_cache), to_device(wl.v_cache)
    dbt, dl = torch.from_numpy(bt).cuda(), torch.from_numpy(lens).cuda()
    ws = torch.empty(fea.fea_decode_workspace_bytes(p, s.batch, bt.shape[1]), dtype=torch.uint8, device="cuda")
    ref = torch.full_like(q, float("nan"))
    got = torch.full_like(q, float("nan"))
    fea.fea_decode_attention(p, q, k, v, dbt, dl, ref, ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    fea.fea_decode_attention_static(p, q, k, v, dbt, dl, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref, got


def test_static_workspace_entry_point_equals_the_workspace_one():
    import torch
    import paper_2605_06046_amd as fea
    # first call: a batch with a shared prefix and ragged tails (several tiles per item, a group, private pieces)
    big = W.generate(W.scaled(W.CONFIGS["c3"], batch_div=4, len_div=4, name="c3_static"))
    bt, lens = library_tables(big)
    W.poison_dead_slots(big, bt, lens)
    ref, got = _both(big, bt, lens)
    assert torch.equal(ref, got)
    assert_close(got.float().cpu().numpy().astype(np.float64), oracle_for(big, bt, lens), "bf16", what="static, first call")
    # second call, smaller: fewer requests, shorter tables, another dtype and head shape
    small = W.generate(W.CONFIGS["c1"])
    bt2, lens2 = library_tables(small)
    W.poison_dead_slots(small, bt2, lens2)
    ref2, got2 = _both(small, bt2, lens2)
    assert torch.equal(ref2, got2)
    assert_close(got2.float().cpu().numpy().astype(np.float64), oracle_for(small, bt2, lens2), "f32", what="static, second call")
    # the small batch as the library takes it by default (one launch, nothing kept in the buffer but a header)
    ref2f, got2f = _both(small, bt2, lens2, fused_max=0)
    assert torch.equal(ref2f, got2f)
    assert_close(got2f.float().cpu().numpy().astype(np.float64), oracle_for(small, bt2, lens2), "f32", what="static, one launch")
    # and the first batch again after the small one
    ref3, got3 = _both(big, bt, lens)
    assert torch.equal(ref3, got3) and torch.equal(ref3, ref)


def test_static_workspace_entry_point_refuses_what_it_cannot_hold():
    import torch
    import paper_2605_06046_amd as fea
    s = W.CONFIGS["c5"]
    p = fea.AttnParams(s.num_q_heads, s.num_kv_heads, s.head_dim, fea.FEA_DTYPE_BF16)
    B, stride = 512, 256
    assert fea.fea_decode_workspace_bytes(p, B, stride) > (48 << 20)
    q = torch.zeros((B, s.num_q_heads, s.head_dim), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((4, s.num_kv_heads, 16, s.head_dim), dtype=torch.bfloat16, device="cuda")
    bt = torch.zeros((B, stride), dtype=torch.int32, device="cuda")
    lens = torch.zeros(B, dtype=torch.int32, device="cuda")
    out = torch.full_like(q, 7.0)
    with pytest.raises(fea.FeaError) as ei:
        fea.fea_decode_attention_static(p, q, kv, kv, bt, lens, out)
    assert ei.value.code == -3
    torch.cuda.synchronize()
    assert (out == 7.0).all()                      # nothing was launched
    for flag in (fea.FEA_FLAG_REUSE_PLAN, fea.FEA_FLAG_PLAN_ONLY):
        p2 = fea.AttnParams(8, 2, 64, fea.FEA_DTYPE_F32, flags=flag)
        with pytest.raises(fea.FeaError) as ei:
            fea.fea_decode_attention_static(p2, q[:4, :8, :64].contiguous().float(), kv.float()[:, :2, :, :64].contiguous(),
                                            kv.float()[:, :2, :, :64].contiguous(), bt[:4, :20].contiguous(), lens[:4], out[:4, :8, :64].contiguous().float())
        assert ei.value.code == -1
    # B == 0 is a no-op
    fea.fea_decode_attention_static(p, q[:0], kv, kv, bt[:0], lens[:0], out[:0])
