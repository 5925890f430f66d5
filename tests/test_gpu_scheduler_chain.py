"""The whole chain on the device side of the boundary against the same chain in the oracle:
Chunked Hash Tree batch formation (rule-based and learned stop policies, Section 4.2 / 4.3 and the
appendix "Batch Formation") -> block tables with prefix aliasing -> decode attention.

256 requests with the structure of the eight-group batch (8 prefix groups x 32, arriving
interleaved) at a sixteenth of its lengths: the by-definition tree oracle recomputes every set on
every query, which bounds the size it finishes in seconds.  Batch membership must be equal,
tables bit-exact, attention within the bf16 tolerance, for every batch until the queue is empty.
The reward handed to the learned policies is a stand-in computed from the tables (requests per
distinct block), the same number on both sides: what a policy learns is not under test here, that
both sides take the same decisions from the same history is."""
import numpy as np
import pytest

import workloads as W
from gpu_harness import assert_close, run_hip, values
from oracle.attention import decode_attention
from oracle.block_tables import build_block_tables
from oracle.cht import ChunkedHashTree, build_batch
from oracle.policy import QLearner, UcbBandit, build_batch_learned

pytestmark = pytest.mark.gpu

RULE = dict(small_batch=2, loss_small=1 << 30, loss_limit=4, peers_relax=8, loss_relaxed=12)
BINS = dict(b_bins=8, w_bins=8, loss_thresholds=(0, 2, 8))
MAX_BATCH = 32


@pytest.mark.parametrize("kind", ["rule_based", "bandit", "q_learning"])
def test_scheduler_tables_attention_chain(kind):
    import paper_2605_06046_amd as fea
    spec = W.scaled(W.CONFIGS["c3"], batch_div=1, len_div=16, name="c3_chain")
    wl = W.generate(spec)
    B = spec.batch
    reqs = [wl.request_tokens(i) for i in range(B)]
    o_tree, l_tree = ChunkedHashTree(), fea.Cht()
    for i, r in enumerate(reqs):
        o_tree.insert(i, tokens=r)
        l_tree.insert(i, tokens=r)
    o_pol = l_pol = None
    if kind == "bandit":
        o_pol = UcbBandit(c=0.5)
        l_pol = fea.Policy(fea.FEA_POLICY_UCB, c=0.5, **BINS)
    elif kind == "q_learning":
        o_pol = QLearner(alpha=0.5, gamma=0.9, eps=0.4, eps_min=0.05, eps_decay=0.8)
        l_pol = fea.Policy(fea.FEA_POLICY_QLEARN, alpha=0.5, gamma=0.9, eps=0.4, eps_min=0.05, eps_decay=0.8, **BINS)
    rng = np.random.default_rng(12)
    s = wl.spec
    served, n_batches, mixes = 0, 0, []
    while o_tree.waiting:
        draws = rng.random((MAX_BATCH, 2))
        if kind == "rule_based":
            want_ids = build_batch(o_tree, MAX_BATCH, **RULE)
            ids = l_tree.build_batch(MAX_BATCH, **RULE)
        else:
            want_ids = build_batch_learned(o_tree, o_pol, MAX_BATCH, [tuple(d) for d in draws], **BINS)
            ids = l_tree.build_batch_learned(l_pol, MAX_BATCH, draws)
        assert ids == want_ids, f"batch {n_batches}: membership differs"
        if not ids:                                    # a learned policy stopped at once: serve the best candidate alone
            best = o_tree.find_best()
            assert l_tree.find_best() == best
            o_tree.add_to_batch(best[0]); l_tree.add_to_batch(best[0])
            ids = [best[0]]
        seqs = [reqs[i] for i in ids]
        toks = np.concatenate(seqs)
        offs = np.zeros(len(ids) + 1, dtype=np.int64)
        offs[1:] = np.cumsum([len(x) for x in seqs])
        pool = fea.fea_kv_alloc(wl.num_blocks, 16, 0)
        bt, lens, _, _ = fea.fea_build_block_tables(pool, toks, offs, wl.max_blocks_per_seq)
        obt, olens, _ = build_block_tables(seqs, wl.num_blocks, 0, wl.max_blocks_per_seq)
        assert np.array_equal(bt, obt) and np.array_equal(lens, olens), f"batch {n_batches}: tables differ"
        q = wl.q[np.array(ids)]
        out, info = run_hip(q, wl.k_cache, wl.v_cache, bt, lens, s.num_q_heads, s.num_kv_heads, s.head_dim, s.dtype)
        want = decode_attention(values(q), values(wl.k_cache), values(wl.v_cache), bt, lens)
        assert_close(out, want, "bf16", what=f"{kind} batch {n_batches}")
        reward = len(ids) / max(1, len(np.unique(bt[bt >= 0]))) * 100.0
        if o_pol is not None:
            o_pol.reward(reward)
            l_pol.reward(reward)
        for rid in ids:
            o_tree.finish(rid)
            l_tree.finish(rid)
        served += len(ids)
        n_batches += 1
        mixes.append(len({int(wl.group_of[i]) for i in ids}))
    assert served == B and l_tree.stats()["waiting"] == 0 and l_tree.stats()["active"] == 0
    print(kind, "batches", n_batches, "mean prefix groups per batch", float(np.mean(mixes)))
    if kind == "rule_based":
        assert n_batches == 8 and max(mixes) == 1       # the tree forms one batch per prefix group
