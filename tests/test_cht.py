"""Chunked Hash Tree: the oracle against what the paper states, then the library against the oracle.

Pins of the oracle (nothing here is derived from the oracle itself):
  * the walk-through of Section 4.2 (requests as hash vectors over tokens A-F with K = 2: tip after the
    first addition, the candidate FindBest returns, the tip dropping by one level, the tip extending to
    the remaining request's last level when the first completes);
  * the R1..R4 example of the appendix "Find Best Request - Alternative Heuristic";
  * the four (m_W, m_S) values in the caption of the two-case figure of the same appendix;
  * the appendix's theorem: among equally long requests, the one minimising the working-set metric also
    minimises the tip metric (random trees).
"""
import random

import numpy as np
import pytest

from oracle.cht import ChunkedHashTree, build_batch
from oracle.hashing import chunk_hashes


def vec(*path):
    """A hash vector for a path of chunk labels: cumulative by construction (one value per prefix)."""
    return [hash(tuple(path[:i + 1])) & ((1 << 64) - 1) for i in range(len(path))]


def test_walkthrough_of_section_4_2():
    t = ChunkedHashTree(chunk_tokens=2)
    A, B, Cc, D, E, F, G, H, X, Y = range(10)
    t.insert(1, tokens=[A, B, Cc, D, E, F])          # three chunks: hash(A-B), hash(A-D), hash(A-F)
    t.insert(2, tokens=[A, B, Cc, D, G, H])          # shares two levels with R1
    t.insert(3, tokens=[A, B, X, Y, G, H])           # shares one
    assert len(t.hashes[1]) == 3
    t.add_to_batch(1)
    assert t.tip() == (3, t.hashes[1][2])            # a single active request: the tip is its last level
    assert len(t.working_set()) == 3                 # R1's nodes are the working set
    assert (t.missing(2), t.missing(3)) == (1, 2)
    rid, before, after, peers, miss = t.find_best()
    assert (rid, before, after, miss) == (2, 3, 2, 1)   # R2 on top of the heap; adding it costs one level
    assert peers == 1                                # only R2 itself carries hash(A-D) among the waiting
    t.add_to_batch(2)
    assert t.tip()[0] == 2
    t.finish(1)
    assert t.tip() == (3, t.hashes[2][2])            # the tip extends to R2's final level


def test_r1_to_r4_example_of_the_appendix():
    t = ChunkedHashTree()
    t.insert(1, hash_vector=vec("root", "a"))
    t.insert(2, hash_vector=vec("root", "b"))
    t.insert(3, hash_vector=vec("root", "b"))
    t.insert(4, hash_vector=vec("root", "c"))
    t.add_to_batch(1)
    t.add_to_batch(2)
    assert t.tip()[0] == 1                           # restricted to level 1
    assert t.missing(3) < t.missing(4)               # R3 needs fewer missing chunks than R4
    assert t.find_best()[0] == 3
    # admitting R4 instead would leave the tip stuck once R1 finishes; admitting R3 lets it extend
    import copy
    alt = copy.deepcopy(t)
    alt.add_to_batch(4); alt.finish(1)
    assert alt.tip()[0] == 1
    t.add_to_batch(3); t.finish(1)
    assert t.tip()[0] == 2


@pytest.mark.parametrize("case,rw,rs,want", [
    (1, ("1", "2", "x3", "x4"), ("1", "2", "3", "y4"), dict(mw_w=2, mw_s=1, ms_w=1, ms_s=0)),
    (2, ("1", "x2", "x3", "x4"), ("1", "2", "y3", "y4"), dict(mw_w=3, mw_s=2, ms_w=2, ms_s=1)),
])
def test_caption_values_of_the_two_case_figure(case, rw, rs, want):
    # r1 and r2 active, tip at the third level; r_W and r_S as the caption describes them
    t = ChunkedHashTree()
    t.insert(1, hash_vector=vec("1", "2", "3", "a4"))
    t.insert(2, hash_vector=vec("1", "2", "3", "b4"))
    t.insert(10, hash_vector=vec(*rw))
    t.insert(11, hash_vector=vec(*rs))
    t.add_to_batch(1); t.add_to_batch(2)
    assert t.tip()[0] == 3
    got = dict(mw_w=t.missing(10), mw_s=t.missing(11), ms_w=t.missing_from_tip(10), ms_s=t.missing_from_tip(11))
    assert got == want


def random_tree_requests(rng, n, depth, branching):
    out = []
    for _ in range(n):
        path = [rng.randrange(branching if l else 1) for l in range(depth)]
        # cumulative: once two paths diverge they stay apart (vec hashes whole prefixes)
        out.append(vec(*path))
    return out


@pytest.mark.parametrize("seed", range(20))
def test_minimising_the_working_set_metric_also_minimises_the_tip_metric(seed):
    rng = random.Random(seed)
    reqs = random_tree_requests(rng, 14, depth=5, branching=2)
    t = ChunkedHashTree()
    for i, h in enumerate(reqs):
        t.insert(i, hash_vector=h)
    for i in rng.sample(range(14), 3):
        t.add_to_batch(i)
    best = t.find_best()[0]
    assert t.missing_from_tip(best) == min(t.missing_from_tip(w) for w in t.waiting)


# ---------------------------------------------------------------- the library against the oracle
def lib_tree():
    from paper_2605_06046_amd import Cht
    return Cht()


def token_requests(rng, n):
    """Token sequences with nested shared prefixes of whole and partial chunks."""
    roots = [[rng.randrange(32000) for _ in range(rng.choice([16, 48, 160, 200]))] for _ in range(3)]
    out = []
    for _ in range(n):
        r = list(rng.choice(roots))
        if rng.random() < 0.5:
            r = r[:rng.randrange(1, len(r) + 1)]
        r += [rng.randrange(32000) for _ in range(rng.choice([0, 1, 15, 16, 17, 40]))]
        out.append(r)
    return out


@pytest.mark.parametrize("seed", range(12))
def test_library_follows_the_oracle_through_random_operation_sequences(seed):
    rng = random.Random(1000 + seed)
    reqs = token_requests(rng, 40)
    o, l = ChunkedHashTree(), lib_tree()
    next_id, waiting, active = 0, [], []
    for step in range(300):
        op = rng.random()
        if (op < 0.35 and next_id < len(reqs)) or (not waiting and not active and next_id < len(reqs)):
            rid = next_id if seed % 2 == 0 else 1000 - next_id      # ids need not be dense or increasing
            o.insert(rid, tokens=reqs[next_id]); l.insert(rid, tokens=reqs[next_id])
            waiting.append(rid); next_id += 1
        elif op < 0.65 and waiting:
            want = o.find_best()
            assert l.find_best() == want
            assert l.find_best() == want                            # cached answer
            o.add_to_batch(want[0]); l.add_to_batch(want[0])
            waiting.remove(want[0]); active.append(want[0])
        elif op < 0.9 and active:
            rid = rng.choice(active)
            o.finish(rid); l.finish(rid); active.remove(rid)
        elif waiting:
            rid = rng.choice(waiting)
            o.remove(rid); l.remove(rid); waiting.remove(rid)
        st = l.stats()
        tip = o.tip()
        assert (st["waiting"], st["active"], st["tip_level"]) == (len(o.waiting), len(o.active), tip[0])
        assert st["tip_hash"] == (tip[1] or 0)
        assert st["working_set"] == len(o.working_set())
        for w in waiting:
            assert l.missing(w) == o.missing(w)
        assert l.find_best() == o.find_best()


def test_library_hash_vectors_and_errors():
    from paper_2605_06046_amd import FeaError
    l = lib_tree()
    toks = list(range(100, 150))
    l.insert(7, tokens=toks)
    o = ChunkedHashTree(); o.insert(7, hash_vector=chunk_hashes(toks, 16))
    l.insert(8, hash_vector=np.array(o.hashes[7][:2], dtype=np.uint64))   # a prefix of request 7, given as hashes
    l.add_to_batch(7)
    assert l.missing(8) == 0 and l.stats()["tip_level"] == 4
    with pytest.raises(FeaError):
        l.insert(7, tokens=toks)          # duplicate id
    with pytest.raises(FeaError):
        l.add_to_batch(7)                 # already active
    with pytest.raises(FeaError):
        l.finish(8)                       # not active
    with pytest.raises(FeaError):
        l.remove(99)
    l.finish(7); l.remove(8)
    assert l.find_best() is None and l.stats()["working_set"] == 0


@pytest.mark.parametrize("seed", range(6))
def test_build_batch_matches_the_oracle_loop(seed):
    rng = random.Random(50 + seed)
    reqs = token_requests(rng, 30)
    pol = dict(small_batch=rng.choice([1, 2, 4]), loss_small=rng.choice([2, 100]), loss_limit=rng.choice([0, 1, 3]),
               peers_relax=rng.choice([2, 5]), loss_relaxed=rng.choice([2, 6]))
    o, l = ChunkedHashTree(), lib_tree()
    for i, r in enumerate(reqs):
        o.insert(i, tokens=r); l.insert(i, tokens=r)
    for rounds in range(4):
        want = build_batch(o, 8, **pol)
        assert l.build_batch(8, **pol) == want
        for rid in want[: len(want) // 2 + 1]:
            o.finish(rid); l.finish(rid)
