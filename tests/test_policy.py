"""Learned stop policies (Section 4.3): the oracle against worked values and known bounds, then the
library against the oracle.

Pins of the oracle (values worked by hand from the two update rules, a table of bins written out, and
the regret argument of the UCB rule; nothing is computed by the oracle itself):
  * bins: 0 | 1 | 2-3 | 4-7 | ... with a cap; thresholds counted;
  * UCB with mu = (8, 3), n = (4, 1), S = 5, c = 1: 2 + sqrt(ln 5 / 4) and 3 + sqrt(ln 5);
  * UCB's bound on the pulls of a worse arm with deterministic rewards: while that arm is still taken
    its index is at least the better arm's mean, so n <= c^2 ln S / gap^2 + 1;
  * Q-learning: two passes over a three-step episode with alpha = 1/2, gamma = 0.9, r = 2 give 1, 1, 1
    then 1.95, 1.95, 1.5; with the reward on the last transition only 0, 0, 1 then 0, 0.45, 1.5; with
    alpha = 1 the table reaches r (1 + gamma + gamma^2) = 5.42 at the first state in three passes;
  * epsilon: 1 -> 0.5 -> 0.25 -> 0.125 -> floor 0.1.
"""
import math
import random

import numpy as np
import pytest

from oracle.cht import ChunkedHashTree
from oracle.policy import ADD, STOP, QLearner, UcbBandit, build_batch_learned, discretize, exp_bin

BINS = dict(b_bins=10, w_bins=10, loss_thresholds=(0, 2, 8))


def test_bins_written_out():
    want = {0: 0, 1: 1, 2: 2, 3: 2, 4: 3, 7: 3, 8: 4, 15: 4, 16: 5, 255: 8, 256: 9, 500: 9, 100000: 9}
    for x, b in want.items():
        assert exp_bin(x, 10) == b, x
    assert exp_bin(500, 6) == 5 and exp_bin(-3, 6) == 0
    assert [discretize(0, d, 0, **BINS)[1] for d in (-1, 0, 1, 2, 3, 8, 9, 1000)] == [0, 0, 1, 1, 2, 2, 3, 3]
    assert discretize(5, 3, 40, **BINS) == (3, 2, 6)


def test_ucb_worked_values():
    p = UcbBandit(c=1.0)
    s = (1, 0, 2)
    assert p.decide(s) == ADD and p.episode == [(s, ADD)]       # nothing tried: ADD first
    p.episode = []
    p.mu = {(s, ADD): 8.0, (s, STOP): 3.0}
    p.n = {(s, ADD): 4, (s, STOP): 1}
    p.S = 5
    assert p.ucb(s, ADD) == pytest.approx(2.63431812058976, abs=1e-12)
    assert p.ucb(s, STOP) == pytest.approx(4.26863624117952, abs=1e-12)
    assert p.decide(s) == STOP
    p.reward(1.0)
    assert p.n[(s, STOP)] == 2 and p.mu[(s, STOP)] == 4.0 and p.S == 6
    other = (2, 0, 2)
    assert p.decide(other) == ADD                               # states do not share statistics
    p.reward(0.0)
    assert p.decide(other) == STOP                              # the untried action comes next


@pytest.mark.parametrize("c", [0.5, 1.0, math.sqrt(2.0)])
def test_ucb_pulls_of_the_worse_arm_stay_within_the_bound(c):
    p = UcbBandit(c=c)
    s = (0, 0, 0)
    reward = {ADD: 0.5, STOP: 1.0}
    for _ in range(3000):
        a = p.decide(s)
        p.reward(reward[a])
    worse = p.n[(s, ADD)]
    assert 2 <= worse <= c * c * math.log(p.S) / 0.25 + 1
    assert p.n[(s, ADD)] + p.n[(s, STOP)] == p.S == 3000


def test_ucb_without_exploration_is_greedy():
    p = UcbBandit(c=0.0)
    s = (0, 0, 0)
    seen = []
    for r in (0.3, 0.7, 0.1, 0.1):
        seen.append(p.decide(s))
        p.reward(r)
    assert seen == [ADD, STOP, STOP, STOP]                      # each once, then the better mean (0.7, then 0.4)


def test_bandit_credits_every_decision_of_the_episode():
    p = UcbBandit(c=1.0)
    a0 = p.decide((0, 0, 1)); a1 = p.decide((1, 0, 1)); a2 = p.decide((2, 1, 1))
    p.reward(2.5)
    assert (a0, a1, a2) == (ADD, ADD, ADD) and p.S == 3
    for s in ((0, 0, 1), (1, 0, 1), (2, 1, 1)):
        assert p.value(s, ADD) == (2.5, 1) and p.value(s, STOP) == (0.0, 0)


def run_episode(q, steps, r):
    for s, a in steps:
        # force the action: explore with certainty, u_action picks it
        eps, q.eps = q.eps, 1.0
        assert q.decide(s, 0.0, 0.0 if a == ADD else 0.9) == a
        q.eps = eps
    q.reward(r)


def test_q_learning_worked_values():
    steps = [("s0", ADD), ("s1", ADD), ("s2", STOP)]
    q = QLearner(alpha=0.5, gamma=0.9, eps=0.0, eps_min=0.0, eps_decay=1.0, reward_every_step=True)
    run_episode(q, steps, 2.0)
    assert [q.q(*k) for k in steps] == [1.0, 1.0, 1.0]
    run_episode(q, steps, 2.0)
    assert [q.q(*k) for k in steps] == pytest.approx([1.95, 1.95, 1.5], abs=1e-15)
    assert q.q("s0", STOP) == 0.0 and q.value("s2", STOP) == (1.5, 2)

    q = QLearner(alpha=0.5, gamma=0.9, eps=0.0, eps_min=0.0, eps_decay=1.0, reward_every_step=False)
    run_episode(q, steps, 2.0)
    assert [q.q(*k) for k in steps] == [0.0, 0.0, 1.0]
    run_episode(q, steps, 2.0)
    assert [q.q(*k) for k in steps] == pytest.approx([0.0, 0.45, 1.5], abs=1e-15)


def test_q_learning_reaches_the_bellman_fixed_point():
    steps = [("s0", ADD), ("s1", ADD), ("s2", STOP)]
    q = QLearner(alpha=1.0, gamma=0.9, eps=0.0, eps_min=0.0, eps_decay=1.0)
    for _ in range(3):
        run_episode(q, steps, 2.0)
    assert [q.q(*k) for k in steps] == pytest.approx([5.42, 3.8, 2.0], abs=1e-12)
    for _ in range(5):
        run_episode(q, steps, 2.0)                              # a fixed point: nothing moves any more
    assert [q.q(*k) for k in steps] == pytest.approx([5.42, 3.8, 2.0], abs=1e-12)


def test_q_learning_bootstraps_from_the_better_action_of_the_next_state():
    q = QLearner(alpha=1.0, gamma=0.5, eps=0.0, eps_min=0.0, eps_decay=1.0)
    q.Q[("s1", STOP)] = 6.0
    q.Q[("s1", ADD)] = 1.0
    run_episode(q, [("s0", ADD), ("s1", ADD)], 1.0)
    assert q.q("s0", ADD) == 1.0 + 0.5 * 6.0                    # max over the next state's actions, not the one taken
    assert q.q("s1", ADD) == 1.0                                # last transition: no future


def test_epsilon_greedy_and_decay():
    q = QLearner(alpha=0.5, gamma=0.9, eps=1.0, eps_min=0.1, eps_decay=0.5)
    assert q.decide("s", 0.99, 0.2) == ADD and q.decide("s", 0.99, 0.7) == STOP   # exploring: u_action decides
    q.episode = []
    seen = []
    for _ in range(5):
        q.decide("s", 0.0, 0.0)
        q.reward(1.0)
        seen.append(q.eps)
    assert seen == [0.5, 0.25, 0.125, 0.1, 0.1]
    q.Q = {("s", ADD): 1.0, ("s", STOP): 2.0}
    assert q.decide("s", 0.5, 0.0) == STOP                      # 0.5 >= eps: greedy
    assert q.decide("s", 0.05, 0.0) == ADD                      # 0.05 < eps: explores
    q.Q[("s", ADD)] = 2.0
    assert q.decide("s", 0.5, 0.9) == ADD                       # greedy tie: ADD


class Scripted:
    def __init__(self, actions):
        self.actions, self.states = list(actions), []

    def decide(self, s, u1, u2):
        self.states.append(s)
        return self.actions.pop(0)


def test_build_batch_forms_the_state_from_find_best():
    t = ChunkedHashTree()
    # two levels shared by 1, 2, 3; request 4 shares one level; request 5 nothing
    t.insert(1, hash_vector=[10, 20, 31])
    t.insert(2, hash_vector=[10, 20, 32])
    t.insert(3, hash_vector=[10, 20, 33])
    t.insert(4, hash_vector=[10, 24, 34])
    t.insert(5, hash_vector=[15, 25, 35])
    pol = Scripted([ADD, ADD, ADD, ADD, STOP])
    draws = [(0.0, 0.0)] * 8
    batch = build_batch_learned(t, pol, 8, draws, **BINS)
    assert batch == [1, 2, 3, 4]
    # b: 0,1,2,3,4 -> bins 0,1,2,2,3.  Losses: none on an empty batch; 3 -> 2 (one level) when the second
    # joins; 0 for the third; 2 -> 1 for request 4; 1 -> 0 for request 5.  Peers at the new depth: all 5
    # waiting at depth 0; 2 and 3 carry hash 20 (2 waiting); then 3 alone; 4 alone at level 1; 5 at depth 0.
    assert pol.states == [(0, 0, exp_bin(5, 10)), (1, 1, exp_bin(2, 10)), (2, 0, 1), (2, 1, 1), (3, 1, 1)]
    assert sorted(t.waiting) == [5] and t.active == [1, 2, 3, 4]
    # the cap ends the episode without a STOP decision
    t2 = ChunkedHashTree()
    for i in range(4):
        t2.insert(i, hash_vector=[7, 100 + i])
    pol2 = Scripted([ADD] * 4)
    assert build_batch_learned(t2, pol2, 2, draws, **BINS) == [0, 1] and len(pol2.states) == 2


# ----------------------------------------------------------------- the library against the oracle

fea = pytest.importorskip("paper_2605_06046_amd")


def make_pair(kind, **kw):
    if kind == "ucb":
        lib = fea.Policy(fea.FEA_POLICY_UCB, BINS["b_bins"], BINS["w_bins"], BINS["loss_thresholds"], c=kw["c"])
        ora = UcbBandit(c=kw["c"])
    else:
        lib = fea.Policy(fea.FEA_POLICY_QLEARN, BINS["b_bins"], BINS["w_bins"], BINS["loss_thresholds"], **kw)
        ora = QLearner(**kw)
    return lib, ora


def same_tables(lib, ora, states):
    for s in states:
        for a in (ADD, STOP):
            lv, ln = lib.entry(s, a)
            ov, on = ora.value(s, a)
            assert ln == on, (s, a)
            assert lv == pytest.approx(ov, rel=1e-13, abs=1e-13), (s, a)


def test_library_bins_match():
    lib, _ = make_pair("ucb", c=1.0)
    rng = random.Random(5)
    cases = [(0, 0, 0), (1, -1, 1), (500, 9, 100000), (2 ** 31 - 1, 2 ** 31 - 1, 2 ** 31 - 1)]
    cases += [(rng.randrange(0, 600), rng.randrange(-2, 40), rng.randrange(0, 3000)) for _ in range(300)]
    for b, d, w in cases:
        assert lib.state(b, d, w) == discretize(b, d, w, **BINS)


@pytest.mark.parametrize("kind,kw", [
    ("ucb", dict(c=1.0)), ("ucb", dict(c=0.0)), ("ucb", dict(c=2.5)),
    ("q", dict(alpha=0.3, gamma=0.9, eps=1.0, eps_min=0.05, eps_decay=0.97, reward_every_step=True)),
    ("q", dict(alpha=1.0, gamma=0.5, eps=0.5, eps_min=0.0, eps_decay=0.9, reward_every_step=False)),
])
def test_library_policy_follows_the_oracle(kind, kw):
    lib, ora = make_pair(kind, **kw)
    rng = random.Random(11)
    seen = set()
    for ep in range(400):
        b = 0
        for _ in range(rng.randrange(0, 12)):
            loss, peers = rng.choice([0, 0, 1, 2, 3, 9, 20]), rng.randrange(0, 70)
            u1, u2 = rng.random(), rng.random()
            s = discretize(b, loss, peers, **BINS)
            seen.add(s)
            a = lib.decide(b, loss, peers, u1, u2)
            assert a == ora.decide(s, u1, u2), (ep, b)
            if a == STOP:
                break
            b += 1
        assert lib.info()["open"] == len(ora.episode)
        r = rng.choice([0.25, 0.5, 1.0, 1.5]) * (1.0 + 0.1 * rng.random())
        lib.reward(r)
        ora.reward(r)
        if ep % 50 == 0:
            same_tables(lib, ora, seen)
    same_tables(lib, ora, seen)
    info = lib.info()
    assert info["episodes"] == 400 and info["open"] == 0
    if kind == "ucb":
        assert info["decisions"] == ora.S
    else:
        assert info["eps"] == pytest.approx(ora.eps, rel=1e-13)


@pytest.mark.parametrize("kind", ["ucb", "q"])
def test_library_batch_formation_follows_the_oracle(kind):
    from oracle.hashing import chunk_hashes
    rng = random.Random(3)
    nprng = np.random.default_rng(3)
    kw = dict(c=0.7) if kind == "ucb" else dict(alpha=0.4, gamma=0.8, eps=0.6, eps_min=0.02, eps_decay=0.95)
    lib, ora = make_pair(kind, **kw)
    prefixes = [nprng.integers(0, 50000, size=rng.choice([64, 160, 320]), dtype=np.int32) for _ in range(4)]
    t_lib, t_ora = fea.Cht(), ChunkedHashTree()
    next_id = 0
    for rnd in range(60):
        for _ in range(rng.randrange(2, 9)):                 # arrivals
            pre = prefixes[rng.randrange(4)]
            keep = rng.choice([len(pre), len(pre), len(pre) // 2])
            toks = np.concatenate([pre[:keep], nprng.integers(0, 50000, size=rng.randrange(1, 70), dtype=np.int32)])
            hv = chunk_hashes(toks, 16)
            t_lib.insert(next_id, hash_vector=hv)
            t_ora.insert(next_id, hash_vector=hv)
            next_id += 1
        cap = rng.choice([3, 8, 32])
        draws = [(rng.random(), rng.random()) for _ in range(cap)]
        got = t_lib.build_batch_learned(lib, cap, draws)
        want = build_batch_learned(t_ora, ora, cap, draws, **BINS)
        assert got == want, rnd
        r = len(want) / (1.0 + 0.01 * sum(len(t_ora.hashes[i]) for i in want))     # any deterministic reward
        lib.reward(r)
        ora.reward(r)
        for rid in want:
            t_lib.finish(rid)
            t_ora.finish(rid)
    assert lib.info()["episodes"] == 60


def test_library_policy_errors():
    with pytest.raises(fea.FeaError):
        fea.Policy(7, 4, 4)
    with pytest.raises(fea.FeaError):
        fea.Policy(fea.FEA_POLICY_UCB, 0, 4, c=1.0)
    with pytest.raises(fea.FeaError):
        fea.Policy(fea.FEA_POLICY_UCB, 4, 4, (3, 3), c=1.0)          # thresholds must ascend
    with pytest.raises(fea.FeaError):
        fea.Policy(fea.FEA_POLICY_UCB, 4, 4, c=-1.0)
    with pytest.raises(fea.FeaError):
        fea.Policy(fea.FEA_POLICY_QLEARN, 4, 4, alpha=0.0, gamma=0.5)
    with pytest.raises(fea.FeaError):
        fea.Policy(fea.FEA_POLICY_QLEARN, 4, 4, alpha=0.5, gamma=1.5)
    p = fea.Policy(fea.FEA_POLICY_QLEARN, 4, 4, (1,), alpha=0.5, gamma=0.5, eps=0.0)
    with pytest.raises(fea.FeaError):
        p.entry((4, 0, 0), ADD)
    with pytest.raises(fea.FeaError):
        p.entry((0, 2, 0), ADD)
    with pytest.raises(fea.FeaError):
        p.entry((0, 0, 0), 2)
    with pytest.raises(fea.FeaError):
        p.reward(float("nan"))
    with pytest.raises(fea.FeaError):
        fea.Cht().build_batch_learned(p, 4, None)                     # Q-learning needs draws
    p.reward(1.0)                                                     # an empty episode is fine
    assert p.info() == {"decisions": 0, "episodes": 1, "eps": 0.0, "open": 0}
