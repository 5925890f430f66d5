"""Learned stop policies of batch formation, by their definitions (test infrastructure only).

Section 4.3 ("Batching and Reinforcement Learning") frames the decision taken
for every candidate that FindBest proposes -- admit it (ADD) or dispatch the
batch as it stands (STOP) -- over the state s = (b, Delta, w): requests in the
batch so far, levels the shared prefix tip would lose, waiting requests that
share the prefix at the new depth.  The state is discretised (b and w into
exponential bins, Delta by coarse thresholds); the reward is the decode
throughput observed when the batch has run (appendix "Batch Formation").

  * contextual bandit: UCB(s, a) = mu(s, a) / n(s, a) + c sqrt(ln S / n(s, a))
    with mu the summed reward, n the times a was taken in s, S all decisions;
  * Q-learning: Q(s, a) <- Q(s, a) + alpha [r + gamma max_a' Q(s', a') - Q(s, a)],
    applied after the episode (one batch formation), epsilon-greedy selection
    with epsilon decaying from its start value to a floor.

Every query here walks plain dictionaries; nothing is cached or vectorised.
Random draws are arguments (u_explore, u_action in [0, 1)), never drawn here.

Readings where the paper is silent (none of the constants is given either):
  * exponential bin of x >= 0: 0 for x = 0, else 1 + floor(log2 x), capped at
    bins - 1 (so 1 | 2-3 | 4-7 | ...);
  * Delta bin: how many of the ascending thresholds Delta exceeds;
  * an action never taken in a state has no UCB value: it is taken first, ADD
    before STOP; later ties go to ADD;
  * S counts the decisions whose reward has been credited;
  * every decision of an episode, the closing STOP included, is credited the
    episode's reward (bandit); an episode cut short by an empty queue or by the
    batch-size cap has no STOP decision;
  * Q-learning walks the episode's transitions in the order they were taken,
    each update seeing the ones before it; the state after the last decision
    is terminal (value 0).  reward_every_step = True hands r to every
    transition, as the update rule reads; False hands it to the last one only
    (the earlier ones then learn through the bootstrap term alone);
  * a greedy tie goes to ADD; exploring picks ADD when u_action < 1/2;
  * epsilon is multiplied by the decay factor after every episode, not below
    the floor.
"""
from __future__ import annotations

import math

ADD, STOP = 0, 1


def exp_bin(x: int, bins: int) -> int:
    if x <= 0:
        return 0
    k = 0
    while (1 << (k + 1)) <= x:      # k = floor(log2 x)
        k += 1
    return min(1 + k, bins - 1)


def discretize(b: int, loss: int, peers: int, *, b_bins: int, w_bins: int, loss_thresholds):
    """(b, Delta, w) -> (b^, Delta^, w^)."""
    return exp_bin(b, b_bins), sum(1 for t in loss_thresholds if loss > t), exp_bin(peers, w_bins)


class UcbBandit:
    def __init__(self, c: float):
        self.c = c
        self.mu = {}        # (state, action) -> summed reward
        self.n = {}         # (state, action) -> times taken (credited)
        self.S = 0          # credited decisions
        self.episode = []   # decisions awaiting their reward

    def ucb(self, s, a):
        n = self.n.get((s, a), 0)
        if n == 0:
            return math.inf
        return self.mu[(s, a)] / n + self.c * math.sqrt(math.log(self.S) / n)

    def decide(self, s, u_explore=0.0, u_action=0.0):
        a = ADD if self.ucb(s, ADD) >= self.ucb(s, STOP) else STOP
        self.episode.append((s, a))
        return a

    def reward(self, r: float):
        for key in self.episode:
            self.mu[key] = self.mu.get(key, 0.0) + r
            self.n[key] = self.n.get(key, 0) + 1
            self.S += 1
        self.episode = []

    def value(self, s, a):
        """(mean reward, count) of an entry; (0, 0) when never credited."""
        n = self.n.get((s, a), 0)
        return (self.mu[(s, a)] / n if n else 0.0), n


class QLearner:
    def __init__(self, alpha: float, gamma: float, eps: float, eps_min: float, eps_decay: float,
                 reward_every_step: bool = True):
        self.alpha, self.gamma = alpha, gamma
        self.eps, self.eps_min, self.eps_decay = eps, eps_min, eps_decay
        self.every = reward_every_step
        self.Q = {}
        self.visits = {}
        self.episode = []

    def q(self, s, a):
        return self.Q.get((s, a), 0.0)

    def decide(self, s, u_explore: float, u_action: float):
        if u_explore < self.eps:
            a = ADD if u_action < 0.5 else STOP
        else:
            a = ADD if self.q(s, ADD) >= self.q(s, STOP) else STOP
        self.episode.append((s, a))
        return a

    def reward(self, r: float):
        T = len(self.episode)
        for i, (s, a) in enumerate(self.episode):
            last = i == T - 1
            future = 0.0 if last else max(self.q(self.episode[i + 1][0], ADD), self.q(self.episode[i + 1][0], STOP))
            r_i = r if (self.every or last) else 0.0
            self.Q[(s, a)] = self.q(s, a) + self.alpha * (r_i + self.gamma * future - self.q(s, a))
            self.visits[(s, a)] = self.visits.get((s, a), 0) + 1
        self.episode = []
        self.eps = max(self.eps_min, self.eps * self.eps_decay)

    def value(self, s, a):
        return self.q(s, a), self.visits.get((s, a), 0)


def build_batch_learned(cht, policy, max_batch: int, draws, **bins):
    """BuildBatch (appendix "Batch Formation") with a learned policy.

    draws: one (u_explore, u_action) pair per decision, consumed in order.  The
    caller runs the batch and then calls policy.reward(throughput).
    """
    batch = []
    k = 0
    while len(batch) < max_batch:
        cand = cht.find_best()
        if cand is None:
            break
        rid, before, after, peers, _ = cand
        s = discretize(len(batch), before - after, peers, **bins)
        u1, u2 = draws[k]
        k += 1
        if policy.decide(s, u1, u2) == STOP:
            break
        cht.add_to_batch(rid)
        batch.append(rid)
    return batch
