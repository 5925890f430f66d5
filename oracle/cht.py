"""Chunked Hash Tree scheduler state, by its definitions (test infrastructure only).

The paper's scheduler (Section 4.2 "Chunked Hash Tree"; appendix "Algorithms":
Insert, FindBest, AddToBatch, Finish, Remove) keeps, for requests given as
cumulative chunk-hash vectors H^r = (h_1 .. h_C):

  * the working set  W = { (l, h_l^r) : r active }                (Section 4.2)
  * the missing count of a waiting request  m_W(r) = |H^r \\ W|    (appendix,
    "Find Best Request - Alternative Heuristic")
  * the shared prefix tip: the deepest level at which all active requests
    carry the same hash, (0, none) when nothing is active
  * FindBest: the waiting request with the smallest missing count, together
    with the tip depth now, the depth the tip would have with that request
    added, and the number of waiting requests that carry the candidate's hash
    at that depth.

The paper maintains these incrementally (a lazy min-heap keyed by (count,
request), a reverse index hash -> waiting requests, reference counts).  This
module does none of that: every query recomputes its answer from the sets
above, so that it can be checked against the paper by eye.  The heap orders
entries as (count, request id) pairs, hence ties go to the smaller id.

Readings where the paper's text and listings disagree or are silent:
  * the first request added to an empty batch puts its hashes into the working
    set like any other (the text and the figure say so; the listing returns
    early);
  * the tip after AddToBatch is the least common ancestor of the active
    requests, as the text says (the listing tests membership after having
    inserted the new request's own hash, which would always succeed);
  * "peers" counts every waiting request carrying the candidate's hash at the
    prospective depth, the candidate included; at depth 0 (nothing shared, or
    nothing active) every waiting request qualifies;
  * Finish always removes the finished request from the auxiliary structures.

Hash vectors come from oracle.hashing.chunk_hashes (or are given directly: the
tests that follow the paper's figures pass small hand-made vectors).
"""
from __future__ import annotations

from .hashing import chunk_hashes


class ChunkedHashTree:
    def __init__(self, chunk_tokens: int = 16):
        self.K = chunk_tokens
        self.hashes = {}      # request id -> tuple of cumulative hashes
        self.waiting = set()
        self.active = []      # in order of admission

    # ---- registration
    def insert(self, rid: int, tokens=None, hash_vector=None):
        if rid in self.hashes:
            raise KeyError(f"request {rid} already present")
        H = tuple(hash_vector) if hash_vector is not None else tuple(chunk_hashes(tokens, self.K))
        self.hashes[rid] = H
        self.waiting.add(rid)

    def remove(self, rid: int):
        """Withdraw a waiting request."""
        if rid not in self.waiting:
            raise KeyError(f"request {rid} is not waiting")
        self.waiting.discard(rid)
        del self.hashes[rid]

    # ---- the sets of Section 4.2, recomputed on demand
    def working_set(self):
        return {(l + 1, h) for r in self.active for l, h in enumerate(self.hashes[r])}

    def missing(self, rid: int) -> int:
        W = self.working_set()
        return sum(1 for l, h in enumerate(self.hashes[rid]) if (l + 1, h) not in W)

    def tip(self):
        """(level, hash) of the deepest node shared by all active requests; (0, None) if none."""
        if not self.active:
            return 0, None
        first = self.hashes[self.active[0]]
        depth = min(len(self.hashes[r]) for r in self.active)
        level = 0
        while level < depth and all(self.hashes[r][level] == first[level] for r in self.active):
            level += 1
        return (level, first[level - 1]) if level else (0, None)

    # ---- the operations
    def find_best(self):
        """(request, tip depth now, tip depth with it added, peers, its missing count) or None."""
        if not self.waiting:
            return None
        best = min(self.waiting, key=lambda r: (self.missing(r), r))
        H = self.hashes[best]
        before = self.tip()[0]
        W = self.working_set()
        after = 0
        for l in range(min(before, len(H)), 0, -1):
            if (l, H[l - 1]) in W:
                after = l
                break
        if after == 0:
            peers = len(self.waiting)
        else:
            peers = sum(1 for w in self.waiting if len(self.hashes[w]) >= after and self.hashes[w][after - 1] == H[after - 1])
        return best, before, after, peers, self.missing(best)

    def add_to_batch(self, rid: int):
        if rid not in self.waiting:
            raise KeyError(f"request {rid} is not waiting")
        self.waiting.discard(rid)
        self.active.append(rid)

    def finish(self, rid: int):
        if rid not in self.active:
            raise KeyError(f"request {rid} is not active")
        self.active.remove(rid)
        del self.hashes[rid]

    # ---- the second metric of the appendix (used by the pins only)
    def missing_from_tip(self, rid: int) -> int:
        """m_S(r) = |S \\ H^r| with S the working-set hashes at or above the tip level."""
        level = self.tip()[0]
        S = {(l, h) for (l, h) in self.working_set() if l <= level}
        Hr = {(l + 1, h) for l, h in enumerate(self.hashes[rid])}
        return len(S - Hr)


def heuristic_policy(batch_size: int, loss: int, peers: int, *, small_batch: int, loss_small: int,
                     loss_limit: int, peers_relax: int, loss_relaxed: int) -> bool:
    """The rule-based stop policy of Section 4.3 ("Heuristic Policy"): True = add, False = stop.

    Free additions are always taken; a small batch tolerates more loss; otherwise
    the loss must stay within a threshold, slightly relaxed when many waiting
    requests share the resulting prefix.  The paper gives no constants: they are
    parameters here, and nothing pins their values.
    """
    if loss <= 0:
        return True
    if batch_size < small_batch:
        return loss <= loss_small
    if loss <= loss_limit:
        return True
    return peers >= peers_relax and loss <= loss_relaxed


def build_batch(cht: ChunkedHashTree, max_batch: int, **policy):
    """BuildBatch (appendix "Batch Formation") with the heuristic policy: the admitted request ids, in order."""
    batch = []
    while len(batch) < max_batch:
        cand = cht.find_best()
        if cand is None:
            break
        rid, before, after, peers, _ = cand
        if not heuristic_policy(len(batch), before - after, peers, **policy):
            break
        cht.add_to_batch(rid)
        batch.append(rid)
    return batch
