"""CPU oracle for paged decode attention over prefix-aliased KV blocks.

TEST INFRASTRUCTURE ONLY.  Everything in this package is a plain, slow,
by-the-definition CPU implementation used to check the HIP library.  It shares
no code with the library (no common helpers, constants or tables), imports
nothing from it, and must never be called from the product path: only the test
suite, the smoke check and the benchmark's CPU-baseline leg use it.

What pins each function (see the tests that do not need a GPU):

* attention.decode_attention - brute-force scalar loops on tiny inputs; closed
  forms of softmax attention (one token, equal keys, constant values, a
  dominating key); a third opinion from a dense fp64 library attention on a
  contiguous table; invariance under physical block placement and under
  duplicated histories; exact split-and-merge identity.
* block_tables.build_block_tables - the aliasing rule is written out directly
  on token prefixes (no hash); pinned by the structure the paper's sharing
  patterns imply (shared columns, distinct ids, reference counts) and by a
  quadratic all-pairs prefix comparison on small batches.
* hashing.chunk_hashes - count, cumulativity and the prefix-consistency
  property ("equal at level l iff equal first l*K tokens") follow the paper's
  worked example and Algorithm 2's structure.  The paper prints no hash values
  and leaves Hash/InitConst open, so the *values* follow this library's written
  specification only: parity of hash values is "parity unpinned" beyond two
  independently written implementations agreeing bit for bit.
* cht.ChunkedHashTree - the scheduler's sets and queries written out from their
  definitions (no heap, no reverse index, no incremental state); pinned by the
  walk-through of Section 4.2, the R1..R4 example and the four caption values of
  the appendix on the alternative FindBest heuristic, and that appendix's
  theorem checked on random trees.  The constants of the stop policy are free
  parameters in the paper: policy parity is unpinned.
* policy.UcbBandit / policy.QLearner - the two update rules of Section 4.3 taken
  literally over dictionaries; pinned by values worked by hand (one UCB index,
  two passes of a three-step Q-learning episode, the Bellman fixed point of a
  chain), the logarithmic bound on the pulls of a worse arm under deterministic
  rewards, and written-out bin tables.  The bins' shape, the tie rules and
  which transitions receive the reward are readings (listed in that module);
  the paper gives no constants, so learned *behaviour* on a workload is
  unpinned.
"""
