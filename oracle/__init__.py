"""CPU oracle for the packed-attention hot path.

TEST INFRASTRUCTURE ONLY: nothing here is used by the product path.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It shares no code with the HIP library.

Modules:
  attention -- plain causal GQA attention on logical per-request tensors
               (C, fp64 accumulation), prefill and decode; pinned.
  merge     -- log-sum-exp merge of partial attention results; pinned.
  paged     -- logical KV of a request from a paged pool, and the dense
               group buffer B_g that Alg. 1 Part 2 describes; pinned.
  planner   -- Alg. 1 (greedy length-balanced grouping, prefix-first layout)
               restated from the paper; pinned.  The values of the headroom
               delta and of M_max are "parity unpinned": the paper prints no
               number for either.  Also the decode-step evolution rules: group
               loads after t steps, the drift and the regrouping trigger of
               Eq. 4 (pinned by hand-worked examples and a brute force of the
               definition); the cadence the paper mentions for its own
               workloads (every 20-40 steps) is "parity unpinned".
  trie      -- TriePartition from token ids: the one-level choice of shared prefixes that
               minimises Eq. 5; pinned (hand-worked examples, exhaustive search on tiny inputs).
  planner.make_plan_tree, paged.group_buffer_tree, trie.trie_tree -- nested shared prefixes
               (a forest of segments): plan, dense buffer and the whole-tree TriePartition; pinned
               (hand-worked words, invariants, reduction to the one-level plan).
  paged.append_step -- the headroom slot a generated token goes to (Sec. 3.2); pinned.
"""
