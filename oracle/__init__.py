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
               number for either.
"""
