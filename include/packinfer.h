/*
 * packinfer.h -- C ABI of the MI355X (gfx950) packed-attention library.
 *
 * The calls follow the problem statement of the PackInfer paper (Alg. 1,
 * inputs and outputs; Sec. 3.1 packed computation; Sec. 3.2 packed I/O):
 *
 *   pk_pack_plan            lengths, prefix families, budget C -> groups S_g,
 *                           offset tables O_g                    (Alg. 1)
 *   pk_kv_reorganize        paged KV -> group-contiguous buffers B_g
 *                           (Alg. 1 Part 2, Sec. 3.2 consolidation)
 *   pk_packed_prefill_attn  causal attention over the packed query-key
 *                           regions of each group                (Sec. 3.1)
 *   pk_packed_decode_attn   one query per request over B_g, shared prefix
 *                           read once per group, split-KV + LSE merge
 *                           (Sec. 3.2; Sec. 1 lossless merge)
 *   pk_padded_*             per-request padded execution, the in-run
 *                           comparison the paper argues against (Sec. 2.2)
 *
 * Conventions
 *   - "host" / "device" is stated for every pointer.  Device buffers are
 *     caller-owned; the library never allocates or frees device memory.
 *   - Kernels are enqueued on the caller's hipStream_t (passed as void*,
 *     NULL = default stream) and the call returns without synchronising.
 *     Small integer tables are copied host->device on that stream when a
 *     plan is first used with a workspace (see pk_plan_bind).
 *   - All tensors are in CALLER REQUEST ORDER; the permutation into groups
 *     is internal.  Every tensor pointer (q, k, v, out, pages, kv_buf, new
 *     rows) must be 16-byte aligned (PK_EINVAL otherwise).
 *   - A plan carries its device tables and the workspace it is bound to:
 *     calls on ONE plan must not run concurrently from several host threads,
 *     and launches that share a workspace must be ordered on the stream(s)
 *     by the caller (decode keeps partial results there).  Different plans
 *     may be used from different threads.  A workspace has ONE owner at a
 *     time, the plan that bound it last: a compute call of another plan on
 *     the same workspace uploads that plan's tables again (the library keeps
 *     track of the last binder per workspace address).  The caller must not
 *     write to, free or reuse the memory of a workspace while a plan that is
 *     bound to it is still in use; after doing so, call pk_plan_bind, which
 *     always uploads.
 *   - Return value: PK_OK (0) or a negative PK_E* code; the message is
 *     available from pk_last_error() (thread-local).  Arguments are checked
 *     before anything is launched.  Nothing throws or aborts: every entry
 *     point catches host exceptions (PK_ENOMEM when host memory runs out).
 *   - dtype: PK_BF16 (MFMA path) or PK_F32 (plain-FMA debug path).
 *     out_dtype: PK_BF16 or PK_F32 for the attention outputs.
 */
#ifndef PACKINFER_H
#define PACKINFER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PK_OK = 0, PK_EINVAL = -1, PK_ENOMEM = -2, PK_EUNSUPPORTED = -3, PK_EHIP = -4 };
enum { PK_BF16 = 0, PK_F32 = 1 };

/* Layout constants of the group-contiguous buffer. */
#define PK_GROUP_ALIGN 32      /* group bases are multiples of this many tokens */
#define PK_KV_BLOCK    32      /* tokens per tile of the bf16 buffer layout     */

typedef struct pk_plan pk_plan; /* opaque; host memory owned by the library */

/* ------------------------------------------------------------------------
 * pk_pack_plan -- Alg. 1 Part 1 (greedy length-balanced grouping under the
 * feasibility test of Eq. 2, token term) and the bookkeeping of Part 2
 * (prefix-first layout, offset tables O_g).  Deterministic, integer only.
 *
 *   kv_lens     host [n]  L_i: KV tokens request i attends to (incl. the
 *                         current token); > 0
 *   q_lens      host [n]  query rows of request i; NULL = kv_lens (plain
 *                         prefill); 1 = decode; < kv_len = chunked prefill.
 *                         Queries are the last q_len positions.
 *   prefix_ids  host [n]  family id (>= 0) or -1; NULL = no families
 *   prefix_lens host [n]  shared-prefix length, equal inside a family,
 *                         0 <= prefix_len <= kv_len; NULL iff prefix_ids NULL
 *   n                     number of requests (0 is allowed: empty plan)
 *   token_budget          C > 0, unique KV tokens per group (Sec. 3.2)
 *   headroom              delta >= 0 tokens reserved after every suffix
 *   out                   receives the plan; free with pk_plan_destroy
 *
 * Grouping rules: a family is one atomic item of length L_P + sum(L_Q); a
 * family longer than C is cut in member order into the fewest consecutive
 * sub-families that fit; items are sorted by (length desc, lowest member
 * index), the least-loaded group (lowest index on ties) takes the item if it
 * stays within C, otherwise a new group is opened; an item longer than C is
 * alone in its group; empty groups are dropped.
 * Errors: PK_EINVAL for any violated precondition.
 */
int pk_pack_plan(const int32_t* kv_lens, const int32_t* q_lens,
                 const int32_t* prefix_ids, const int32_t* prefix_lens,
                 int32_t n, int64_t token_budget, int32_t headroom, pk_plan** out);

/* pk_pack_plan_tree -- the same planner for NESTED shared prefixes (Sec. 3.2
 * "Prefix-Aware Grouping and Reuse": TriePartition yields shared prefixes at
 * every level of the prefix tree; Eq. 5 counts each shared segment once).
 * The prefixes are given as a forest of segments:
 *   node_parent host [n_nodes]  parent of node k, in [-1, k) (-1: a root)
 *   node_len    host [n_nodes]  tokens of the segment, > 0; a node stands for
 *                               the tokens [depth(parent), depth(parent)+len)
 *                               of every request below it
 *   req_node    host [n]        deepest node above request i, or -1; the
 *                               request's own suffix is what follows
 *                               depth(req_node[i]) (it may be empty)
 *   kv_lens, q_lens, token_budget, headroom, out: as for pk_pack_plan.
 * Every node needs at least one request below it.  The caller guarantees
 * that requests below a node hold identical K/V on that segment.
 * Grouping: a whole tree is one atomic item of length sum(node_len) +
 * sum(suffixes) and is never cut (a tree above C is alone in its group);
 * otherwise as pk_pack_plan.  Layout inside a group, per tree in pre-order:
 * the node's segment, the suffixes (+ headroom) of the requests attached
 * directly to it in ascending order, then its children in ascending order.
 * pk_trie_tree produces this input from token ids.  A forest of roots only
 * gives the layout of pk_pack_plan with uncut families.
 * Errors: PK_EINVAL for any violated precondition.
 */
int pk_pack_plan_tree(const int32_t* kv_lens, const int32_t* q_lens, int32_t n,
                      const int32_t* node_parent, const int32_t* node_len, int32_t n_nodes,
                      const int32_t* req_node, int64_t token_budget, int32_t headroom,
                      pk_plan** out);

void pk_plan_destroy(pk_plan* plan);

/* Read-only accessors (host). */
int32_t pk_plan_num_requests(const pk_plan* plan);
int32_t pk_plan_num_groups(const pk_plan* plan);
/* Tokens of the whole buffer (all groups, each base rounded up to
 * PK_GROUP_ALIGN; the total is a multiple of PK_KV_BLOCK). */
int64_t pk_plan_buf_tokens(const pk_plan* plan);
/* Unique KV tokens summed over groups: the I/O volume M of Eq. 5 without
 * headroom. */
int64_t pk_plan_unique_tokens(const pk_plan* plan);

/* Canonical serialisation, int32 words:
 *   magic 0x504B504C, version 1, n, G, C lo, C hi, headroom, PK_GROUP_ALIGN,
 *   buf_tokens lo, hi, then per group:
 *   load lo, hi, buf_tokens lo, hi, buf_base lo, hi, n_members, then per
 *   member (layout order): request, prefix_off, L_P, suffix_off, L_Q
 *   (offsets in tokens relative to the group base) -- the tuple O_g[i] of
 *   Alg. 1.
 * A plan of pk_pack_plan_tree has version 2 and per group, after buf_base:
 *   n_nodes, n_members, then per node (layout order): caller's node number,
 *   offset, tokens, parent (index among the group's nodes or -1), then per
 *   member (layout order): request, node (index among the group's nodes or
 *   -1), suffix_off, suffix tokens.
 * pk_plan_serialized_words returns the word count; pk_plan_serialize copies
 * them to host `out` (capacity `cap` words) and returns the count or
 * PK_EINVAL if cap is too small. */
int64_t pk_plan_serialized_words(const pk_plan* plan);
int64_t pk_plan_serialize(const pk_plan* plan, int32_t* out, int64_t cap);

/* ------------------------------------------------------------------------
 * Sizes of the caller-allocated device buffers.
 *
 * pk_kv_buf_bytes: bytes of the group-contiguous KV buffer.
 *   PK_BF16 layout: [Hkv][buf_tokens / 32] tiles; one tile holds 32 tokens of
 *   one KV head: first the K part (32*d bf16), then the V part (32*d bf16).
 *     K part: two sub-tiles u (tokens 16u..16u+15), each d/32 steps s of
 *       64 chunks l of 8 bf16: chunk (u,s,l)[j] = K[16u + l%16][32s + 8(l/16) + j]
 *     V part: d/16 column blocks t of 64 chunks l of 8 bf16:
 *       chunk (t,l)[j] = V[kappa(l/16, j)][16t + l%16],
 *       kappa(g, j) = 4g + j for j < 4, 16 + 4g + (j-4) otherwise.
 *   (This is the operand order of the 16x16x32 bf16 MFMA, so the decode
 *   kernel streams tiles with fully coalesced 16-byte loads.)  Token slots
 *   that hold no valid token (headroom, alignment) are written as zeros.
 *   PK_F32 layout: K as [Hkv][buf_tokens][d] floats, then V likewise.
 *
 * pk_workspace_bytes: bytes of the workspace that carries the plan's device
 *   tables and the split-KV partial results for the given head shape.
 */
size_t pk_kv_buf_bytes(const pk_plan* plan, int Hkv, int d, int dtype);
size_t pk_workspace_bytes(const pk_plan* plan, int Hq, int Hkv, int d, int dtype);

/* Builds the device tables of the plan for this head shape and copies them
 * into `workspace` (device, >= pk_workspace_bytes, 256-byte aligned) on
 * `stream`.  Optional: the compute calls bind on first use of a
 * (workspace, shape) pair; rebinding to another workspace is allowed.  The
 * caller must not modify the workspace while the plan is in use. */
int pk_plan_bind(pk_plan* plan, int Hq, int Hkv, int d, int dtype,
                 void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * pk_kv_reorganize -- Alg. 1 Part 2 / Sec. 3.2 "Contiguous Memory
 * Consolidation": gathers the valid tokens of every request from the paged
 * pool into the group buffers, each shared prefix once (taken through the
 * block table of the family's lowest-index member in the group).
 *
 *   k_pages, v_pages  device [num_blocks][page_size][Hkv][d], dtype
 *   block_table       device [n][max_blocks_per_req] int32, logical page b
 *                     of request i -> physical block; entries beyond the
 *                     request's length are ignored
 *   num_blocks        physical blocks in the pool (for bounds validation of
 *                     nothing but the caller's own sizes; block ids are
 *                     clamped into [0, num_blocks))
 *   kv_buf            device, pk_kv_buf_bytes; written
 * Errors: PK_EINVAL (null pointer, page_size <= 0, max_blocks too small for
 * the longest request), PK_EUNSUPPORTED (bf16 path needs d in {64, 128}).
 */
int pk_kv_reorganize(pk_plan* plan, const void* k_pages, const void* v_pages,
                     const int32_t* block_table, int32_t max_blocks_per_req,
                     int32_t page_size, int64_t num_blocks, int Hkv, int d, int dtype,
                     void* kv_buf, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * pk_packed_prefill_attn -- Sec. 3.1: attention computed directly over the
 * union of valid query-key regions of each group: query tiles are cut from
 * the group's packed token stream (a tile may span requests), only key tiles
 * holding at least one unmasked pair are visited, block-diagonal causal mask,
 * online softmax.  out[t,h,:] = softmax_j(scale * q[t,h].k[j,g(h)]) v[j,g(h)]
 * over the keys j <= ctx + t of the same request, g(h) = h / (Hq/Hkv).
 *
 *   q    device [sum q_lens][Hq][d]    k, v  device [sum kv_lens][Hkv][d]
 *   out  device [sum q_lens][Hq][d], out_dtype
 *   scale  finite and positive (here and in every attention call below)
 * Errors: PK_EINVAL; PK_EUNSUPPORTED (bf16 path: d in {64,128}, Hq % Hkv == 0).
 */
int pk_packed_prefill_attn(pk_plan* plan, const void* q, const void* k, const void* v,
                           void* out, float scale, int Hq, int Hkv, int d,
                           int dtype, int out_dtype,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * pk_packed_decode_attn -- Sec. 3.2: every request has ONE query row (the
 * plan must have been made with q_lens == 1).  KV is read from the group
 * buffer written by pk_kv_reorganize; a shared prefix segment is streamed
 * once for all members of its (sub-)family in the group; segments are cut
 * into fixed-size splits whose partial results are merged by log-sum-exp
 * (the lossless merge of Sec. 1).
 *
 *   q    device [n][Hq][d]       kv_buf  device, as written by reorganize
 *   out  device [n][Hq][d], out_dtype
 * Errors: PK_EINVAL; PK_EUNSUPPORTED (bf16 path: d in {64,128}, Hq/Hkv <= 32,
 * any ratio; a work item carries 32 / (Hq/Hkv) requests of a shared prefix).
 */
int pk_packed_decode_attn(pk_plan* plan, const void* q, const void* kv_buf,
                          void* out, float scale, int Hq, int Hkv, int d,
                          int dtype, int out_dtype,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * pk_packed_mixed_step -- Sec. 3 (overview): the prefill and the decode
 * requests of one continuous-batching step go through the same packed
 * execution.  One call for both halves of such a step: the packed prefill
 * tiles of `prefill_plan` and the packed decode work items of `decode_plan`
 * run in ONE launch in which workgroups of the two kinds alternate, so that
 * the HBM-bound decode work runs beside the matrix-bound prefill work on the
 * same compute units; the LSE merge of the decode partials follows as a
 * second launch.  Results are those of pk_packed_prefill_attn and
 * pk_packed_decode_attn (same arithmetic per tile and per work item).
 *   prefill half: prefill_plan, q, k, v, out, prefill_workspace (as for
 *                 pk_packed_prefill_attn)
 *   decode half:  decode_plan (q_lens == 1), decode_q, kv_buf (written by
 *                 pk_kv_reorganize), decode_out, decode_workspace (as for
 *                 pk_packed_decode_attn); the workspaces must differ
 *   scale, Hq, Hkv, d, dtype, out_dtype: common to both halves (one layer)
 * A plan with n = 0 makes the call equal to the other half's own call.
 * Errors: as for the two calls; PK_EUNSUPPORTED unless dtype is PK_BF16 and
 * d is 64 or 128. */
int pk_packed_mixed_step(pk_plan* prefill_plan, const void* q, const void* k, const void* v, void* out,
                         void* prefill_workspace, size_t prefill_workspace_bytes,
                         pk_plan* decode_plan, const void* decode_q, const void* kv_buf, void* decode_out,
                         void* decode_workspace, size_t decode_workspace_bytes,
                         float scale, int Hq, int Hkv, int d, int dtype, int out_dtype, void* stream);

/* pk_packed_decode_attn_static -- pk_packed_decode_attn for callers that
 * cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It takes no workspace: the plan's
 * device tables and the split-KV partial results live in a fixed array of
 * PK_STATIC_SCRATCH_BYTES that is part of the library's code object (every
 * GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing, on the device or through the runtime.
 *   - The first call of a plan on a device (and the first after another plan
 *     used the scratch) uploads the plan's tables with one host-to-device copy
 *     on `stream`; further calls of that plan only launch kernels.
 *   - A plan whose tables and partial results need more than
 *     PK_STATIC_SCRATCH_BYTES is rejected with PK_EUNSUPPORTED and a message
 *     that states both sizes (use pk_packed_decode_attn with a workspace).
 *   - All calls on one GPU share the one array, which keeps the contents of
 *     the last call: calls that overlap in time on one GPU (different
 *     streams, different threads) race and must be ordered by the caller.
 *     Nothing in it has to start at zero: every partial slot is written
 *     before the merge reads it.
 * Other arguments, results and errors as pk_packed_decode_attn; the outputs
 * are bit-identical to that call's. */
#define PK_STATIC_SCRATCH_BYTES (16u << 20)
int pk_packed_decode_attn_static(pk_plan* plan, const void* q, const void* kv_buf,
                                 void* out, float scale, int Hq, int Hkv, int d,
                                 int dtype, int out_dtype, void* stream);

/* ------------------------------------------------------------------------
 * pk_trie_partition -- TriePartition of Alg. 1 Part 2 from token ids (Sec.
 * 3.2: the requests of a batch form a prefix tree whose common prefixes are
 * stored once).  Produces the prefix_ids / prefix_lens that pk_pack_plan
 * takes: every request is assigned to at most one shared prefix, a prefix
 * has at least min_prefix tokens and at least two requests, and among all
 * such assignments the one with the largest saving sum d_k * (m_k - 1) is
 * returned (d_k tokens shared by m_k requests: the reduction of Eq. 5); on a
 * tie between a prefix and the prefixes nested below it the outer one wins.
 * Families are numbered by their lowest request index.  Host only.
 *
 *   token_ids     host, the n token sequences one after the other
 *   kv_lens       host [n], length of each sequence (> 0)
 *   prefix_ids    host [n] out: family or -1     prefix_lens  host [n] out
 *   saved_tokens  optional out: the saving
 * Errors: PK_EINVAL (NULL, n < 0, min_prefix < 1, kv_len <= 0).
 */
int pk_trie_partition(const int32_t* token_ids, const int32_t* kv_lens, int32_t n,
                      int32_t min_prefix, int32_t* prefix_ids, int32_t* prefix_lens,
                      int64_t* saved_tokens);

/* pk_trie_tree -- the whole prefix tree of a batch as the forest of shared
 * segments pk_pack_plan_tree takes (Sec. 3.2; Eq. 5 at every level: a segment
 * of len tokens above m requests saves len * (m - 1) tokens).  A node is made
 * for every branching point of the tree (or end of a request) below which at
 * least two requests lie and whose depth is at least min_prefix; runs without
 * branching are one segment.  Host only.
 *   token_ids, kv_lens, n, min_prefix: as for pk_trie_partition
 *   node_parent, node_len host [n] out: the first *n_nodes entries are set
 *                         (there are at most n - 1 nodes)
 *   n_nodes     host out
 *   req_node    host [n] out: deepest node above request i or -1
 *   saved_tokens host out (may be NULL)
 * Nodes are numbered by (lowest request below, depth), so parents precede
 * children and the output does not depend on the sort inside.
 * Errors: PK_EINVAL for any violated precondition.
 */
int pk_trie_tree(const int32_t* token_ids, const int32_t* kv_lens, int32_t n,
                 int32_t min_prefix, int32_t* node_parent, int32_t* node_len,
                 int32_t* n_nodes, int32_t* req_node, int64_t* saved_tokens);

/* ------------------------------------------------------------------------
 * Decoding over several steps with one plan (Sec. 3.2: every suffix is
 * allocated L_Q + delta tokens, "which reserves space for future token
 * generation"; Sec. 3.1 "Adaptive Grouping", Eq. 4: when to regroup).
 *
 * Step s = 0, 1, ... of a decode loop:
 *   1. pk_kv_append(step = s) writes the K/V rows of the token that every
 *      request has just produced into the headroom behind its suffix in
 *      kv_buf (buffer token suffix_off + L_Q + s; layout as documented at
 *      pk_kv_buf_bytes).  k_new, v_new: device [n][Hkv][d], dtype, request
 *      order.  Needs 0 <= s < headroom, else PK_EINVAL (no slot left: make a
 *      new plan from the grown lengths and reorganize).
 *   2. pk_packed_decode_attn_grown(grown = s + 1) is pk_packed_decode_attn
 *      with every request's suffix extended by the `grown` appended tokens
 *      (request i then has kv_len_i + grown keys).  grown in [0, headroom].
 * Both use the plan's tables as they are; nothing is re-planned or copied.
 * Calls of one step are ordered by the stream.
 *
 * pk_regroup_due evaluates the trigger of Eq. 4 after `steps` decode steps
 * since the plan was made: with L_g(steps) = L(S_g) + steps * |S_g| (every
 * member adds one unique token per step, prefixes do not grow) and
 * DeltaL = max_g L_g - min_g L_g, it sets PK_REGROUP_DRIFT in *flags when
 * steps * DeltaL >= C / 2, and PK_REGROUP_HEADROOM when steps >= headroom
 * (the next append has no slot).  *drift (optional) receives DeltaL.
 * PK_REGROUP_DRIFT_WITHIN_BUDGET is the same rule over the groups whose
 * initial load is at most C: a group that Alg. 1 opened for one item longer
 * than C cannot be balanced by regrouping and makes the plain rule fire at
 * the first step.  Host only, no device work.
 * Errors: PK_EINVAL (NULL, steps < 0).
 */
#define PK_REGROUP_DRIFT               1
#define PK_REGROUP_HEADROOM            2
#define PK_REGROUP_DRIFT_WITHIN_BUDGET 4
int pk_kv_append(pk_plan* plan, const void* k_new, const void* v_new, void* kv_buf,
                 int32_t step, int Hkv, int d, int dtype,
                 void* workspace, size_t workspace_bytes, void* stream);
int pk_packed_decode_attn_grown(pk_plan* plan, const void* q, const void* kv_buf,
                                void* out, float scale, int32_t grown, int Hq, int Hkv, int d,
                                int dtype, int out_dtype,
                                void* workspace, size_t workspace_bytes, void* stream);
int pk_regroup_due(const pk_plan* plan, int32_t steps, int32_t* flags, int64_t* drift);

/* ------------------------------------------------------------------------
 * In-run comparison: per-request padded execution (Sec. 2.2: request-aligned
 * tile grids, padding to the tile size, no cross-request packing).  Same
 * mathematics and tensor conventions as the packed calls.
 *   prefill: grid (request, query tile, head) sized by the longest request;
 *            every request's last tile is padded; natural request order.
 *   decode:  reads the PAGED pool through the block table, uniform number
 *            of splits sized by the longest request, shared prefixes re-read
 *            by every member.  bf16 only, d in {64,128}, Hq/Hkv <= 16
 *            (PK_EUNSUPPORTED otherwise).
 */
int pk_padded_prefill_attn(pk_plan* plan, const void* q, const void* k, const void* v,
                           void* out, float scale, int Hq, int Hkv, int d,
                           int dtype, int out_dtype,
                           void* workspace, size_t workspace_bytes, void* stream);
int pk_padded_decode_attn(pk_plan* plan, const void* q,
                          const void* k_pages, const void* v_pages,
                          const int32_t* block_table, int32_t max_blocks_per_req,
                          int32_t page_size, int64_t num_blocks,
                          void* out, float scale, int Hq, int Hkv, int d,
                          int dtype, int out_dtype,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Counts for the benchmark's work accounting (host).  1..7 refer to the
 * tables of the head shape the plan was last sized or bound for (0 before).
 *   what = 0: unmasked (query,key) pairs per head summed over requests
 *   what = 1: (query,key) pairs issued to the MFMA units by the packed
 *             prefill schedule, per head
 *   what = 2: same for the padded prefill schedule
 *   what = 3: decode work items; 4: split-KV partial slots;
 *   what = 5: tokens per decode split chosen by the schedule builder
 *   what = 6: query tiles of the packed prefill schedule; 7: of the padded
 */
int64_t pk_plan_stat(const pk_plan* plan, int what);

/* Offline profiling of schedule parameters (Sec. 3.1: capacity and tile
 * shapes are found by profiling a range of settings).  Overrides a choice of
 * the schedule builder for this plan; the next pk_workspace_bytes /
 * pk_plan_bind builds the tables again.  Results never depend on it.
 *   PK_TUNE_DECODE_SPLIT     tokens per split-KV work item (rounded up to
 *                            PK_KV_BLOCK); 0 = the builder's own choice
 *   PK_TUNE_PREFILL_PIPELINE how the bf16 prefill kernels (packed and padded)
 *                            bring K/V tiles into LDS: 0 = copied straight
 *                            from memory into LDS, three K and two V stages
 *                            (default); 1 = staged through registers, two
 *                            stages with padded rows.  Same tile shape (128
 *                            query rows x 64 keys), same arithmetic.
 *                            (pk_packed_mixed_step always runs pipeline 0.)
 * Errors: PK_EINVAL (NULL plan, unknown knob, value out of range). */
#define PK_TUNE_DECODE_SPLIT 0
#define PK_TUNE_PREFILL_PIPELINE 1
int pk_plan_tune(pk_plan* plan, int knob, int64_t value);

/* Message of the last error on this thread ("" if none). */
const char* pk_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PACKINFER_H */
