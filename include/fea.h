/*
 * fea - paged decode attention over prefix-aliased KV blocks, for gfx950.
 *
 * C ABI of libfea.so.  Plain pointers and sizes only.  Every pointer argument
 * is marked HOST or DEVICE below.  The library never allocates or frees device
 * memory: the caller owns q, the KV caches, tables, outputs and the workspace.
 * The library owns only host bookkeeping behind fea_kv_pool.
 *
 * Every call returns a status: FEA_OK (0) or a negative code.  After a failure
 * fea_last_error() returns a thread-local, human-readable message, and no
 * output argument has been written (fea_build_block_tables additionally rolls
 * the pool back to its state before the call).  Nothing throws or aborts: no
 * C++ exception leaves the library; if the host itself runs out of memory a call
 * returns FEA_ENOMEM, and a handle (pool, tree, policy) that was being changed
 * by that call should be destroyed, its contents are then unspecified.
 *
 * Device work is enqueued on the caller's HIP stream and the call returns
 * without synchronising.  Contents of device buffers are never inspected on
 * the host.
 */
#ifndef FEA_H
#define FEA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FEA_OK       0
#define FEA_EINVAL  (-1)   /* bad argument (null pointer, unsupported shape, ...)        */
#define FEA_ENOMEM  (-2)   /* the KV pool has too few free blocks (or the host no memory) */
#define FEA_ERANGE  (-3)   /* a caller-provided table or workspace is too small          */
#define FEA_EHIP    (-4)   /* the HIP runtime reported an error (message has the detail) */

#define FEA_DTYPE_F32   0  /* q, caches, out are float32; arithmetic float32             */
#define FEA_DTYPE_BF16  1  /* q, caches, out are bfloat16; products/accumulation float32 */

#define FEA_GROUPABLE_REQUESTS 2048  /* requests with a batch index at or beyond this are
                                        never grouped with others (see fea_decode_attention) */

#define FEA_BLOCK_TOKENS 16  /* tokens per KV block (the paper's Section 3 setup; also the
                                chunk size K of the prefix hashes, Section 4.2)          */

/* flags for fea_attn_params.flags */
#define FEA_FLAG_REUSE_PLAN 1  /* skip alias detection: the workspace still holds the plan
                                  of the previous call, and tables/lengths/B/params are
                                  unchanged since (e.g. the other layers of one step)    */
#define FEA_FLAG_PLAN_ONLY 2   /* only alias detection: the plan is left in the workspace
                                  for later FEA_FLAG_REUSE_PLAN calls.  It depends on the
                                  tables and lengths alone, so the plan of the next decode
                                  step can be made on another stream while this step's
                                  attention runs (q, caches and out may be NULL)         */

#define FEA_FLAG_REFRESH_PLAN 4 /* the workspace holds the plan of an earlier call on this batch
                                  and since then the requests have only grown: lengths went
                                  up (decode steps), table rows got new columns at their
                                  ends, everything else is unchanged.  Alias detection is
                                  skipped; the split of the work is kept and every request's
                                  last piece is stretched to its length now (a few
                                  microseconds instead of a new plan).  The balance of the
                                  split drifts as the requests grow apart: plan anew every
                                  few dozen steps.  A request that had no blocks of its own
                                  when the plan was made (empty, or every block shared) and
                                  has grown since has no piece to stretch: the call then
                                  fills every output row with NaN and
                                  fea_decode_plan_info reports overflow flag 2            */

typedef struct fea_kv_pool fea_kv_pool;

/* Shape of one attention call.  Query head h reads KV head h / (num_q_heads /
 * num_kv_heads) (grouped-query attention with contiguous groups). */
typedef struct fea_attn_params {
    int32_t num_q_heads;
    int32_t num_kv_heads;   /* must divide num_q_heads                                   */
    int32_t head_dim;       /* f32: 32, 64, 128 or 256.  bf16: 64, 128 or 256            */
    int32_t block_size;     /* must be FEA_BLOCK_TOKENS                                  */
    int32_t dtype;          /* FEA_DTYPE_*                                               */
    float   scale;          /* softmax scale; 0 means 1/sqrt(head_dim) (Section 2.1)     */
    int32_t split_blocks;   /* KV blocks per work item; 0 lets the planner choose        */
    int32_t max_group;      /* 0: group any number of requests that alias a leading run
                               of blocks; 1: treat every request on its own              */
    int32_t flags;          /* FEA_FLAG_*                                                */
    int32_t run_kernel_min; /* alias detection compares the table rows on many workgroups
                               ahead of the planner's one workgroup when the batch has at
                               least 128 requests and this many table entries.  0: the
                               library's default (49152); < 0: always; > 0: that many    */
    int32_t merge_rows_min; /* the merge takes several output rows per wave from this
                               many rows (B * num_q_heads) on.  0: the library's default
                               (8192); < 0: always; > 0: that many                       */
    int32_t fused_max;      /* batches too small to be worth a plan are done in ONE launch,
                               a workgroup per (request, KV head) walking the whole
                               history (no plan; a shared block is then read once per
                               request, which at this size the L2 serves).  0: the library
                               decides, from an estimate of both ways' durations (about:
                               rows of up to 64 entries, as many (request, KV head) pairs
                               as the GPU has compute units, 4 query heads per KV head;
                               more for float32 caches); < 0: never; > 0: every batch
                               whose table rows have at most this many entries          */
} fea_attn_params;

/* Message of the last failure on this thread ("" if none).  HOST string owned
 * by the library, valid until the next failing call on the same thread. */
const char* fea_last_error(void);

/* ------------------------------------------------------------------------
 * KV block pool (host bookkeeping only).
 *
 * The paper's engines keep the KV cache in 16-token blocks and reuse a block
 * between requests whose token prefixes agree up to and including that block
 * (Section 2.2, hash-identified block reuse; Section 3, paged KV).  The pool
 * hands out block ids (indices into dimension 0 of the caller's K/V tensors),
 * counts references, and remembers which prefix each shared block stores.
 *
 * perm_seed == 0: ids are handed out 0, 1, 2, ...  Otherwise the initial free
 * list is shuffled: s = perm_seed; for k = num_blocks-1 .. 1: s += GAMMA;
 * j = mix(s) mod (k+1); swap(free[k], free[j])  (mix and GAMMA as documented at
 * fea_chunk_hashes).  Blocks are taken from the head of the free list; released
 * blocks are appended at its tail.
 *
 * Errors: FEA_EINVAL for num_blocks == 0, block_size != 16 or out == NULL.
 */
int32_t fea_kv_alloc(uint32_t num_blocks, uint32_t block_size, uint64_t perm_seed,
                     fea_kv_pool** out /* HOST */);
int32_t fea_kv_free(fea_kv_pool* pool);

/* Pool counters.  Any output pointer may be NULL.  refcounts: HOST int32[num_blocks]. */
int32_t fea_kv_stats(const fea_kv_pool* pool, uint32_t* num_blocks, uint32_t* free_blocks,
                     uint32_t* hash_collisions, int32_t* refcounts);

/* ------------------------------------------------------------------------
 * Chunked cumulative prefix hashes of one token sequence (HOST in, HOST out).
 *
 * The chunk-parallel formulation of the paper's prefix hash computation
 * (Appendix "Prefix Hash Computation", Algorithm 2; Section 4.2 "Hash
 * Vectors"): each chunk of K = 16 tokens is hashed independently into a leaf,
 * the leaves are chained h_c = Hash(h_{c-1} || leaf_c) from a fixed h_0, and a
 * trailing partial chunk is hashed too, giving C = ceil(T/16) values with the
 * property that h_c is equal for two sequences iff their first 16c tokens are.
 * The paper leaves Hash and h_0 open; this library fixes (mod 2^64):
 *   mix(x):  x ^= x>>30; x *= 0xBF58476D1CE4E5B9; x ^= x>>27;
 *            x *= 0x94D049BB133111EB; x ^= x>>31
 *   GAMMA  = 0x9E3779B97F4A7C15
 *   leaf   : a = mix(GAMMA ^ n); a = mix(a ^ (uint32)t_j), j = 1..n; n = chunk length
 *   chain  : h_0 = 0x243F6A8885A308D3; h_c = mix(mix(h_{c-1} + GAMMA) ^ leaf_c)
 *
 * hashes must hold ceil(T/16) values.  T == 0 writes nothing.
 * Errors: FEA_EINVAL for T < 0 or a NULL pointer with T > 0.
 */
int32_t fea_chunk_hashes(const int32_t* tokens /* HOST [T] */, int64_t T,
                         uint64_t* hashes /* HOST [ceil(T/16)] */);

/* The sequential formulation of the same vector (appendix "Prefix Hash
 * Computation", Algorithm 1): one incremental xxHash-64 state is fed the tokens
 * in order (each as 4 little-endian bytes) and digested after every 16th token
 * and after the last, so h_c = XXH64(first min(16c, T) tokens, seed).  Same
 * count, same prefix-consistency property, different values than
 * fea_chunk_hashes (the paper notes the two formulations differ in value).
 * Errors: as fea_chunk_hashes. */
int32_t fea_chunk_hashes_xxh64(const int32_t* tokens /* HOST [T] */, int64_t T, uint64_t seed,
                               uint64_t* hashes /* HOST [ceil(T/16)] */);

/* fea_chunk_hashes for a whole batch on the DEVICE (asynchronous on hip_stream;
 * Algorithm 2 as it is meant to run: the chunks of all requests hashed in
 * parallel, then one short chain per request).  tokens [n_tokens], tok_offsets
 * [B+1] and hash_offsets [B+1] are DEVICE arrays; request i's ceil(T_i/16) values
 * go to hashes[hash_offsets[i] ...] (DEVICE [n_hashes]), bit-identical to
 * fea_chunk_hashes.  A request whose offsets are negative, descending, beyond
 * n_tokens, or whose values would not fit below n_hashes is skipped (nothing is
 * written for it; the device cannot report an error without a synchronisation).
 * Never allocates or synchronises.
 * Errors: FEA_EINVAL for negative sizes or NULL pointers; FEA_EHIP if the launch
 * fails. */
int32_t fea_chunk_hashes_device(const int32_t* tokens /* DEVICE */, int64_t n_tokens,
                                const int64_t* tok_offsets /* DEVICE [B+1] */, int32_t B,
                                const int64_t* hash_offsets /* DEVICE [B+1] */,
                                uint64_t* hashes /* DEVICE [n_hashes] */, int64_t n_hashes, void* hip_stream);

/* Which formulation a pool (fea_build_block_tables) or a tree (fea_cht_insert)
 * hashes with: FEA_HASH_CHAINED (fea_chunk_hashes, the default; seed ignored) or
 * FEA_HASH_XXH64.  Block tables do not depend on the choice (aliasing is verified
 * on tokens); the hash vectors handed back do.
 * Errors: FEA_EINVAL for NULL, an unknown kind, a pool that already holds
 * registered prefixes or a tree that already holds requests. */
enum { FEA_HASH_CHAINED = 0, FEA_HASH_XXH64 = 1 };
int32_t fea_kv_set_hash(fea_kv_pool* pool, int32_t kind, uint64_t seed);
/* fea_cht_set_hash: declared with the tree below. */

/* ------------------------------------------------------------------------
 * Block tables for a batch, with prefix aliasing (HOST in, HOST out).
 *
 * For request i (tokens[tok_offsets[i] .. tok_offsets[i+1])) and column c the
 * table entry is the physical block holding tokens [16c, 16c+16) of exactly
 * that request's prefix.  Two requests get the same block in column c iff c is
 * a full chunk of both and their first 16(c+1) tokens are equal (Section 4.2:
 * same hash at level l iff same first l*K tokens; Section 2.2: block reuse when
 * hash sequences match).  A trailing partial chunk always gets a fresh block of
 * its own (decode appends into it).  Requests are processed in index order and
 * columns left to right; a column whose prefix is already stored (by this call
 * or an earlier one on the same pool) reuses that block and takes a reference,
 * any other column takes the head of the free list.  Lookup is by (level,
 * cumulative hash) and every hit is verified against the stored tokens and the
 * parent block, so a hash collision can never alias different prefixes.
 *
 *   block_tables  HOST int32 [B, max_blocks_per_seq], unused columns = -1
 *   seq_lens      HOST int32 [B]      = tok_offsets[i+1] - tok_offsets[i]
 *   hashes        HOST uint64, all requests back to back, or NULL
 *   hash_offsets  HOST int64 [B+1] start of each request's hashes, or NULL
 *
 * Errors: FEA_EINVAL (NULL/negative arguments, non-monotone offsets),
 * FEA_ERANGE (a request needs more than max_blocks_per_seq blocks), FEA_ENOMEM
 * (pool exhausted).  On any error the pool and all outputs are as before.
 */
int32_t fea_build_block_tables(fea_kv_pool* pool,
                               const int32_t* tokens, const int64_t* tok_offsets, int32_t B,
                               int32_t max_blocks_per_seq,
                               int32_t* block_tables, int32_t* seq_lens,
                               uint64_t* hashes, int64_t* hash_offsets);

/* Drops one reference from each of the nb blocks of a finished request's table
 * row (HOST).  A block whose count reaches zero forgets its prefix and joins the
 * tail of the free list - the pool-side counterpart of removing a finished
 * request (Section 4.2, "Removing a Request from the Active Batch").
 * Errors: FEA_EINVAL for ids out of range or blocks that hold no reference;
 * nothing is released in that case. */
int32_t fea_release(fea_kv_pool* pool, const int32_t* block_table_row /* HOST [nb] */, int32_t nb);

/* Host-side check of a table (for tests and debugging; HOST pointers): every
 * entry in columns < ceil(seq_lens[i]/16) lies in [0, num_blocks), seq_lens are
 * non-negative and fit table_stride.  Returns FEA_OK or FEA_EINVAL. */
int32_t fea_validate_block_tables(const int32_t* block_tables, int32_t table_stride,
                                  const int32_t* seq_lens, int32_t B, uint32_t num_blocks);

/* ------------------------------------------------------------------------
 * Decode attention (DEVICE pointers, asynchronous on hip_stream).
 *
 * For every request i and query head h, with L = seq_lens[i] cached tokens
 * found through block_tables[i]:
 *     out[i,h,:] = sum_t softmax_t( q[i,h,:] . k_t * scale ) v_t
 * i.e. softmax(Q K^T / sqrt(d)) V for the single decode query of each request
 * against its whole KV history (Section 2.1; the full-cache sweep per decode
 * step of Section 1).  seq_lens[i] counts the tokens attended to; the current
 * token's K/V must already be in the cache.  seq_lens[i] == 0 gives a zero row.
 *
 * Layouts (all contiguous):
 *   q, out        [B, num_q_heads, head_dim]
 *   k_cache       [num_blocks, num_kv_heads, 16, head_dim]   (v_cache alike)
 *   block_tables  int32 [B, table_stride]; only columns < ceil(L_i/16) are read
 *   seq_lens      int32 [B], each <= 16 * table_stride
 * The result is correct for ANY table whose read entries are valid block ids:
 * blocks may repeat inside a row and alias between rows at any position.
 * The device cannot check ids against the cache size: an id beyond the cache is
 * the caller's error and reads outside it; a negative entry inside a request's
 * length (e.g. lengths uploaded ahead of their tables) is read as block 0, so
 * the output of that request is wrong but no address before the cache is formed.
 * Requests whose rows start with the same run of block ids are detected on the
 * device and that run is swept once for all of them.  Only the first
 * FEA_GROUPABLE_REQUESTS requests of a batch take part in that detection: a
 * request with a higher index sweeps its whole history on its own (same result,
 * more KV reads); fea_decode_plan_info reports how many requests were grouped.
 * Which kernel sweeps the KV history follows from the parameters alone (the
 * result does not depend on it beyond rounding): bf16 caches with head_dim 64,
 * 128 or 256 and at most 64 query heads per KV head (32 at head_dim 256) go
 * through the matrix cores; float32 caches and wider query groups through the
 * vector unit, several times slower (fea_decode_plan_info: kernel
 * variant).  A batch within fea_attn_params.fused_max takes one launch of the
 * vector unit and makes no plan: FEA_FLAG_REUSE_PLAN and FEA_FLAG_REFRESH_PLAN
 * change nothing for it, FEA_FLAG_PLAN_ONLY still makes the plan (for
 * fea_decode_plan_info), and after an attention call fea_decode_plan_info
 * reports variant 2 and no groups.
 *
 *   workspace     DEVICE scratch of at least fea_decode_workspace_bytes() bytes,
 *                 256-byte aligned; contents are overwritten.  Calls that share
 *                 a workspace must be ordered on one stream.
 *   hip_stream    a hipStream_t (NULL = the default stream)
 *
 * Errors: FEA_EINVAL (NULL pointer, unsupported params, B < 0), FEA_ERANGE
 * (workspace_bytes too small), FEA_EHIP (launch failure).  B == 0 is a no-op.
 */
int32_t fea_decode_workspace_bytes(const fea_attn_params* p, int32_t B, int32_t table_stride,
                                   size_t* out_bytes /* HOST */);

int32_t fea_decode_attention(const fea_attn_params* p,
                             const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* block_tables, int32_t table_stride,
                             const int32_t* seq_lens, int32_t B,
                             void* out,
                             void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/* fea_decode_attention for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments, same result, bit for bit; the plan and the
 * partial results live in a buffer of FEA_STATIC_WORKSPACE_BYTES that is part of the
 * library's device image (every GPU the library runs on holds its own copy until
 * the process ends).  The call allocates nothing, on the host or on the device
 * (the buffer's device address is looked up once per GPU, at the first call on it).
 * A batch whose fea_decode_workspace_bytes() exceeds FEA_STATIC_WORKSPACE_BYTES is
 * refused with FEA_ERANGE (use fea_decode_attention with a workspace of your own).
 * All calls on one GPU share the buffer: it keeps the previous call's contents
 * (nothing in it has to start at zero - every call writes its plan before reading
 * it), and calls that overlap in time on one GPU - different streams, different
 * threads - race on it and give undefined results; order them on one stream.
 * FEA_FLAG_REUSE_PLAN, FEA_FLAG_PLAN_ONLY and FEA_FLAG_REFRESH_PLAN are refused
 * (FEA_EINVAL): another caller may have used the buffer in between.  Other errors as fea_decode_attention. */
#define FEA_STATIC_WORKSPACE_BYTES (48u << 20)
int32_t fea_decode_attention_static(const fea_attn_params* p,
                                    const void* q, const void* k_cache, const void* v_cache,
                                    const int32_t* block_tables, int32_t table_stride,
                                    const int32_t* seq_lens, int32_t B,
                                    void* out, void* hip_stream);

/* Summary of the plan the last fea_decode_attention call left in `workspace`
 * (synchronises hip_stream; for tests, tuning and the benchmark's reporting).
 * info: HOST int32[9] = { work items, prefix groups, requests in groups,
 * blocks per work item, partial rows, shared-run blocks (sum over groups),
 * kernel variant (0 generic, 1 MFMA, 2 one fused launch without a plan), overflow flag (1: the plan did not fit
 * its buffers, 2: FEA_FLAG_REFRESH_PLAN met a request it cannot stretch), sweep waves that
 * were given a share }. */
int32_t fea_decode_plan_info(const void* workspace /* DEVICE */, void* hip_stream,
                             int32_t* info /* HOST [9] */);

/* ------------------------------------------------------------------------
 * One decode step's growth of the KV history (Section 2.1: every decode step
 * appends one token's key and value per request; Section 3: in 16-token blocks).
 *
 * fea_kv_extend (HOST bookkeeping): every request's length grows by one; a
 * request whose length was a multiple of 16 (0 included) gets a fresh block from
 * the head of the free list, requests in index order, written into its table row
 * at column old_length / 16.  Such a block is private: it holds no registered
 * prefix and is never aliased.  block_tables (HOST [B x table_stride]) and
 * seq_lens (HOST [B]) are updated in place; *n_new_blocks (may be NULL) receives
 * the number of table entries written, so the caller knows whether the device
 * copy of the tables is stale.  Errors: FEA_ERANGE if a row has no column left,
 * FEA_ENOMEM if the pool has too few free blocks, FEA_EINVAL; nothing changed then.
 *
 * fea_kv_append (DEVICE, asynchronous on hip_stream): writes request i's new key
 * and value rows (k_new, v_new: [B, num_kv_heads, head_dim], the caches' dtype)
 * into the caches at token position seq_lens[i] - 1 - the lengths passed already
 * count the new token, as after fea_kv_extend.  Requests with length 0, a table
 * too narrow for the position or a padding entry there are skipped.  Only
 * num_kv_heads, head_dim, block_size and dtype of params are read.
 * Errors: FEA_EINVAL (NULL, shape, alignment: all device pointers 16-byte
 * aligned), FEA_EHIP.
 */
int32_t fea_kv_extend(fea_kv_pool* pool, int32_t* block_tables /* HOST in/out */, int32_t table_stride,
                      int32_t* seq_lens /* HOST in/out */, int32_t B, int32_t* n_new_blocks /* HOST, may be NULL */);
int32_t fea_kv_append(const fea_attn_params* params, const void* k_new /* DEVICE */, const void* v_new /* DEVICE */,
                      void* k_cache /* DEVICE */, void* v_cache /* DEVICE */,
                      const int32_t* block_tables /* DEVICE */, int32_t table_stride,
                      const int32_t* seq_lens /* DEVICE */, int32_t B, void* hip_stream);

/* ------------------------------------------------------------------------
 * Chunked Hash Tree: which waiting requests should join the running batch
 * (Section 4.2 "Chunked Hash Tree"; appendix "Algorithms": Insert, FindBest,
 * AddToBatch, Finish, Remove, BuildBatch).  Host bookkeeping only; it is the
 * step before fea_build_block_tables: the batch it forms is what gets tables.
 *
 * A request is its vector of cumulative chunk hashes (fea_chunk_hashes).  The
 * tree keeps the working set {(level, hash) of every active request}, for each
 * waiting request its missing count (hashes of it not in the working set), a
 * min-heap of (missing count, request id) with lazy deletion, a reverse index
 * from (level, hash) to the waiting requests carrying it, and the shared prefix
 * tip: the deepest level at which all active requests carry the same hash
 * (level 0 when nothing is active).  Request ids are the caller's; ties in the
 * missing count go to the smaller id (the heap orders pairs).
 *
 * Readings of the paper where its text and listings differ: the first request
 * of a batch enters the working set like any other; the tip after an addition
 * is the least common ancestor of the active requests; Finish always drops the
 * request from all structures.
 *
 * All pointers HOST.  Not thread-safe.  Errors: FEA_EINVAL (NULL, unknown id,
 * id in the wrong state, duplicate id), FEA_ENOMEM.  On error nothing changed.
 */
typedef struct fea_cht fea_cht;

/* chunk_tokens must be FEA_BLOCK_TOKENS (the chunk size of fea_chunk_hashes). */
int32_t fea_cht_create(int32_t chunk_tokens, fea_cht** out);
void    fea_cht_destroy(fea_cht* t);
int32_t fea_cht_set_hash(fea_cht* tree, int32_t kind, uint64_t seed);   /* see fea_kv_set_hash */

/* Insert: register a request as waiting, from its tokens (hashed here) or from a
 * ready hash vector of n values. */
int32_t fea_cht_insert(fea_cht* t, int64_t request_id, const int32_t* tokens /* [n_tokens] */, int64_t n_tokens);
int32_t fea_cht_insert_hashes(fea_cht* t, int64_t request_id, const uint64_t* hashes /* [n] */, int32_t n);

/* FindBest: the waiting request with the smallest missing count.  Also yields
 * the tip depth now, the depth the tip would have with the request added (the
 * deepest level, not below the tip, whose node of the request is in the working
 * set; 0 if none), the number of waiting requests that carry the request's hash
 * at that depth (the request included; every waiting request when that depth is
 * 0) and its missing count; any of these four may be NULL.  Changes nothing (the
 * answer is cached until the next mutation).  Returns FEA_OK, or 1 if no request
 * is waiting (then nothing is written). */
int32_t fea_cht_find_best(fea_cht* t, int64_t* request_id, int32_t* tip_before, int32_t* tip_after,
                          int32_t* peers, int32_t* missing);

/* AddToBatch / Finish / Remove: waiting -> active, active -> gone, waiting -> gone. */
int32_t fea_cht_add_to_batch(fea_cht* t, int64_t request_id);
int32_t fea_cht_finish(fea_cht* t, int64_t request_id);
int32_t fea_cht_remove(fea_cht* t, int64_t request_id);

/* Missing count of a waiting request; sizes and the tip (any pointer may be NULL;
 * working_set = distinct (level, hash) nodes of the active requests, heap_entries
 * counts stale entries too). */
int32_t fea_cht_missing(const fea_cht* t, int64_t request_id, int32_t* missing);
int32_t fea_cht_stats(const fea_cht* t, int64_t* n_waiting, int64_t* n_active, int32_t* tip_level,
                      uint64_t* tip_hash, int64_t* working_set, int64_t* heap_entries);

/* The rule-based stop policy of Section 4.3 ("Heuristic Policy").  With b requests
 * in the batch so far, a candidate whose addition would shorten the tip by `loss`
 * levels and which has `peers` waiting requests at the new depth is added if
 * loss <= 0; else if b < small_batch: if loss <= loss_small; else if loss <=
 * loss_limit; else if peers >= peers_relax and loss <= loss_relaxed.  The paper
 * gives no constants: all five are the caller's. */
typedef struct fea_stop_policy {
    int32_t small_batch, loss_small, loss_limit, peers_relax, loss_relaxed;
} fea_stop_policy;

/* BuildBatch: FindBest / policy / AddToBatch until the policy stops, nothing is
 * waiting, or max_batch requests were added.  ids (HOST [max_batch]) receives the
 * added requests in order, *n_out their number.  Requests added stay added. */
int32_t fea_cht_build_batch(fea_cht* t, const fea_stop_policy* policy, int32_t max_batch,
                            int64_t* ids, int32_t* n_out);

/* Learned stop policies of Section 4.3 ("Contextual Bandit", "Q-Learning Policy").
 * The state of a decision is (b, loss, peers) as for the rule-based policy,
 * discretised: b and peers into exponential bins (0 for 0, else 1 + floor(log2 x),
 * capped at bins - 1), loss into the number of the ascending loss_thresholds it
 * exceeds.  Actions: FEA_ADD, FEA_STOP.
 *   FEA_POLICY_UCB: takes the action with the larger mu/n + c sqrt(ln S / n)
 *     (mu: summed reward of the entry, n: times credited, S: all credited
 *     decisions); an entry never credited goes first, ADD before STOP; ties: ADD.
 *   FEA_POLICY_QLEARN: epsilon-greedy over a table Q (all zero at first); after
 *     an episode each of its transitions, in the order taken, is updated by
 *     Q += alpha (r + gamma max_a' Q(next state, a') - Q); the state after the
 *     last decision is terminal.  reward_every_step != 0 hands the reward to
 *     every transition, 0 to the last one only.  Then eps = max(eps_min,
 *     eps * eps_decay).
 * The paper fixes none of the constants. */
enum { FEA_ADD = 0, FEA_STOP = 1 };
enum { FEA_POLICY_UCB = 1, FEA_POLICY_QLEARN = 2 };
#define FEA_POLICY_MAX_THRESHOLDS 8
typedef struct fea_policy_params {
    int32_t kind;                    /* FEA_POLICY_UCB | FEA_POLICY_QLEARN */
    int32_t b_bins, w_bins;          /* 1..64 each */
    int32_t n_loss_thresholds;       /* 0..FEA_POLICY_MAX_THRESHOLDS */
    int32_t loss_thresholds[FEA_POLICY_MAX_THRESHOLDS];   /* ascending */
    int32_t reward_every_step;       /* Q-learning only */
    double c;                        /* UCB exploration coefficient, >= 0 */
    double alpha, gamma;             /* Q-learning: 0 < alpha <= 1, 0 <= gamma <= 1 */
    double eps, eps_min, eps_decay;  /* Q-learning: all in [0, 1] */
} fea_policy_params;
typedef struct fea_policy fea_policy;

/* Creates a policy with empty tables (b_bins x (n_loss_thresholds + 1) x w_bins x 2
 * entries).  Errors: FEA_EINVAL for NULL or parameters outside the ranges above. */
int32_t fea_policy_create(const fea_policy_params* params, fea_policy** out);
void    fea_policy_destroy(fea_policy* p);

/* The discretised state of (b, loss, peers); any output may be NULL. */
int32_t fea_policy_state(const fea_policy* p, int32_t b, int32_t loss, int32_t peers,
                         int32_t* b_bin, int32_t* loss_bin, int32_t* w_bin);

/* One decision: writes FEA_ADD or FEA_STOP to *action and appends (state, action)
 * to the open episode.  u_explore and u_action are the caller's uniform draws in
 * [0, 1) (used by Q-learning only: explore when u_explore < eps, and then ADD when
 * u_action < 1/2). */
int32_t fea_policy_decide(fea_policy* p, int32_t b, int32_t loss, int32_t peers,
                          double u_explore, double u_action, int32_t* action);

/* Closes the open episode with the observed decode throughput as its reward and
 * updates the tables as described above (an empty episode only decays eps). */
int32_t fea_policy_reward(fea_policy* p, double reward);

/* One table entry: UCB: *value = mean reward (0 if never credited), *count = n;
 * Q-learning: *value = Q, *count = updates of the entry.  FEA_ERANGE for a bin or
 * action outside the table. */
int32_t fea_policy_entry(const fea_policy* p, int32_t b_bin, int32_t loss_bin, int32_t w_bin,
                         int32_t action, double* value, int64_t* count);

/* Credited decisions (S), closed episodes, the current eps (0 for UCB), decisions
 * in the open episode; any pointer may be NULL. */
int32_t fea_policy_info(const fea_policy* p, int64_t* decisions, int64_t* episodes, double* eps,
                        int32_t* open_decisions);

/* BuildBatch (appendix "Batch Formation") with a learned policy: FindBest, state,
 * decision, AddToBatch until the policy stops, nothing is waiting, or max_batch
 * requests were added.  draws (HOST [2 * max_batch]) holds one (u_explore,
 * u_action) pair per decision, read in order; may be NULL for FEA_POLICY_UCB.
 * The caller runs the batch and then calls fea_policy_reward. */
int32_t fea_cht_build_batch_learned(fea_cht* t, fea_policy* policy, int32_t max_batch,
                                    const double* draws, int64_t* ids, int32_t* n_out);

/* Per-kernel timing for measurement runs.  fea_profile_enable(n, which) with n > 0
 * makes the next fea_decode_attention calls attach a pair of library-owned HIP events
 * to their launches; each pair takes the begin and end time of that one dispatch (no
 * extra packets on the stream, no synchronisation).  The events of the most recent n
 * calls are kept.  which = 0, 1 or 2 times only the alias detection, the KV sweep or
 * the merge; which = -1 times all three.  fea_profile_read(c, ms) waits for the c-th
 * call since enabling (0-based) and returns the durations in milliseconds (HOST
 * float[3], zero where not timed, e.g. the first under FEA_FLAG_REUSE_PLAN).
 * fea_profile_enable(0, -1) switches recording off.  Process-wide (calls from several
 * threads are recorded in the order in which they take their slot; a lock is taken only
 * while recording is on); leave it off in production.  Under a profiler that intercepts the launches
 * (rocprofv3 and other tools loaded through ROCP_TOOL_LIBRARIES) recording is
 * refused with FEA_EINVAL: the tool times the dispatches itself, and the two ways
 * of attaching to a dispatch are not combined.
 * Errors: FEA_EHIP if events cannot be created or read; FEA_EINVAL for NULL, bad
 * arguments, a call that was not recorded, or a profiler being attached. */
int32_t fea_profile_enable(int32_t max_calls, int32_t which);
int32_t fea_profile_read(int32_t call, float* ms);

/* Measurement aid: the rate at which this GPU streams memory through the KV sweep's
 * own fetch path (one single-wave workgroup per SIMD, 16 KB tiles of four 4 KB chunks
 * fetched global -> LDS, two tiles in flight), nothing computed.  Reads the largest
 * power-of-two number of 4 KB chunks that fits `bytes` exactly once per repeat -
 * chunk after chunk (scattered == 0) or in a fixed pseudo-random order, like KV blocks
 * scattered over a pool (scattered != 0) - and writes bytes read per second, in
 * GB/s (1e9), to *gbs.  Use a buffer well beyond the 256 MB memory-side cache.
 * DEVICE buffer (16-byte aligned, contents irrelevant, not modified); HOST gbs.
 * Times with events on hip_stream and synchronises it.
 * Errors: FEA_EINVAL (NULL, alignment, fewer than 4 MiB, repeats outside 1..1000),
 * FEA_EHIP. */
int32_t fea_stream_read_gbs(const void* buffer, size_t bytes, int32_t scattered, int32_t repeats,
                            void* hip_stream, double* gbs);

#ifdef __cplusplus
}
#endif
#endif /* FEA_H */
