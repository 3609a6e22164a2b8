/*
 * sk.h - C ABI of the stateful-session attention library for MI355X (gfx950).
 *
 * One attention layer of the paper's stateful-session model: a short segment of
 * new tokens attends against a long, persistent, per-session KV cache.
 *
 *   data plane  (Alg. 1, the append step; Sec. 3.4): sk_session_append commits the
 *                chunk's K/V into the session cache and the chunk attends causally
 *                over cache + chunk; nothing already cached is recomputed;
 *   query plane (Alg. 2, the forward pass of the query tokens; Sec. 3.2 Eq. 2;
 *                Sec. 3.3 Region 2; Sec. 3.9.3 Extend/Clear): sk_session_query
 *                attends over the cache and commits nothing;
 *   both planes for many sessions in one step (Sec. 3.7 heterogeneous
 *                PREFILL+DECODE batches): sk_batch_step;
 *   a batch of registered questions sharing a prefix, evaluated against one session
 *                after a data update (Alg. 3; Sec. 3.7 grouped prefill):
 *                sk_session_query_shared_prefix.
 *
 * The result of every attention call is softmax(Q K^T * scale) V (Sec. 3.2 Eq. 1)
 * with grouped-query mapping "query head h reads KV head h / (Hq/Hkv)" and causal
 * limit "the token at absolute position p sees positions 0..p inclusive".
 *
 * General rules
 *   - Every function returns SK_OK (0) or a negative sk_status; nothing throws,
 *     aborts or synchronises the device unless stated.
 *   - The caller owns every device buffer (kv_mem, workspace, q/k/v/out/lse).  The
 *     library owns host metadata and the layout inside kv_mem and workspace.  The
 *     library calls hipHostMalloc once per pool (a small pinned staging ring) and
 *     never hipMalloc.
 *   - Kernels are enqueued on the stream passed in (a hipStream_t cast to void*);
 *     host metadata (lengths, block tables, free list) advances at enqueue time;
 *     device results are valid once the stream reaches that point.  All calls on a
 *     pool must be issued from one thread at a time and on one stream (or be
 *     ordered externally), mirroring the paper's single GPU worker (Sec. 3.6).
 *   - Device pointers must be 16-byte aligned.
 *   - Same inputs, same block tables, same n_splits => bit-identical outputs.
 *   - Token-major layouts: q [T][Hq][d], k and v [T][Hkv][d], out [T][Hq][d],
 *     lse [T][Hq] (natural-log log-sum-exp of the scaled scores, float).
 *   - Precision, bf16 pools: scores, softmax statistics and accumulators are fp32; the softmax
 *     weights enter the second contraction rounded to bf16 and the row sums that normalise the
 *     output add those same rounded weights, so an output row is an exact convex combination of
 *     V rows; lse is taken from the sum of the weights before rounding (fp32).  fp32 pools
 *     compute in fp32 throughout.
 */
#ifndef SK_H
#define SK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sk_status {
    SK_OK = 0,
    SK_E_INVAL = -1,      /* null/misaligned pointer, negative size, bad enum, repeated session */
    SK_E_SHAPE = -2,      /* head counts / head_dim / block_tokens not supported */
    SK_E_DTYPE = -3,
    SK_E_NOMEM = -4,      /* pool out of blocks, sessions, or table space; nothing changed */
    SK_E_BADSESSION = -5,
    SK_E_EMPTY = -6,      /* softmax over zero keys (cache-only query on an empty session) */
    SK_E_WORKSPACE = -7,  /* kv_mem / workspace too small, or step exceeds max_batch_tokens */
    SK_E_HIP = -8,        /* a HIP runtime call failed; see sk_last_hip_error() */
    SK_E_NODEVICE = -9    /* compute call on a metadata-only pool */
} sk_status;

enum { SK_F32 = 0, SK_BF16 = 1 };                       /* element types */
enum { SK_OP_APPEND = 0, SK_OP_QUERY_A = 1, SK_OP_QUERY_B = 2 };  /* sk_batch_step ops */
enum { SK_POOL_METADATA_ONLY = 1 };                     /* sk_pool_desc.flags */

typedef struct sk_pool sk_pool;

/*
 * Pool description, filled by the caller.  The pool is the paper's unified KV cache
 * (the cells of Sec. 3.7 and Sec. 3.10.1) for ONE layer, cut into blocks of block_tokens
 * tokens; a session owns a list of blocks (its block table).  Per token the pool
 * stores 2 * n_kv_heads * head_dim elements (Sec. 5.3 with d = n_kv_heads*head_dim).
 */
typedef struct sk_pool_desc {
    int32_t dtype;            /* SK_F32 | SK_BF16: type of q,k,v and of the cache (the
                                 commit is a bit copy) */
    int32_t n_q_heads;        /* multiple of n_kv_heads */
    int32_t n_kv_heads;
    int32_t head_dim;         /* 64 or 128.  bf16 pools with at most 128 query heads per KV head
                                 (any such group size) run on the matrix pipe; fp32 pools take the
                                 fp32-FMA kernel (at most 16 per KV head) */
    int32_t block_tokens;     /* power of two, 16..1024 */
    int32_t max_sessions;     /* >= 1 */
    int64_t n_blocks;         /* blocks in the pool */
    int64_t max_session_tokens; /* longest session; 0 => n_blocks * block_tokens; capped at 2^20 blocks */
    int32_t max_batch_tokens; /* most new tokens (appends + queries) in one call; 0 => 4096 */
    int32_t flags;            /* 0 or SK_POOL_METADATA_ONLY (host bookkeeping only: no device
                                 memory, compute calls only do their allocation part; lets a
                                 scheduler rehearse admission, Sec. 3.7) */
    float   softmax_scale;    /* 0 => 1/sqrt(head_dim) (Sec. 3.2 Eq. 1) */
    int32_t reserved;
    void*   kv_mem;           /* DEVICE, >= sk_pool_kv_bytes(desc), 256-byte aligned */
    size_t  kv_bytes;
    void*   workspace;        /* DEVICE, >= sk_pool_workspace_bytes(desc), 256-byte aligned:
                                 device block tables, work lists, split partials, staging
                                 for uncommitted query K/V */
    size_t  workspace_bytes;
} sk_pool_desc;

/* Sizes implied by a description (kv_mem/workspace fields ignored).  0 on a bad description. */
size_t sk_pool_kv_bytes(const sk_pool_desc* desc);
size_t sk_pool_workspace_bytes(const sk_pool_desc* desc);

/* Creates host metadata (and, unless metadata-only, a pinned staging ring on the current
 * device; zeroes nothing in kv_mem).  *out is NULL on error.
 * Tuning switches, read from the environment here and fixed for the life of the pool (none
 * changes a result beyond the rounding order of the split merge; they exist for sweeps):
 *   SK_TARGET_WGS=n    workgroups a single-session call is cut into (default: 256 or 512 by shape)
 *   SK_FORCE_SIMPLE=1  always the fp32-FMA attention kernel
 *   SK_NO_256=1        never the 256-row eight-wave instance of the bf16 kernel
 *   SK_NO_PACK=1       a question batch gives every question a row tile of its own
 *   SK_NO_INTERLEAVE=1 the splits of a query take contiguous chunks of the cache instead of
 *                      interleaved 64-key pieces
 *   SK_NO_P128=1       never the eight-wave (two key phases) instance of the 128-row tile
 *   SK_P128_MIN_TOKENS=n  cached tokens from which a single-session call of 65-128 rows takes that
 *                      instance (default 30720: below, its longer start outweighs the gain)
 *   SK_NO_STREAM_LOADS=1  calls with one row tile per KV head load the cache with the default cache
 *                      policy instead of non-temporal
 *   SK_STREAM_MIN_TOKENS=n  cached tokens from which the 128-row instances do so (default 65536;
 *                      the 64-row instance always does)
 *   SK_FUSE=1          single-session calls merge their split partials inside the attention kernel
 *                      instead of in a second kernel (one launch per call; measured slower on
 *                      MI355X, so not the default; the same function merges a row either way, the
 *                      results are bit-identical)
 *   SK_WAIT_POLLS=n    with SK_FUSE: how many polls a workgroup waits for the other workgroups
 *                      of its row tile before it leaves the merge to the last one (default 256;
 *                      0: never wait)
 *   SK_FUSE_LIST=1     batched calls merge inside the attention kernel (last workgroup only)
 *   SK_MERGE_FENCES=1  with SK_FUSE: full device-scope fences around the arrival (for comparison) */
int sk_pool_create(const sk_pool_desc* desc, sk_pool** out);
/* Frees host metadata and the staging ring; caller memory is untouched.  The caller must
 * have synchronised the stream(s) the pool was used on. */
int sk_pool_destroy(sk_pool* pool);
int sk_pool_blocks_free(const sk_pool* pool, int64_t* out);
/* Replaces the free list by perm[0..n-1] (a permutation of 0..n_blocks-1; blocks are handed
 * out in that order).  Only legal while no session owns a block.  Lets a harness reproduce
 * fragmented, randomly permuted block tables. */
int sk_pool_set_alloc_order(sk_pool* pool, const int32_t* perm, int64_t n);

/* Sessions (Sec. 3.4).  Ids are small non-negative integers, reused after destroy. */
int sk_session_create(sk_pool* pool, int32_t* out_id);
int sk_session_destroy(sk_pool* pool, int32_t id);          /* blocks go back to the free list */
int sk_session_length(const sk_pool* pool, int32_t id, int64_t* out_tokens);
/* Host view of the block table, valid until the next call that changes the session. */
int sk_session_block_table(const sk_pool* pool, int32_t id, const int32_t** table, int64_t* n_blocks);

/*
 * DATA PLANE (Alg. 1).  q [L][Hq][d], k,v [L][Hkv][d] DEVICE, pool dtype.  Commits k,v bit for
 * bit at positions n..n+L-1 of the session and writes, for chunk token i, attention over
 * positions 0..n+i.  out [L][Hq][d] of out_dtype (SK_F32 or the pool dtype); lse [L][Hq]
 * float or NULL.  q/out may be NULL together: commit only.  All or nothing: every check that
 * can refuse the call runs before anything changes, and if a HIP call fails afterwards
 * (SK_E_HIP) the host side is taken back, so on error the session's length and block table
 * and the free list are as before (one exception that no caller can observe through the API
 * other than by counting free blocks: when the session's last block was shared with a fork and
 * the commit kernel was already enqueued, the session keeps its private copy of that block).
 * L == 0 is a no-op.  L <= max_batch_tokens.
 */
int sk_session_append(sk_pool* pool, int32_t id, const void* q, const void* k, const void* v,
                      int32_t L, void* out, int out_dtype, float* lse, void* hip_stream);

/*
 * QUERY PLANE (Alg. 2; Sec. 3.2 Eq. 2).  Never changes kv_mem, tables or lengths.
 * k == v == NULL: keys are the cache only, no mask (the literal Eq. 2).  k,v given
 * [nq][Hkv][d]: the query's own tokens follow the cache causally and are dropped afterwards
 * (Region 2, Sec. 3.3; Extend then Clear, Sec. 3.9.3); the output equals what
 * sk_session_append would have written.  n_splits: partitions of the cached tokens
 * processed by separate workgroups and merged by log-sum-exp; 0 = chosen by the library.
 * An empty cache with k == NULL gives SK_E_EMPTY.  nq == 0 is a no-op.
 * The call enqueues kernels only (its decomposition travels in the kernel arguments, and so does
 * the list that stages its own k,v while they span at most 80 groups of 16 tokens): it can be
 * captured in a HIP graph and replayed, as long as the session is not changed in between (its
 * length is baked into the captured arguments).
 */
int sk_session_query(sk_pool* pool, int32_t id, const void* q, const void* k, const void* v,
                     int32_t nq, void* out, int out_dtype, float* lse, int32_t n_splits,
                     void* hip_stream);

/*
 * RAGGED MULTI-SESSION STEP (Sec. 3.7).  Item i owns packed token rows
 * cu_tokens[i]..cu_tokens[i+1]-1 of q/k/v/out/lse; op[i] is SK_OP_APPEND, SK_OP_QUERY_A
 * (cache only) or SK_OP_QUERY_B (own K/V, causal).  session_id, op, cu_tokens are HOST
 * arrays.  A session may appear once per step.  Equal to issuing the items one by one
 * (outputs up to summation order, cache bits exactly).  All or nothing for the whole step,
 * as for sk_session_append: a step that is refused, or that fails half way, leaves every
 * session's length and block table and the free list as they were.
 */
int sk_batch_step(sk_pool* pool, int32_t n_items, const int32_t* session_id, const int32_t* op,
                  const int32_t* cu_tokens, const void* q, const void* k, const void* v,
                  void* out, int out_dtype, float* lse, void* hip_stream);

/*
 * REGISTERED-QUESTION BATCH (Alg. 3 loop body for all f_i at once; Sec. 3.7 grouped prefill).
 * Question j = prefix (P tokens, shared) ++ suffix_j (Sfx tokens); each is evaluated like a
 * query with own K/V; the prefix rows are computed once.  qp [P][Hq][d], kp,vp [P][Hkv][d],
 * qs [NQ][Sfx][Hq][d], ks,vs [NQ][Sfx][Hkv][d]; out_prefix [P][Hq][d], out_suffix
 * [NQ][Sfx][Hq][d]; lse_* float or NULL.  P may be 0.  Commits nothing.
 */
int sk_session_query_shared_prefix(sk_pool* pool, int32_t id,
                                   const void* qp, const void* kp, const void* vp, int32_t P,
                                   const void* qs, const void* ks, const void* vs,
                                   int32_t NQ, int32_t Sfx,
                                   void* out_prefix, void* out_suffix, int out_dtype,
                                   float* lse_prefix, float* lse_suffix, void* hip_stream);

/*
 * Reads a session's committed K/V back in token order: k_out, v_out [count][Hkv][d] DEVICE,
 * pool dtype, retained tokens first..first+count-1 (evicted tokens do not count).  Bit copy
 * through the block table (used to check the commit and to export a session).
 */
int sk_session_gather(const sk_pool* pool, int32_t id, int64_t first, int64_t count,
                      void* k_out, void* v_out, void* hip_stream);

/*
 * Drops every cached token behind the first new_length retained ones: the
 * SeqRemove(s, p, infinity) of Sec. 3.9.3 / Alg. 3, by which a caller can also reproduce the
 * literal Strip / Extend / Clear cycle (append, read the output, truncate).  Host metadata only:
 * whole blocks past the new end return to the free list, no device work, kv_mem bytes are not
 * touched.  new_length > current length gives SK_E_INVAL.
 */
int sk_session_truncate(sk_pool* pool, int32_t id, int64_t new_length);

/*
 * REGION 0 / REGION 1 (Sec. 3.3; Alg. 1, the capacity check in front of the append).
 * sk_session_freeze marks the first n_frozen tokens of the session as Region 0: they are never
 * evicted.  n_frozen may only grow, must not exceed the session's length, and cannot change once
 * tokens have been evicted behind it (SK_E_INVAL).
 * sk_session_evict_oldest removes the n_tokens oldest tokens that are not frozen (FIFO eviction
 * of the sliding Region 1); more than the session holds there gives SK_E_INVAL and changes
 * nothing.  Attention then runs over [Region 0 ; what is left of Region 1]; the order of the
 * retained tokens is kept, and sk_session_length / gather / truncate count retained tokens only.
 * Re-encoding positions after an eviction is the caller's concern (as for every K the cache is
 * given).  Metadata only: blocks that hold nothing but evicted tokens return to the free list at
 * once; evicted tokens that share a block with retained ones stay in kv_mem and are skipped by
 * the kernels.  The only device work is a copy of the moved part of the session's block table,
 * ordered on hip_stream (which must be the stream of the session's other calls).
 */
int sk_session_freeze(sk_pool* pool, int32_t id, int64_t n_frozen);
int sk_session_evict_oldest(sk_pool* pool, int32_t id, int64_t n_tokens, void* hip_stream);

/*
 * FORK (Sec. 3.7 prefix-aware grouped prefill: followers alias the leader's state; Sec. 3.10
 * metadata-only sequence aliasing).  Creates a session whose cache is the first n_prefix retained
 * tokens of session src (including src's frozen region and evicted range as far as the prefix
 * reaches).  The blocks of the prefix are shared, not copied (per-block reference counts; a
 * block returns to the free list when its last holder drops it); only when the prefix ends
 * inside a block does the new session get a copy of that one block, into which its own appends
 * then go.  Cost: n_prefix / block_tokens table entries and at most one block of K/V, whatever the
 * prefix length.  Afterwards the two sessions are independent: appends, evictions, truncations
 * and destruction of one never change what the other reads.  A shared block is never written:
 * when a truncation has left a session's end inside one, that session's next append first
 * replaces the block by a copy of its own (one more free block needed, part of the append's
 * all-or-nothing check; the copy is ordered on the append's stream).
 * The device work (table upload, block copy) is ordered on hip_stream, which must be the stream
 * of src's earlier calls.  SK_E_NOMEM when no session id or (if needed) no block is free.
 */
int sk_session_fork(sk_pool* pool, int32_t src, int64_t n_prefix, int32_t* out_id, void* hip_stream);

/*
 * GREEDY SAMPLING WITH A CONFIDENCE GAP (Sec. 3.8 on-device greedy sampling: the argmax of a
 * ~128k-entry logit row is taken on the device instead of copying the row to the host;
 * Sec. 3.9.2 confidence gamma = top-1 logit - top-2 logit; Sec. 3.9.4 Delta_ready).
 * Independent of any pool.  logits: DEVICE float32 [rows][row_stride], the first `vocab` entries
 * of a row count; 16-byte aligned, row_stride a multiple of 4, vocab >= 2, rows <= 65535.
 * Outputs, DEVICE, one per row: idx1 = lowest index of the row maximum, idx2 = lowest index of
 * the maximum among the other entries (int32); val1, val2 = those logits, gap = val1 - val2 in
 * fp32 (each of the three may be NULL).  Equal logits: the lower index comes first (the paper
 * does not say).  Logits are assumed not to be NaN.
 * workspace: DEVICE scratch of sk_top2_workspace_bytes(rows, vocab) bytes, 16-byte aligned,
 * owned by the caller (the library allocates nothing); too small gives SK_E_WORKSPACE.
 */
size_t sk_top2_workspace_bytes(int32_t rows, int32_t vocab);
int sk_top2(const float* logits, int32_t rows, int32_t vocab, int64_t row_stride,
            void* workspace, size_t workspace_bytes,
            int32_t* idx1, int32_t* idx2, float* val1, float* val2, float* gap, void* hip_stream);

/*
 * sk_top2 for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the
 * workspace, same kernels, same results bit for bit.  The first-pass pairs go to a fixed array
 * inside the library's device image instead (SK_TOP2_STATIC_BYTES, held by every GPU the library
 * runs on until the process ends), so rows * ceil(vocab / 8192) * 16 bytes must not exceed that:
 * otherwise SK_E_WORKSPACE, and nothing is launched.  The call allocates nothing and frees nothing.
 * The array's device address is looked up once per device, on the first call there (with that
 * device current); a call with rows == 0 does only that, so a caller can get it out of the way
 * before a capture.  Every call on a GPU uses that GPU's one array: calls that overlap in time on
 * one GPU (two streams, two threads) race and must be ordered by the caller; nothing in the array
 * needs clearing between calls (the first pass writes every entry the second reads).
 */
enum { SK_TOP2_STATIC_BYTES = 1 << 20 };
int sk_top2_static(const float* logits, int32_t rows, int32_t vocab, int64_t row_stride,
                   int32_t* idx1, int32_t* idx2, float* val1, float* val2, float* gap, void* hip_stream);

/* Byte offset inside kv_mem of element (block, kv_head, is_v, slot, dim), so a harness can
 * address the pool without knowing the layout.  Negative on bad arguments. */
int64_t sk_pool_element_offset(const sk_pool* pool, int64_t block, int32_t kv_head, int32_t is_v,
                               int32_t slot, int32_t dim);

/* Counters since creation: tokens appended, query tokens, kernel launches, cached-token
 * bytes the attention kernels were asked to stream, tokens evicted, sessions forked. */
typedef struct sk_pool_stats {
    int64_t tokens_appended, tokens_queried, launches, kv_bytes_streamed, tokens_evicted, forks;
} sk_pool_stats;
int sk_pool_get_stats(const sk_pool* pool, sk_pool_stats* out);

/* Launch geometry of the most recent attention call (for checking that it depends on the
 * shapes only, not on how the cache was built): workgroups, splits per row tile, row tiles. */
typedef struct sk_launch_info {
    int32_t workgroups, n_splits, row_tiles, kernel_variant;
    int32_t fused_merge;   /* 1: the split partials were merged inside the attention kernel */
    int32_t reserved[3];
} sk_launch_info;
int sk_pool_last_launch(const sk_pool* pool, sk_launch_info* out);

/*
 * Optional timing of the kernels themselves, for benchmarks: while enabled, every attention and
 * combine kernel is launched with a pair of events that the runtime fills with the dispatch's own
 * start and end time stamps (what a profiler reports as the kernel's duration; nothing is recorded
 * on the stream between kernels).  sk_pool_read_profile waits for the recorded events, returns the
 * sums since the last read (and, if the arrays are given, the first `capacity` calls one by one, in
 * call order, in milliseconds: the attention kernels of a call added up, and its combine kernels) and
 * clears them.  At most 16,384 kernel dispatches are kept between reads.
 */
typedef struct sk_profile {
    int64_t calls;
    double attention_ms;   /* attention kernel(s) */
    double combine_ms;     /* cross-split combine kernel(s) */
} sk_profile;
int sk_pool_set_profiling(sk_pool* pool, int enable);
int sk_pool_read_profile(sk_pool* pool, sk_profile* out, float* attention_ms_per_call /*HOST or NULL*/,
                         float* combine_ms_per_call /*HOST or NULL*/, int32_t capacity);

/*
 * Measurement probes (benchmarks only; the attention path does not call them).
 * sk_probe_read: a plain streaming read of `bytes` bytes at src (DEVICE, 16-byte aligned) by
 * n_workgroups workgroups of 256 threads, 16 bytes per load (non_temporal != 0: with the cache
 * policy for data used once); the time it takes is the floor of anything that has to read that
 * many bytes once (Sec. 3.2: a query reads the cache once).
 * sk_probe_mfma: n_workgroups workgroups of eight waves, each wave `iters` rounds of eight bf16
 * 32x32x16 matrix products on register operands, read once from `operands` (DEVICE, bf16 data of
 * the caller's choice, operand_bytes >= 64, 16-byte aligned; the rate the pipe sustains depends on
 * how much the operand bits toggle) or, with operands NULL, made up in the kernel; *flops_out
 * (HOST, optional) receives the floating-point operations of the launch.  sink: DEVICE, 4 bytes,
 * in practice never written.
 */
int sk_probe_read(const void* src, size_t bytes, int32_t n_workgroups, int32_t non_temporal, void* sink, void* hip_stream);
int sk_probe_mfma(int32_t n_workgroups, int32_t iters, const void* operands, size_t operand_bytes, void* sink,
                  double* flops_out, void* hip_stream);

/*
 * Test hook for the error paths: the countdown-th time the pool reaches `site` from now on, that
 * step fails as if its HIP call had (SK_E_HIP; SK_SITE_PLAN: SK_E_WORKSPACE) without touching the
 * device.  Metadata-only pools pass the same sites, so the taking back of a half-done call can be
 * checked without a GPU.  countdown 0 disarms.
 */
enum { SK_SITE_NONE = 0, SK_SITE_RING = 1,   /* waiting for a pinned upload slot */
       SK_SITE_UPLOAD = 2,                   /* host-to-device copy of a list or block table */
       SK_SITE_BLOCK_COPY = 3,               /* copy of a shared or partly filled block */
       SK_SITE_SCATTER = 4, SK_SITE_ATTENTION = 5, SK_SITE_COMBINE = 6,   /* kernel launches */
       SK_SITE_PLAN = 7 };                   /* the lists of a batched call do not fit */
int sk_pool_inject_failure(sk_pool* pool, int32_t site, int32_t countdown);

const char* sk_strerror(int status);     /* static storage */
int sk_last_hip_error(void);             /* hipError_t of the last failing HIP call in this thread */
int sk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SK_H */
