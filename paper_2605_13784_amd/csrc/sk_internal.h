// Internal structures shared by the host planner (sk_pool.cpp) and the kernels
// (sk_kernels.hip).  Not part of the C ABI.
#pragma once
#include <stdint.h>
#include <stddef.h>

// ---------------------------------------------------------------------------------------------
// Pool geometry (constant for the life of a pool).
//
// kv_mem layout, chosen for gfx950: [kv_head][block][ K | V ] with, per (head, block),
//   K : [block_tokens][head_dim]            one 128/256-byte row per token
//   V : bf16 pools  [block_tokens / 16][head_dim][16]  (transposed within each 16-token group:
//                   8 consecutive tokens of one dimension are one 16-byte MFMA operand for the
//                   P*V contraction)
//       f32 pools   [block_tokens][head_dim]
// so a 16-token group of one head is a contiguous 4 KiB (bf16, d=128) for K and for V whatever
// the block size, every
// global load is a whole 128-byte line, and the blocks of one head (what one workgroup
// streams) are contiguous when a session's table is in order.
// The staging area for uncommitted (query-plane) K/V in the workspace has the same layout
// with 16-token blocks and an identity block table.
// ---------------------------------------------------------------------------------------------
struct sk_geom {
    const unsigned char* kv;      // pool base
    const unsigned char* eph;     // staging base (workspace)
    const int32_t* tables;        // device block tables, [max_sessions][max_blocks_per_session]
    const int32_t* eph_ident;     // identity table 0,1,2,.. over the staging blocks
    int64_t blk_stride;           // bytes from one block to the next (same head)
    int64_t head_stride;          // bytes from one KV head to the next (same block)
    int64_t eph_blk_stride;       // the same two for the staging area (16-token blocks)
    int64_t eph_head_stride;
    int32_t v_off;                // byte offset of V inside (block, head)
    int32_t eph_v_off;
    int32_t B, log2B;             // pool block_tokens
    int32_t Hq, Hkv, G, log2G;    // log2G = -1 when G is not a power of two (informational: the kernels divide by G)
    int32_t d;
    int32_t elem;                 // bytes per element (2 or 4)
    float scale_log2e;            // softmax scale * log2(e)
    int32_t pad;
};

#define SK_NO_CAUSAL (1 << 30)    // pos0 at or above this: rows see every key of every segment

// One workgroup of an attention kernel: a tile of query rows of one KV head against a range of
// cached tokens plus up to two uncommitted segments.
struct sk_work {
    int32_t tbl_off;      // int32 offset of the session's block table in sk_geom::tables
    int32_t kv_head;
    int32_t q_tok0;       // first packed token row of the tile in q/out/lse
    int32_t n_tok;        // tokens in the tile (rows = n_tok * G)
    int32_t pos0;         // absolute position of token q_tok0; token i sits at pos0 + i
    int32_t kv_begin;     // cached tokens [kv_begin, kv_end) (positions = token index)
    int32_t kv_end;
    int32_t part;         // partial slot, or -1: the only split, final output written directly
    int32_t eph_blk[2];   // first staging block of each uncommitted segment
    int32_t eph_cnt[2];   // tokens in it (0 = absent)
    int32_t eph_pos0[2];  // absolute position of its first token
    int32_t hole_lo;      // cached tokens [hole_lo, hole_hi) are evicted (Region-1 FIFO eviction): their
    int32_t hole_hi;      // blocks are still streamed, the keys never attended to; empty when lo == hi
    int32_t tok_period;   // > 0: the tile packs sequences of tok_period tokens each, all starting at pos0;
    int32_t sub_blocks;   // sequence k's second uncommitted segment starts at staging block eph_blk[1] + k * sub_blocks
    int32_t kv_step;      // keys from one 64-key iteration over [kv_begin, kv_end) to the next; 0 = 64 (contiguous)
    // in-kernel merge of the split partials (part >= 0 and sk_launch::fuse): the workgroups of one
    // (row tile, KV head) are a unit; its partial slots are part0, part0 + Hkv, .. (n_parts of them)
    int32_t unit;         // index of the unit's pair of counters in sk_launch::sync
    int32_t part0;
    int32_t n_parts;
};

// One row tile of the cross-split combine.
struct sk_comb {
    int32_t part0, n_parts, part_stride;
    int32_t q_tok0, n_tok, kv_head;
    int32_t pad[2];
};

// One destination 16-token group of one scatter (commit or staging).
struct sk_scatter {
    int64_t dst_off;      // byte offset of the destination block in kv_mem or staging
    int32_t src_tok0;     // first packed token row in k/v
    int32_t count;        // tokens (1..16), all inside one 16-token group of the block
    int32_t dst_slot0;    // slot of the first token inside the destination block
    int32_t to_eph;       // 0: pool (block size B), 1: staging (block size 16)
    int32_t tbl_index;    // >= 0: also write tables[tbl_index] = block_id
    int32_t block_id;
};

// A short scatter list that travels in the kernel arguments.
#define SK_SCATTER_ARGS_MAX 80
struct sk_scatter_list { sk_scatter item[SK_SCATTER_ARGS_MAX]; };

enum { SK_MODE_REGULAR = 0, SK_MODE_LIST = 1 };
// attention kernel variants: fp32-FMA kernel; bf16 MFMA kernel with 128-, 64- and 256-row tiles; the
// 128-row tile again with eight waves (two key phases per row group, one workgroup per CU)
enum { SK_KV_SIMPLE = 0, SK_KV_MFMA128 = 1, SK_KV_MFMA64 = 2, SK_KV_MFMA256 = 3, SK_KV_MFMA128P = 4 };

// Kernel argument block of the attention and combine kernels.
struct sk_launch {
    sk_geom g;
    const void* q;
    void* out;
    float* lse;
    float* part_ml;       // [slot][rows_per_slot][4]  (reference maximum in log2 units, sum of the weights as
                          //  rounded for the matrix pipe, sum of the unrounded weights, unused)
    float* part_o;        // [slot][rows_per_slot][d]  unnormalised
    const sk_work* work;  // list mode
    const sk_comb* comb;  // list mode
    int32_t out_dtype;
    int32_t mode;
    int32_t rows_per_slot;   // rows reserved per partial slot (tile height of the variant)
    // regular mode: one session, n_tok tokens cut into n_tiles tiles of tok_per_tile tokens,
    // cached tokens cut into n_splits chunks of `chunk` tokens.
    int32_t tbl_off, n_tok, tok_per_tile, n_tiles, pos0, kv_len, chunk, n_splits;
    int32_t eph_blk[2], eph_cnt[2], eph_pos0[2];
    int32_t hole_lo, hole_hi;    // evicted cached tokens of the session (regular mode)
    // regular mode, no causal limit inside the cached range: split s takes the 64-key pieces s, s + S,
    // s + 2S, .. of the cache instead of one contiguous chunk, so that the workgroups of a head walk
    // through memory side by side instead of as S separate streams (the host decides when)
    int32_t interleave;
    // In-kernel merge of the split partials (optional; the default is the combine kernel, which
    // measured faster).  sync holds two counters per unit, both zero between
    // launches: arrivals (low 16 bits; the high bits count workgroups that gave up waiting) and
    // departures.  A workgroup writes its partial, arrives, and waits up to wait_polls polls for the
    // others; then every workgroup of the unit merges its own share of the rows.  One that gives up
    // leaves its share to the last arriver, which always sees everything (no wait is unbounded).
    // The last to leave clears the counters.
    uint32_t* sync;
    int32_t fuse;
    int32_t wait_polls;
    int32_t merge_fences;   // 1: full device-scope fences around the arrival (slow: an L2 walk each); 0: see the kernel
    int32_t kv_once;        // 1: every key is read by exactly one workgroup of the launch (loaded non-temporal)
};

// Launchers implemented in sk_kernels.hip (return hipError_t as int).
int sk_launch_scatter(const sk_geom& g, const void* k, const void* v, const sk_scatter* items,
                      int32_t n_items, int32_t* tables_rw, unsigned char* kv_rw,
                      unsigned char* eph_rw, void* stream);
int sk_launch_scatter_args(const sk_geom& g, const void* k, const void* v, const sk_scatter_list& items,
                           int32_t n_items, int32_t* tables_rw, unsigned char* kv_rw,
                           unsigned char* eph_rw, void* stream);
int sk_launch_attention(const sk_launch& L, int variant, int32_t n_workgroups, void* stream, void* ev_start, void* ev_stop);
int sk_launch_combine(const sk_launch& L, int32_t n_row_tiles, void* stream, void* ev_start, void* ev_stop);
int sk_launch_gather(const sk_geom& g, int32_t tbl_off, int64_t first, int64_t count,
                     void* k_out, void* v_out, void* stream);
int sk_launch_copy_block(const sk_geom& g, unsigned char* kv_rw, int32_t src, int32_t dst, void* stream);
