// Host side of the library: pool bookkeeping (free list, sessions, block tables), argument
// checks, the planner that cuts a call into workgroups, and the C ABI of include/sk.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <new>
#include <vector>

#include "../../include/sk.h"
#include "sk_internal.h"

namespace {

thread_local int g_last_hip = 0;

constexpr int kRingSlots = 4;
constexpr size_t kMinMetaBytes = 4u << 20;       // least size of the device region for uploaded lists (= ring slot size)
constexpr int kPartSlotRows = 128;               // rows reserved per partial slot
constexpr int kDefaultTargetWgs = 512;
constexpr int kDefaultWaitPolls = 256;           // polls a workgroup waits for the others of its unit (about 1 us each)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ilog2_exact(int64_t x) { int l = 0; while ((int64_t(1) << l) < x) ++l; return ((int64_t(1) << l) == x) ? l : -1; }

// A session's tokens live at *storage indices* 0 .. len-1; block i of `blocks` holds storage
// indices i*B .. i*B+B-1.  Storage indices [frozen, win) are evicted (Region-1 FIFO eviction behind
// a frozen Region 0): what the session holds is [0, frozen) followed by [win, len).  Whole blocks
// inside the hole are returned to the pool and the storage indices behind them shifted down, so
// the hole always spans less than two blocks; what is left of it is masked in the kernels.
struct Session {
    bool live = false;
    int64_t len = 0;
    int64_t frozen = 0, win = 0;
    std::vector<int32_t> blocks;
    int64_t retained() const { return frozen + (len - win); }
};

struct Layout {
    int elem = 0, G = 0;
    int64_t head_stride = 0, blk_stride = 0, v_off = 0;
    int64_t eph_head_stride = 0, eph_blk_stride = 0, eph_v_off = 0;
    int64_t max_blocks_per_session = 0, max_session_tokens = 0;
    int32_t max_batch_tokens = 0;
    int64_t eph_blocks = 0;
    int64_t part_slots = 0;
    int64_t sync_units = 0;           // pairs of merge counters
    size_t meta_bytes = 0;            // device region for uploaded lists; also the size of a pinned ring slot
    size_t kv_bytes = 0;
    // workspace offsets
    size_t off_tables = 0, off_ident = 0, off_meta = 0, off_sync = 0, off_part_ml = 0, off_part_o = 0, off_eph = 0, ws_bytes = 0;
};

bool derive_layout(const sk_pool_desc& d, Layout& L)
{
    if (d.dtype != SK_F32 && d.dtype != SK_BF16) return false;
    if (d.n_kv_heads <= 0 || d.n_q_heads <= 0 || d.n_q_heads % d.n_kv_heads) return false;
    if (d.head_dim != 64 && d.head_dim != 128) return false;
    if (d.block_tokens < 16 || d.block_tokens > 1024 || ilog2_exact(d.block_tokens) < 0) return false;
    if (d.n_blocks <= 0 || d.n_blocks > (int64_t(1) << 30) || d.max_sessions <= 0 || d.max_sessions > (1 << 20)) return false;
    if (d.max_session_tokens < 0 || d.max_batch_tokens < 0) return false;
    L.elem = d.dtype == SK_F32 ? 4 : 2;
    L.G = d.n_q_heads / d.n_kv_heads;
    L.v_off = int64_t(d.block_tokens) * d.head_dim * L.elem;
    // [kv_head][block][K | V]: the blocks of one head are contiguous, so a workgroup (which
    // streams one head) reads whole consecutive 8 KiB pieces when the table is in order
    L.blk_stride = 2 * L.v_off;
    L.head_stride = L.blk_stride * d.n_blocks;
    L.eph_v_off = int64_t(16) * d.head_dim * L.elem;
    L.eph_blk_stride = 2 * L.eph_v_off;
    L.eph_head_stride = 0;     // set once the number of staging blocks is known
    int64_t mst = d.max_session_tokens ? d.max_session_tokens : d.n_blocks * d.block_tokens;
    mst = std::min<int64_t>(mst, d.n_blocks * d.block_tokens);
    mst = std::min<int64_t>(mst, int64_t(kMinMetaBytes / 4) * d.block_tokens);    // a session's block table is uploaded in one piece
    if (mst > (int64_t(1) << 29)) return false;       // positions are int32 with head room
    L.max_session_tokens = mst;
    L.max_blocks_per_session = (mst + d.block_tokens - 1) / d.block_tokens;
    // offsets into the device block tables are 32-bit
    if (int64_t(d.max_sessions) * L.max_blocks_per_session >= (int64_t(1) << 31)) return false;
    L.max_batch_tokens = d.max_batch_tokens ? d.max_batch_tokens : 4096;
    if (L.max_batch_tokens > (1 << 20)) return false;
    {   // The lists a batched call uploads always fit when every row tile is one workgroup per KV head
        // (the planner falls back to that): a call has at most max_batch_tokens tokens in at most
        // min(max_sessions, max_batch_tokens) items (question batches: one tile per question at worst),
        // so at most tiles_max row tiles and scat_max 16-token scatter groups.
        const int64_t items_max = std::min<int64_t>(std::max(d.max_sessions, 1024), L.max_batch_tokens);
        const int64_t tpt_min = std::max(1, 16 / L.G);                          // tokens per row tile of the smallest kernel
        const int64_t tiles_max = L.max_batch_tokens / tpt_min + items_max;
        const int64_t scat_max = L.max_batch_tokens / 16 + 2 * items_max + 2;
        const int64_t need = tiles_max * d.n_kv_heads * int64_t(sizeof(sk_work) + sizeof(sk_comb)) + scat_max * int64_t(sizeof(sk_scatter)) + 16 * 256;
        // Capped at 64 MiB: a step whose lists do not fit even then is refused with SK_E_WORKSPACE and
        // leaves every session as it was.
        L.meta_bytes = align_up(std::max<size_t>(kMinMetaBytes, std::min<size_t>(size_t(need), size_t(64) << 20)), 256);
    }
    L.eph_blocks = (L.max_batch_tokens + 15) / 16 + std::max(d.max_sessions, 1024) + 1;
    L.eph_head_stride = L.eph_blk_stride * L.eph_blocks;
    int64_t rows = int64_t(L.max_batch_tokens) * d.n_q_heads;
    L.part_slots = 2048 + 2 * ((rows + kPartSlotRows - 1) / kPartSlotRows);
    L.kv_bytes = size_t(2 * L.v_off) * size_t(d.n_kv_heads) * size_t(d.n_blocks);
    size_t off = 0;
    L.off_tables = off; off = align_up(off + size_t(d.max_sessions) * L.max_blocks_per_session * 4, 256);
    L.off_ident = off;  off = align_up(off + size_t(L.eph_blocks) * 4, 256);
    L.off_meta = off;   off = align_up(off + L.meta_bytes, 256);
    // one unit of merge counters per (row tile, KV head) of a call; the matrix-pipe kernels, which merge
    // in the kernel, have tiles of at least 64 rows
    L.sync_units = (rows / 64 + std::max(d.max_sessions, 1024) + 2) * d.n_kv_heads;
    L.off_sync = off;   off = align_up(off + size_t(L.sync_units) * 8, 256);
    L.off_part_ml = off; off = align_up(off + size_t(L.part_slots) * kPartSlotRows * 4 * 4, 256);
    L.off_part_o = off; off = align_up(off + size_t(L.part_slots) * kPartSlotRows * d.head_dim * 4, 256);
    L.off_eph = off;    off = align_up(off + size_t(L.eph_blocks) * L.eph_blk_stride * d.n_kv_heads, 256);
    L.ws_bytes = off;
    return true;
}

}  // namespace

struct sk_pool {
    sk_pool_desc d;
    Layout L;
    bool device = false;
    std::deque<int32_t> free_blocks;
    std::vector<Session> sessions;
    std::vector<int32_t> free_ids;
    int64_t blocks_in_use = 0;
    std::vector<int32_t> refcnt;         // sessions holding each block (forks share the blocks of a prefix)
    // pinned staging ring for uploaded lists
    unsigned char* ring = nullptr;
    hipEvent_t ring_ev[kRingSlots] = {};
    bool ring_used[kRingSlots] = {};
    int ring_next = 0;
    sk_geom geom;
    sk_pool_stats stats = {};
    sk_launch_info last = {};
    // Tuning switches, read from the environment once when the pool is created (see sk_pool_create).
    int target_wgs = kDefaultTargetWgs;
    bool target_wgs_set = false;
    bool force_simple = false, no_256 = false, no_pack = false, no_interleave = false, no_stream_loads = false;
    bool p128 = true;                    // SK_NO_P128=1: never the eight-wave 128-row instance
    int64_t p128_min_tokens = 30720;     // SK_P128_MIN_TOKENS: cached tokens from which it is taken (break-even measured near 32K)
    int64_t stream_min_tokens = 65536;   // SK_STREAM_MIN_TOKENS: cached tokens from which the 128-row instances load non-temporal
    bool fuse = false;                   // SK_FUSE=1: single-session calls merge their split partials inside the attention kernel
    bool fuse_list = false;              // batched calls too (the last workgroup of a unit merges alone)
    bool merge_fences = false;           // SK_MERGE_FENCES=1: full fences around the arrival (for comparison)
    int wait_polls = kDefaultWaitPolls;
    int n_cus = 256;                     // compute units of the device the pool was created on
    // test hook (sk_pool_inject_failure): the countdown-th arrival at `inject_site` fails
    int inject_site = 0, inject_countdown = 0;
    // optional kernel timing
    bool profiling = false;
    struct ProfRec { hipEvent_t start, stop; int32_t call, kind; };   // one kernel dispatch; kind 0 attention, 1 combine
    std::vector<ProfRec> prof;           // records (events are created once and reused)
    size_t prof_used = 0;                // records in use
    int32_t prof_calls = 0;              // calls since the last read
};

namespace {

#define SK_HIP(expr)                                        \
    do {                                                    \
        hipError_t e_ = (expr);                             \
        if (e_ != hipSuccess) { g_last_hip = (int)e_; return SK_E_HIP; } \
    } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

Session* get_session(sk_pool* p, int32_t id)
{
    if (!p || id < 0 || id >= (int32_t)p->sessions.size() || !p->sessions[id].live) return nullptr;
    return &p->sessions[id];
}
const Session* get_session(const sk_pool* p, int32_t id) { return get_session(const_cast<sk_pool*>(p), id); }

int64_t blocks_needed(const sk_pool* p, int64_t len, int64_t add)
{
    const int64_t B = p->d.block_tokens;
    return (len + add + B - 1) / B - (len + B - 1) / B;
}

// Test hook: true when a failure was ordered for this site and its countdown has run out.  The sites
// are visited in the same order by device pools and by metadata-only pools (which skip the HIP call
// itself), so the error paths behind them can be exercised without a GPU.
bool inject(sk_pool* p, int site)
{
    if (p->inject_site != site || p->inject_site == 0) return false;
    if (--p->inject_countdown > 0) return false;
    p->inject_site = 0;
    g_last_hip = (int)hipErrorUnknown;
    return true;
}

// Takes a ring slot (waiting for the copy that last used it), returns its host pointer (null for a
// metadata-only pool).  Changes nothing when it fails.
int ring_acquire(sk_pool* p, int* slot, unsigned char** host)
{
    if (inject(p, SK_SITE_RING)) return SK_E_HIP;
    *slot = 0; *host = nullptr;
    if (!p->device) return SK_OK;
    int s = p->ring_next;
    if (p->ring_used[s]) SK_HIP(hipEventSynchronize(p->ring_ev[s]));
    p->ring_next = (s + 1) % kRingSlots;
    *slot = s;
    *host = p->ring + size_t(s) * p->L.meta_bytes;
    return SK_OK;
}

// Copies `bytes` from ring slot `slot` to `dev` on the stream and marks the slot busy until then.
int ring_copy(sk_pool* p, int slot, void* dev, size_t bytes, hipStream_t st)
{
    if (inject(p, SK_SITE_UPLOAD)) return SK_E_HIP;
    if (!p->device) return SK_OK;
    SK_HIP(hipMemcpyAsync(dev, p->ring + size_t(slot) * p->L.meta_bytes, bytes, hipMemcpyHostToDevice, st));
    if (hipEventRecord(p->ring_ev[slot], st) != hipSuccess) (void)hipStreamSynchronize(st);   // the slot is free either way
    p->ring_used[slot] = true;
    return SK_OK;
}

int ring_upload(sk_pool* p, int slot, size_t bytes, hipStream_t st)
{
    return ring_copy(p, slot, p->device ? (unsigned char*)p->d.workspace + p->L.off_meta : nullptr, bytes, st);
}

// With profiling on: a call announces itself (prof_call) and asks for a pair of events per kernel
// it launches (prof_pair); the launchers hand them to the runtime, which stamps them with the
// dispatch's own start and end times.
constexpr size_t kProfMax = 4 * 4096;
int32_t prof_call(sk_pool* p) { return p->profiling ? p->prof_calls++ : -1; }
bool prof_pair(sk_pool* p, int32_t call, int32_t kind, void** start, void** stop)
{
    *start = *stop = nullptr;
    if (call < 0 || p->prof_used >= kProfMax) return false;
    if (p->prof.size() <= p->prof_used) {
        sk_pool::ProfRec r = {};
        if (hipEventCreate(&r.start) != hipSuccess) return false;
        if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return false; }
        p->prof.push_back(r);
    }
    sk_pool::ProfRec& r = p->prof[p->prof_used++];
    r.call = call; r.kind = kind;
    *start = r.start; *stop = r.stop;
    return true;
}

// Which attention kernel takes a tile of `max_rows` query rows per KV head.
struct Variant { int id; int rows_per_slot; int tok_per_tile; };

// `allow_256`: the caller can launch one workgroup per CU (single-session calls), which the
// 256-row tile with its 128 KiB key ring needs.
bool pick_variant(const sk_pool* p, int64_t n_tok, Variant& v, bool allow_256 = false)
{
    const int G = p->L.G;
    // any group size up to 128 (multi-query models): a tile holds floor(rows / G) tokens, at least one;
    // head_dim 64 has no 256-row instance
    const bool mfma_ok = p->d.dtype == SK_BF16 && (p->d.head_dim == 128 || p->d.head_dim == 64) && G <= 128;
    if (mfma_ok && !p->force_simple) {
        if (allow_256 && p->d.head_dim == 128 && n_tok * G > 128) { v.id = SK_KV_MFMA256; v.rows_per_slot = 256; v.tok_per_tile = 256 / G; }
        else if (n_tok * G > 64 || G > 64) { v.id = SK_KV_MFMA128; v.rows_per_slot = 128; v.tok_per_tile = 128 / G; }
        else { v.id = SK_KV_MFMA64; v.rows_per_slot = 64; v.tok_per_tile = 64 / G; }
        return true;
    }
    if (G > 16) return false;
    v.id = SK_KV_SIMPLE; v.rows_per_slot = 16; v.tok_per_tile = std::max(1, 16 / G);
    return true;
}

void fill_launch_common(const sk_pool* p, sk_launch& L, const void* q, void* out, int out_dtype, float* lse, const Variant& v)
{
    memset(&L, 0, sizeof L);
    L.g = p->geom;
    L.q = q; L.out = out; L.lse = lse;
    unsigned char* ws = (unsigned char*)p->d.workspace;
    L.part_ml = (float*)(ws + p->L.off_part_ml);
    L.part_o = (float*)(ws + p->L.off_part_o);
    L.sync = (uint32_t*)(ws + p->L.off_sync);
    L.out_dtype = out_dtype == SK_F32 ? 0 : 1;
    L.rows_per_slot = v.rows_per_slot;
}

// Regular-mode attention over one session: n_tok new tokens at positions pos0.. (or no causal
// limit), kv_len cached tokens, optionally one uncommitted segment already in staging block 0.
// plan_regular decides the decomposition and is the only part that can refuse the call (it reads
// nothing but sizes, so it runs before a call changes anything); launch_regular enqueues it.
struct RegPlan {
    Variant v;
    sk_launch L;           // everything but the pointers
    int32_t wgs = 0, base_wgs = 0, parts = 1;
    int64_t kv_len = 0;
};

int plan_regular(const sk_pool* p, int32_t id, int64_t n_tok, int32_t pos0, int64_t kv_len, int32_t eph_cnt, int32_t eph_pos0,
                 int64_t hole_lo, int64_t hole_hi, int32_t n_splits_req, RegPlan& R)
{
    Variant& v = R.v;
    if (!pick_variant(p, n_tok, v, !p->no_256)) return SK_E_SHAPE;
    sk_launch& L = R.L;
    memset(&L, 0, sizeof L);
    L.rows_per_slot = v.rows_per_slot;
    L.mode = SK_MODE_REGULAR;
    L.tbl_off = int32_t(int64_t(id) * p->L.max_blocks_per_session);
    L.n_tok = (int32_t)n_tok;
    L.tok_per_tile = v.tok_per_tile;
    L.n_tiles = int32_t((n_tok + v.tok_per_tile - 1) / v.tok_per_tile);
    L.pos0 = pos0;
    L.kv_len = (int32_t)kv_len;
    const int64_t base_wgs = int64_t(L.n_tiles) * p->d.n_kv_heads;
    const int64_t slots_rows = p->L.part_slots * kPartSlotRows;
    const int has_eph = eph_cnt > 0 ? 1 : 0;
    int64_t S;
    if (n_splits_req > 0) S = n_splits_req;
    else {
        // A call with few row tiles (a query) is bound by streaming the cache once: one workgroup
        // per CU measured faster than two (fewer split partials to write and merge).  Calls with
        // many row tiles (appends) are bound by arithmetic and want two workgroups per CU.
        const int64_t target = p->target_wgs_set ? p->target_wgs : ((L.n_tiles <= 2 || v.id == SK_KV_MFMA256) ? 256 : 512);
        S = std::max<int64_t>(1, (target + base_wgs / 2) / base_wgs);
    }
    int64_t chunk = kv_len > 0 ? (kv_len + S - 1) / S : 64;
    // at least four 64-key iterations per workgroup of the matrix-pipe kernels; the fp32-FMA kernel
    // (32-key tiles, far slower per key) takes shorter pieces so that small caches still spread over the chip
    if (n_splits_req <= 0) chunk = std::max<int64_t>(chunk, v.id == SK_KV_SIMPLE ? 64 : 256);
    chunk = (chunk + 63) / 64 * 64;
    S = kv_len > 0 ? (kv_len + chunk - 1) / chunk : 0;
    int64_t parts = std::max<int64_t>(1, S + has_eph);
    // respect the partial-slot capacity
    while (parts > 1 && base_wgs * parts * v.rows_per_slot > slots_rows) {
        chunk *= 2;
        S = kv_len > 0 ? (kv_len + chunk - 1) / chunk : 0;
        parts = std::max<int64_t>(1, S + has_eph);
        if (S <= 1) break;
    }
    if (parts > 1 && base_wgs * parts * v.rows_per_slot > slots_rows) return SK_E_WORKSPACE;
    if (base_wgs * parts > (int64_t(1) << 30)) return SK_E_WORKSPACE;
    L.chunk = (int32_t)chunk;
    L.n_splits = (int32_t)parts;
    L.eph_blk[0] = 0; L.eph_cnt[0] = eph_cnt; L.eph_pos0[0] = eph_pos0;
    L.hole_lo = (int32_t)hole_lo; L.hole_hi = (int32_t)hole_hi;
    // Small queries (at most 64 rows per KV head; every cached token visible to every row): the splits
    // interleave their 64-key pieces.  Measured 3-5 % faster there (16 tokens at 128K: 99.5 -> 96 us),
    // 2-3 % slower for the 128-row instance, which keeps contiguous chunks.  Larger blocks gain more
    // (16 tokens at 128K: 98 / 96 / 92 us with 16- / 64- / 256-token blocks).
    L.interleave = (!p->no_interleave && v.id == SK_KV_MFMA64 && S > 1 && kv_len <= (int64_t)pos0) ? 1 : 0;
    R.base_wgs = (int32_t)base_wgs; R.parts = (int32_t)parts; R.wgs = int32_t(base_wgs * parts); R.kv_len = kv_len;
    // On request (SK_FUSE=1) the matrix-pipe kernels merge their split partials themselves (one launch per
    // call).  Workgroups only wait for each other when the whole launch fits on the device at once (the
    // 256-row instance holds a CU alone, the others share it in pairs); otherwise the last workgroup of a
    // unit merges alone.  Not the default: a device-scope round trip (atomic, coherent load) measured about
    // 3 us on this hardware and the scheme needs four in a row, against 6-7 us for the combine kernel.
    const bool mfma = v.id != SK_KV_SIMPLE;
    // A 128-row call that gives every CU at most one workgroup takes the eight-wave instance: two key
    // phases per row group, so a wave has half the arithmetic per 64 keys and its SIMD a second wave
    // to overlap it with.  Measured (32-token query, us per query, four waves -> eight): 2,600 cached
    // tokens 18.5 -> 20.1, 8K 22.8 -> 24.7, 14,800 28.3 -> 29.4, 32K 42.3 -> 42.1, 64K 69.5 -> 65.3,
    // 128K 123.8 -> 113.2: the eight waves pay off once the stream outweighs their longer start and
    // their merge of the two phases.
    if (p->p128 && v.id == SK_KV_MFMA128 && R.wgs <= p->n_cus && kv_len >= p->p128_min_tokens) v.id = SK_KV_MFMA128P;
    L.fuse = (p->fuse && mfma && parts > 1 && base_wgs <= p->L.sync_units && parts < 65536) ? 1 : 0;
    const int64_t resident = int64_t(p->n_cus) * ((v.id == SK_KV_MFMA256 || v.id == SK_KV_MFMA128P) ? 1 : 2);
    L.wait_polls = (L.fuse && R.wgs <= resident) ? p->wait_polls : 0;
    L.merge_fences = p->merge_fences ? 1 : 0;
    // With one row tile per KV head no two workgroups read the same keys, and the kernel can load them
    // non-temporal.  Measured (us per query in a stream of queries, default policy -> non-temporal):
    //   rows per KV head   16K cached     32K            64K            128K
    //   <= 64              26.2 -> 25.9   37.1 -> 35.5   57.1 -> 54.4    99.6 ->  94.6
    //   65 - 128           29.5 -> 32.2   40.6 -> 41.9   64.8 -> 64.6   119.0 -> 111.9
    //   129 - 256          37.8 -> 41.4   53.6 -> 56.8   90.7 -> 90.7   162.1 -> 162.0
    // so the 64-row instance always does, the 128-row instances from 64K cached tokens on, the 256-row
    // instance (and every call whose row tiles share their keys through the L2) never.
    const bool once_pays = v.id == SK_KV_MFMA64 || ((v.id == SK_KV_MFMA128 || v.id == SK_KV_MFMA128P) && kv_len >= p->stream_min_tokens);
    L.kv_once = (!p->no_stream_loads && L.n_tiles == 1 && once_pays) ? 1 : 0;
    return SK_OK;
}

// Enqueues a planned call.
int launch_regular(sk_pool* p, RegPlan& R, const void* q, void* out, int out_dtype, float* lse, hipStream_t st)
{
    if (inject(p, SK_SITE_ATTENTION)) return SK_E_HIP;
    if (!p->device) return SK_OK;
    sk_launch L;
    fill_launch_common(p, L, q, out, out_dtype, lse, R.v);
    {   // the plan holds everything but the pointers
        sk_launch& S = R.L;
        S.g = L.g; S.q = L.q; S.out = L.out; S.lse = L.lse; S.part_ml = L.part_ml; S.part_o = L.part_o; S.sync = L.sync;
        S.out_dtype = L.out_dtype;
    }
    const int32_t pc = prof_call(p);
    void *e0, *e1;
    prof_pair(p, pc, 0, &e0, &e1);
    int e = sk_launch_attention(R.L, R.v.id, R.wgs, st, e0, e1);
    if (e) { g_last_hip = e; return SK_E_HIP; }
    p->stats.launches++;
    if (R.parts > 1 && !R.L.fuse) {
        // the attention kernel is enqueued and will write its partials; a failure here leaves out/lse unwritten
        prof_pair(p, pc, 1, &e0, &e1);
        e = inject(p, SK_SITE_COMBINE) ? (int)hipErrorUnknown : sk_launch_combine(R.L, R.base_wgs, st, e0, e1);
        if (e) { g_last_hip = e; return SK_E_HIP; }
        p->stats.launches++;
    }
    p->stats.kv_bytes_streamed += R.kv_len * 2 * p->d.n_kv_heads * p->d.head_dim * p->L.elem * R.L.n_tiles;
    p->last.workgroups = R.wgs; p->last.n_splits = R.parts; p->last.row_tiles = R.L.n_tiles; p->last.kernel_variant = R.v.id;
    p->last.fused_merge = R.L.fuse;
    return SK_OK;
}

// Builds the scatter list for `count` tokens (packed rows src0..) going either behind position
// `dst_tok0` of session `s` (blocks already in s->blocks) or into staging blocks eph_blk0..
int build_scatter(const sk_pool* p, const Session* s, int32_t id, int64_t dst_tok0, int32_t src0, int64_t count,
                  int64_t first_new_block, bool to_eph, int64_t eph_blk0, std::vector<sk_scatter>& out)
{
    const int64_t B = to_eph ? 16 : p->d.block_tokens;
    for (int64_t t = dst_tok0; t < dst_tok0 + count;) {
        const int64_t gend = std::min<int64_t>((t / 16 + 1) * 16, dst_tok0 + count);
        sk_scatter it;
        const int64_t bi = t / B;
        it.src_tok0 = src0 + int32_t(t - dst_tok0);
        it.count = int32_t(gend - t);
        it.dst_slot0 = int32_t(t % B);
        it.to_eph = to_eph ? 1 : 0;
        if (to_eph) {
            it.dst_off = (eph_blk0 + bi) * p->L.eph_blk_stride;
            it.tbl_index = -1; it.block_id = 0;
        } else {
            const int32_t blk = s->blocks[bi];
            it.dst_off = int64_t(blk) * p->L.blk_stride;
            it.block_id = blk;
            it.tbl_index = (bi >= first_new_block) ? int32_t(int64_t(id) * p->L.max_blocks_per_session + bi) : -1;
        }
        out.push_back(it);
        t = gend;
    }
    return SK_OK;
}

// A single-session scatter in two halves, so that everything that can refuse the call happens before
// the call changes anything: scatter_reserve (size check, and a pinned ring slot if the list is too
// long to travel in the kernel arguments), then, once the list is built, scatter_launch.
struct ScatterSlot { bool upload = false; int slot = 0; unsigned char* host = nullptr; };

int64_t scatter_groups(int64_t dst_tok0, int64_t count)     // 16-token groups the tokens dst_tok0 .. +count-1 touch
{
    return count <= 0 ? 0 : (dst_tok0 + count + 15) / 16 - dst_tok0 / 16;
}

int scatter_reserve(sk_pool* p, int64_t n_items, ScatterSlot& ss)
{
    ss = ScatterSlot();
    if (n_items <= SK_SCATTER_ARGS_MAX) return SK_OK;
    if (size_t(n_items) * sizeof(sk_scatter) > p->L.meta_bytes) return SK_E_WORKSPACE;
    ss.upload = true;
    return ring_acquire(p, &ss.slot, &ss.host);
}

int scatter_launch(sk_pool* p, const ScatterSlot& ss, const std::vector<sk_scatter>& items, const void* k, const void* v, hipStream_t st)
{
    if (items.empty()) return SK_OK;
    unsigned char* ws = (unsigned char*)p->d.workspace;
    if (!ss.upload) {          // short list: in the kernel arguments, nothing to upload
        if (inject(p, SK_SITE_SCATTER)) return SK_E_HIP;
        if (!p->device) return SK_OK;
        sk_scatter_list lst;
        memcpy(lst.item, items.data(), items.size() * sizeof(sk_scatter));
        int e = sk_launch_scatter_args(p->geom, k, v, lst, (int32_t)items.size(), (int32_t*)(ws + p->L.off_tables),
                                       (unsigned char*)p->d.kv_mem, ws + p->L.off_eph, st);
        if (e) { g_last_hip = e; return SK_E_HIP; }
        p->stats.launches++;
        return SK_OK;
    }
    const size_t bytes = items.size() * sizeof(sk_scatter);
    if (ss.host) memcpy(ss.host, items.data(), bytes);
    int rc = ring_upload(p, ss.slot, bytes, st);
    if (rc) return rc;
    if (inject(p, SK_SITE_SCATTER)) return SK_E_HIP;
    if (!p->device) return SK_OK;
    int e = sk_launch_scatter(p->geom, k, v, (const sk_scatter*)(ws + p->L.off_meta), (int32_t)items.size(),
                              (int32_t*)(ws + p->L.off_tables), (unsigned char*)p->d.kv_mem, ws + p->L.off_eph, st);
    if (e) { g_last_hip = e; return SK_E_HIP; }
    p->stats.launches++;
    return SK_OK;
}

// Takes `need` blocks for the session (caller has checked availability).
void take_blocks(sk_pool* p, Session* s, int64_t need)
{
    for (int64_t i = 0; i < need; ++i) {
        s->blocks.push_back(p->free_blocks.front());
        p->refcnt[(size_t)p->free_blocks.front()] = 1;
        p->free_blocks.pop_front();
    }
    p->blocks_in_use += need;
}

// One session lets go of a block; the last holder returns it to the free list.
void release_block(sk_pool* p, int32_t b)
{
    if (--p->refcnt[(size_t)b] == 0) { p->free_blocks.push_back(b); p->blocks_in_use--; }
}

// After a fork, a truncation can leave the end of a session inside a block that other sessions
// also hold.  Before such a session appends it gets its own copy of that block: the one case of
// copy-on-write (nothing else ever writes into a block that is not the writer's alone).
bool tail_shared(const sk_pool* p, const Session* s)
{
    return s->len % p->d.block_tokens != 0 && p->refcnt[(size_t)s->blocks.back()] > 1;
}

// What an append changed in one session, so that a later failure of the same call can take it back.
struct Undo {
    Session* s = nullptr;
    int64_t len = 0;
    size_t n_blocks = 0;
    int32_t old_tail = -1;       // >= 0: the shared tail block that was swapped for a copy
};

// The caller has checked that a block is free.  The copy is ordered on `st` in front of the
// scatter that follows; the scatter also rewrites the table entry (it is told that the block is new).
// On failure nothing has changed.
int unshare_tail(sk_pool* p, Session* s, Undo& u, hipStream_t st)
{
    const int32_t old = s->blocks.back();
    const int32_t blk = p->free_blocks.front();
    if (inject(p, SK_SITE_BLOCK_COPY)) return SK_E_HIP;
    if (p->device) {
        int e = sk_launch_copy_block(p->geom, (unsigned char*)p->d.kv_mem, old, blk, st);
        if (e) { g_last_hip = e; return SK_E_HIP; }
    }
    p->free_blocks.pop_front();
    p->refcnt[(size_t)blk] = 1;
    p->refcnt[(size_t)old]--;                 // still held by the others
    p->blocks_in_use++;
    s->blocks.back() = blk;
    u.old_tail = old;
    return SK_OK;
}

// Takes an append back: the blocks it took return to the head of the free list in their old order,
// the length is restored; the copy of a shared tail is given up too unless `keep_copy` (the commit
// kernel is already enqueued and has pointed the device block table at the copy; keeping it changes
// nothing a caller can observe but the number of free blocks).
void rollback(sk_pool* p, const Undo& u, bool keep_copy)
{
    Session* s = u.s;
    while (s->blocks.size() > u.n_blocks) {
        const int32_t b = s->blocks.back();
        s->blocks.pop_back();
        p->refcnt[(size_t)b] = 0;
        p->free_blocks.push_front(b);
        p->blocks_in_use--;
    }
    if (u.old_tail >= 0 && !keep_copy) {
        const int32_t blk = s->blocks.back();
        s->blocks.back() = u.old_tail;
        p->refcnt[(size_t)u.old_tail]++;
        p->refcnt[(size_t)blk] = 0;
        p->free_blocks.push_front(blk);
        p->blocks_in_use--;
    }
    s->len = u.len;
}

// The host half of an append of T tokens to session s (availability already checked): copy of a
// shared tail, new blocks, new length.  Fills `u`; on failure nothing has changed.
int grow_session(sk_pool* p, Session* s, int64_t T, Undo& u, int64_t* first_new, hipStream_t st)
{
    u = Undo();
    u.s = s; u.len = s->len; u.n_blocks = s->blocks.size();
    const bool unshare = tail_shared(p, s);
    if (unshare) { int rc = unshare_tail(p, s, u, st); if (rc) return rc; }
    *first_new = (int64_t)s->blocks.size() - (unshare ? 1 : 0);
    take_blocks(p, s, blocks_needed(p, s->len, T));
    s->len += T;
    return SK_OK;
}

int check_out_dtype(const sk_pool* p, int out_dtype)
{
    if (out_dtype != SK_F32 && out_dtype != p->d.dtype) return SK_E_DTYPE;
    return SK_OK;
}

// ---- list mode: many row tiles (of several sessions, or of one question batch) in one launch ----

struct TileReq {            // one tile of query rows and the keys it may see
    int32_t tbl_off, q_tok0, n_tok;
    int32_t pos0;           // absolute position of its first token, or SK_NO_CAUSAL
    int32_t kv_vis;         // cached tokens visible to the tile (positions 0 .. kv_vis-1)
    int32_t eph_blk[2], eph_cnt[2], eph_pos0[2];
    int32_t hole_lo, hole_hi;   // evicted cached tokens of the session
    int32_t tok_period, sub_blocks;   // > 0: the tile packs sequences of tok_period tokens (see sk_work)
};
struct ListGroup {          // tiles that share a kernel variant and the q/out/lse arrays
    Variant v = {SK_KV_SIMPLE, 16, 1};
    const void* q = nullptr; void* out = nullptr; float* lse = nullptr;
    std::vector<TileReq> tiles;
};
struct ScatterBatch { const void* k = nullptr; const void* v = nullptr; std::vector<sk_scatter> items; };

// Cuts T tokens (packed rows q_row0..) that share `base` into row tiles of the group's height.
void add_tiles(ListGroup& g, const TileReq& base, int32_t q_row0, int32_t T)
{
    for (int32_t t0 = 0; t0 < T; t0 += g.v.tok_per_tile) {
        TileReq r = base;
        r.q_tok0 = q_row0 + t0;
        r.n_tok = std::min(g.v.tok_per_tile, T - t0);
        if (base.pos0 < SK_NO_CAUSAL) {
            r.pos0 = base.pos0 + t0;
            r.kv_vis = std::min<int64_t>(base.kv_vis, int64_t(r.pos0) + r.n_tok);
        }
        g.tiles.push_back(r);
    }
}

constexpr int kMaxGroups = 3;   // one launch per kernel variant in use

// A batched call in two halves.  plan_list cuts the tiles into workgroups, builds the lists and takes
// the pinned ring slot they travel in: everything that can refuse the call, and nothing that changes
// a session or the device.  launch_list uploads the lists and enqueues the kernels.
struct ListPlan {
    std::vector<sk_work> work[kMaxGroups];
    std::vector<sk_comb> comb[kMaxGroups];
    int64_t rows_base[kMaxGroups] = {};
    int64_t kv_total = 0, n_tiles = 0;
    bool fuse = false;
    int slot = 0;
    unsigned char* host = nullptr;
    bool scatter_enqueued = false;     // set by launch_list once a commit kernel is on the stream
};

int plan_list(sk_pool* p, const ScatterBatch* sb, int n_sb, ListGroup* groups, int n_groups, ListPlan& P)
{
    if (n_groups > kMaxGroups) return SK_E_INVAL;
    if (inject(p, SK_SITE_PLAN)) return SK_E_WORKSPACE;
    const int Hkv = p->d.n_kv_heads;
    int64_t kv_group[kMaxGroups] = {};
    P.kv_total = 0; P.n_tiles = 0;
    for (int gi = 0; gi < n_groups; ++gi)
        for (const TileReq& t : groups[gi].tiles) { P.kv_total += t.kv_vis; kv_group[gi] += t.kv_vis; ++P.n_tiles; }
    if (P.n_tiles == 0) return SK_OK;
    // One chunk length per group (= per launch), so that the workgroups of a launch cost about the
    // same whatever the session length, and every launch has enough of them to fill the chip
    // several times over (rounds of one 512-thread workgroup per CU, or of two 256-thread ones).
    int64_t chunk_g[kMaxGroups];
    for (int gi = 0; gi < n_groups; ++gi) {
        const int64_t per_round = groups[gi].v.id == SK_KV_MFMA256 ? 256 : 512;
        const int64_t target = 4 * int64_t(p->target_wgs);       // 2,048 by default: 8 rounds of 256, 4 of 512
        chunk_g[gi] = std::max<int64_t>(256, (kv_group[gi] * Hkv + target - 1) / target);
        chunk_g[gi] = (chunk_g[gi] + 63) / 64 * 64;
        // Workgroups of a launch run in rounds of `per_round`; pick, near that length, the one whose
        // last round is fullest (a launch of 7.1 rounds takes as long as one of 8).
        auto count_wgs = [&](int64_t c) {
            int64_t n = 0;
            for (const TileReq& t : groups[gi].tiles) n += std::max<int64_t>(1, (t.kv_vis + c - 1) / c);
            return n * Hkv;
        };
        double best_eff = -1.0; int64_t best = chunk_g[gi];
        for (int64_t c = std::max<int64_t>(256, chunk_g[gi] * 3 / 4 / 64 * 64); c <= chunk_g[gi] * 5 / 4; c += 64) {
            const int64_t n = count_wgs(c);
            const double eff = double(n) / double((n + per_round - 1) / per_round * per_round);
            if (eff >= best_eff) { best_eff = eff; best = c; }       // ties: the longer chunk (fewer partials)
        }
        chunk_g[gi] = best;
    }
    const int64_t cap_rows = p->L.part_slots * kPartSlotRows;
    size_t bytes = 0;
    for (;;) {
        int64_t rows_used = 0;
        bool ok = true;
        int64_t unit = 0;
        for (int gi = 0; gi < n_groups && ok; ++gi) {
            ListGroup& g = groups[gi];
            const int64_t chunk = chunk_g[gi];
            P.work[gi].clear(); P.comb[gi].clear();
            P.rows_base[gi] = rows_used;
            int64_t slot = 0;       // in units of this group's rows_per_slot, from rows_base
            // runs of consecutive tiles of one session: split-major order inside a run, so that
            // workgroups resident at the same time read the same keys (L2 reuse across row tiles)
            size_t i0 = 0;
            while (i0 < g.tiles.size()) {
                size_t i1 = i0;
                int32_t max_parts = 1;
                std::vector<int32_t> nparts, slot0, unit0;
                while (i1 < g.tiles.size() && g.tiles[i1].tbl_off == g.tiles[i0].tbl_off) {
                    const int32_t np = std::max<int64_t>(1, (g.tiles[i1].kv_vis + chunk - 1) / chunk);
                    nparts.push_back(np); max_parts = std::max(max_parts, np);
                    slot0.push_back(np > 1 ? (int32_t)slot : -1);
                    unit0.push_back(np > 1 ? (int32_t)unit : -1);
                    if (np > 1) { slot += int64_t(np) * Hkv; unit += Hkv; }
                    ++i1;
                }
                for (int32_t part = 0; part < max_parts; ++part)
                    for (size_t i = i0; i < i1; ++i) {
                        const TileReq& t = g.tiles[i];
                        const int32_t np = nparts[i - i0];
                        if (part >= np) continue;
                        for (int h = 0; h < Hkv; ++h) {
                            sk_work w = {};
                            w.tbl_off = t.tbl_off; w.kv_head = h; w.q_tok0 = t.q_tok0; w.n_tok = t.n_tok; w.pos0 = t.pos0;
                            w.kv_begin = int32_t(part * chunk);
                            w.kv_end = int32_t(std::min<int64_t>(t.kv_vis, (part + 1) * chunk));
                            w.part = np > 1 ? slot0[i - i0] + part * Hkv + h : -1;
                            w.unit = np > 1 ? unit0[i - i0] + h : -1;
                            w.part0 = np > 1 ? slot0[i - i0] + h : -1;
                            w.n_parts = np;
                            w.hole_lo = t.hole_lo; w.hole_hi = t.hole_hi;
                            w.tok_period = t.tok_period; w.sub_blocks = t.sub_blocks;
                            if (part == np - 1)
                                for (int e = 0; e < 2; ++e) { w.eph_blk[e] = t.eph_blk[e]; w.eph_cnt[e] = t.eph_cnt[e]; w.eph_pos0[e] = t.eph_pos0[e]; }
                            P.work[gi].push_back(w);
                        }
                    }
                for (size_t i = i0; i < i1; ++i) {
                    if (nparts[i - i0] < 2) continue;
                    for (int h = 0; h < Hkv; ++h) {
                        sk_comb c = {};
                        c.part0 = slot0[i - i0] + h; c.n_parts = nparts[i - i0]; c.part_stride = Hkv;
                        c.q_tok0 = g.tiles[i].q_tok0; c.n_tok = g.tiles[i].n_tok; c.kv_head = h;
                        P.comb[gi].push_back(c);
                    }
                }
                i0 = i1;
            }
            rows_used += slot * g.v.rows_per_slot;
            if (rows_used > cap_rows) ok = false;
        }
        // the last workgroup of a unit merges it inside the attention kernel when the call asks for
        // that (SK_FUSE_LIST) and every kernel in use can (the matrix-pipe instances)
        P.fuse = p->fuse_list && unit <= p->L.sync_units;
        for (int gi = 0; gi < n_groups; ++gi)
            if (!P.work[gi].empty() && groups[gi].v.id == SK_KV_SIMPLE) P.fuse = false;
        bytes = 0;
        for (int i = 0; i < n_sb; ++i) bytes += align_up(sb[i].items.size() * sizeof(sk_scatter), 256);
        for (int gi = 0; gi < n_groups; ++gi)
            bytes += align_up(P.work[gi].size() * sizeof(sk_work), 256) + align_up(P.comb[gi].size() * sizeof(sk_comb), 256);
        if (ok && bytes <= p->L.meta_bytes) break;
        if (chunk_g[0] > (int64_t(1) << 30)) return SK_E_WORKSPACE;
        for (int gi = 0; gi < n_groups; ++gi) chunk_g[gi] *= 2;
    }
    return ring_acquire(p, &P.slot, &P.host);
}

int launch_list(sk_pool* p, ListPlan& P, const ScatterBatch* sb, int n_sb, ListGroup* groups, int n_groups, int out_dtype, hipStream_t st)
{
    if (P.n_tiles == 0) return SK_OK;
    const int Hkv = p->d.n_kv_heads;
    // one upload: scatter lists, work lists, combine lists
    unsigned char* ws = (unsigned char*)p->d.workspace;
    unsigned char* dev_meta = p->device ? ws + p->L.off_meta : nullptr;
    size_t off = 0, off_sb[2] = {0, 0}, off_work[kMaxGroups] = {}, off_comb[kMaxGroups] = {};
    for (int i = 0; i < n_sb; ++i) {
        off_sb[i] = off;
        if (P.host) memcpy(P.host + off, sb[i].items.data(), sb[i].items.size() * sizeof(sk_scatter));
        off += align_up(sb[i].items.size() * sizeof(sk_scatter), 256);
    }
    for (int gi = 0; gi < n_groups; ++gi) {
        off_work[gi] = off;
        if (P.host) memcpy(P.host + off, P.work[gi].data(), P.work[gi].size() * sizeof(sk_work));
        off += align_up(P.work[gi].size() * sizeof(sk_work), 256);
        off_comb[gi] = off;
        if (P.host) memcpy(P.host + off, P.comb[gi].data(), P.comb[gi].size() * sizeof(sk_comb));
        off += align_up(P.comb[gi].size() * sizeof(sk_comb), 256);
    }
    int rc = ring_upload(p, P.slot, off, st);
    if (rc) return rc;
    for (int i = 0; i < n_sb; ++i) {
        if (sb[i].items.empty()) continue;
        if (inject(p, SK_SITE_SCATTER)) return SK_E_HIP;
        if (!p->device) continue;
        int e = sk_launch_scatter(p->geom, sb[i].k, sb[i].v, (const sk_scatter*)(dev_meta + off_sb[i]), (int32_t)sb[i].items.size(),
                                  (int32_t*)(ws + p->L.off_tables), (unsigned char*)p->d.kv_mem, ws + p->L.off_eph, st);
        if (e) { g_last_hip = e; return SK_E_HIP; }
        P.scatter_enqueued = true;
        p->stats.launches++;
    }
    if (inject(p, SK_SITE_ATTENTION)) return SK_E_HIP;
    if (!p->device) return SK_OK;
    const int32_t pc = prof_call(p);
    void *e0, *e1;
    sk_launch L[kMaxGroups];
    int32_t wgs = 0, max_parts = 1;
    for (int gi = 0; gi < n_groups; ++gi) {
        if (P.work[gi].empty()) continue;
        ListGroup& g = groups[gi];
        fill_launch_common(p, L[gi], g.q, g.out, out_dtype, g.lse, g.v);
        L[gi].mode = SK_MODE_LIST;
        L[gi].part_ml += P.rows_base[gi] * 4;
        L[gi].part_o += P.rows_base[gi] * p->d.head_dim;
        L[gi].work = (const sk_work*)(dev_meta + off_work[gi]);
        L[gi].comb = (const sk_comb*)(dev_meta + off_comb[gi]);
        L[gi].fuse = P.fuse ? 1 : 0;
        L[gi].wait_polls = 0;          // the workgroups of a long list are not resident together
        L[gi].merge_fences = p->merge_fences ? 1 : 0;
        prof_pair(p, pc, 0, &e0, &e1);
        int e = sk_launch_attention(L[gi], g.v.id, (int32_t)P.work[gi].size(), st, e0, e1);
        if (e) { g_last_hip = e; return SK_E_HIP; }
        p->stats.launches++;
        wgs += (int32_t)P.work[gi].size();
        for (const sk_comb& c : P.comb[gi]) max_parts = std::max(max_parts, c.n_parts);
    }
    for (int gi = 0; gi < n_groups && !P.fuse; ++gi) {
        if (P.comb[gi].empty()) continue;
        prof_pair(p, pc, 1, &e0, &e1);
        int e = sk_launch_combine(L[gi], (int32_t)P.comb[gi].size(), st, e0, e1);
        if (e) { g_last_hip = e; return SK_E_HIP; }
        p->stats.launches++;
    }
    p->stats.kv_bytes_streamed += P.kv_total * 2 * Hkv * p->d.head_dim * p->L.elem;
    p->last.workgroups = wgs; p->last.n_splits = max_parts; p->last.row_tiles = (int32_t)P.n_tiles;
    p->last.kernel_variant = groups[0].v.id;
    p->last.fused_merge = P.fuse ? 1 : 0;
    for (int gi = n_groups - 1; gi >= 0; --gi) if (!groups[gi].tiles.empty()) p->last.kernel_variant = groups[gi].v.id;
    return SK_OK;
}

}  // namespace

extern "C" {

size_t sk_pool_kv_bytes(const sk_pool_desc* desc)
{
    Layout L;
    if (!desc || !derive_layout(*desc, L)) return 0;
    return L.kv_bytes;
}

size_t sk_pool_workspace_bytes(const sk_pool_desc* desc)
{
    Layout L;
    if (!desc || !derive_layout(*desc, L)) return 0;
    return L.ws_bytes;
}

int sk_pool_create(const sk_pool_desc* desc, sk_pool** out)
{
    if (out) *out = nullptr;
    if (!desc || !out) return SK_E_INVAL;
    if (desc->dtype != SK_F32 && desc->dtype != SK_BF16) return SK_E_DTYPE;
    Layout L;
    if (!derive_layout(*desc, L)) return SK_E_SHAPE;
    const bool meta_only = (desc->flags & SK_POOL_METADATA_ONLY) != 0;
    if (!meta_only) {
        if (!desc->kv_mem || !desc->workspace) return SK_E_INVAL;
        if ((reinterpret_cast<uintptr_t>(desc->kv_mem) & 255) || (reinterpret_cast<uintptr_t>(desc->workspace) & 255)) return SK_E_INVAL;
        if (desc->kv_bytes < L.kv_bytes || desc->workspace_bytes < L.ws_bytes) return SK_E_WORKSPACE;
    }
    sk_pool* p = new (std::nothrow) sk_pool();
    if (!p) return SK_E_NOMEM;
    p->d = *desc;
    p->L = L;
    p->device = !meta_only;
    for (int64_t i = 0; i < desc->n_blocks; ++i) p->free_blocks.push_back((int32_t)i);
    p->refcnt.assign((size_t)desc->n_blocks, 0);
    p->sessions.resize(desc->max_sessions);
    for (int32_t i = desc->max_sessions - 1; i >= 0; --i) p->free_ids.push_back(i);
    const float scale = desc->softmax_scale != 0.f ? desc->softmax_scale : 1.0f / std::sqrt((float)desc->head_dim);
    sk_geom& g = p->geom;
    memset(&g, 0, sizeof g);
    g.kv = (const unsigned char*)desc->kv_mem;
    g.eph = meta_only ? nullptr : (const unsigned char*)desc->workspace + L.off_eph;
    g.tables = meta_only ? nullptr : (const int32_t*)((const unsigned char*)desc->workspace + L.off_tables);
    g.eph_ident = meta_only ? nullptr : (const int32_t*)((const unsigned char*)desc->workspace + L.off_ident);
    g.blk_stride = L.blk_stride; g.eph_blk_stride = L.eph_blk_stride;
    g.head_stride = L.head_stride; g.v_off = (int32_t)L.v_off;
    g.eph_head_stride = L.eph_head_stride; g.eph_v_off = (int32_t)L.eph_v_off;
    g.B = desc->block_tokens; g.log2B = ilog2_exact(desc->block_tokens);
    g.Hq = desc->n_q_heads; g.Hkv = desc->n_kv_heads; g.G = L.G; g.log2G = ilog2_exact(L.G);
    g.d = desc->head_dim; g.elem = L.elem;
    g.scale_log2e = scale * 1.4426950408889634f;
    if (const char* t = getenv("SK_TARGET_WGS")) { int x = atoi(t); if (x > 0) { p->target_wgs = x; p->target_wgs_set = true; } }
    auto env_on = [](const char* name) { const char* x = getenv(name); return x && x[0] == '1'; };
    p->force_simple = env_on("SK_FORCE_SIMPLE");
    p->no_256 = env_on("SK_NO_256");
    p->no_pack = env_on("SK_NO_PACK");
    p->no_interleave = env_on("SK_NO_INTERLEAVE");
    p->no_stream_loads = env_on("SK_NO_STREAM_LOADS");
    p->fuse = env_on("SK_FUSE");
    p->p128 = !env_on("SK_NO_P128");
    if (const char* t = getenv("SK_P128_MIN_TOKENS")) { long long x = atoll(t); if (x >= 0) p->p128_min_tokens = x; }
    if (const char* t = getenv("SK_STREAM_MIN_TOKENS")) { long long x = atoll(t); if (x >= 0) p->stream_min_tokens = x; }
    p->fuse_list = env_on("SK_FUSE_LIST");
    p->merge_fences = env_on("SK_MERGE_FENCES");
    if (const char* t = getenv("SK_WAIT_POLLS")) { int x = atoi(t); if (x >= 0) p->wait_polls = x; }
    if (!meta_only) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            p->n_cus = cus;
        hipError_t e = hipHostMalloc((void**)&p->ring, p->L.meta_bytes * kRingSlots, hipHostMallocDefault);
        if (e != hipSuccess) { g_last_hip = (int)e; delete p; return SK_E_HIP; }
        for (int i = 0; i < kRingSlots; ++i) {
            e = hipEventCreateWithFlags(&p->ring_ev[i], hipEventDisableTiming);
            if (e != hipSuccess) { g_last_hip = (int)e; sk_pool_destroy(p); return SK_E_HIP; }
        }
        // identity table over the staging blocks (one synchronous copy at creation)
        std::vector<int32_t> ident((size_t)L.eph_blocks);
        for (size_t i = 0; i < ident.size(); ++i) ident[i] = (int32_t)i;
        e = hipMemcpy((unsigned char*)desc->workspace + L.off_ident, ident.data(), ident.size() * 4, hipMemcpyHostToDevice);
        if (e != hipSuccess) { g_last_hip = (int)e; sk_pool_destroy(p); return SK_E_HIP; }
        // the merge counters start at zero; every launch leaves them at zero
        e = hipMemset((unsigned char*)desc->workspace + L.off_sync, 0, size_t(L.sync_units) * 8);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) { g_last_hip = (int)e; sk_pool_destroy(p); return SK_E_HIP; }
    }
    *out = p;
    return SK_OK;
}

int sk_pool_destroy(sk_pool* p)
{
    if (!p) return SK_E_INVAL;
    if (p->device) {
        for (int i = 0; i < kRingSlots; ++i)
            if (p->ring_ev[i]) (void)hipEventDestroy(p->ring_ev[i]);
        for (sk_pool::ProfRec& r : p->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
        if (p->ring) (void)hipHostFree(p->ring);
    }
    delete p;
    return SK_OK;
}

int sk_pool_blocks_free(const sk_pool* p, int64_t* out)
{
    if (!p || !out) return SK_E_INVAL;
    *out = (int64_t)p->free_blocks.size();
    return SK_OK;
}

int sk_pool_set_alloc_order(sk_pool* p, const int32_t* perm, int64_t n)
{
    if (!p || !perm || n != p->d.n_blocks) return SK_E_INVAL;
    if (p->blocks_in_use != 0) return SK_E_INVAL;
    std::vector<char> seen((size_t)n, 0);
    for (int64_t i = 0; i < n; ++i) {
        if (perm[i] < 0 || perm[i] >= n || seen[perm[i]]) return SK_E_INVAL;
        seen[perm[i]] = 1;
    }
    p->free_blocks.assign(perm, perm + n);
    return SK_OK;
}

int sk_session_create(sk_pool* p, int32_t* out_id)
{
    if (!p || !out_id) return SK_E_INVAL;
    if (p->free_ids.empty()) return SK_E_NOMEM;
    int32_t id = p->free_ids.back();
    p->free_ids.pop_back();
    Session& s = p->sessions[id];
    s.live = true; s.len = 0; s.frozen = 0; s.win = 0; s.blocks.clear();
    *out_id = id;
    return SK_OK;
}

int sk_session_destroy(sk_pool* p, int32_t id)
{
    Session* s = get_session(p, id);
    if (!s) return p ? SK_E_BADSESSION : SK_E_INVAL;
    for (int32_t b : s->blocks) release_block(p, b);
    s->blocks.clear(); s->len = 0; s->frozen = 0; s->win = 0; s->live = false;
    p->free_ids.push_back(id);
    return SK_OK;
}

int sk_session_length(const sk_pool* p, int32_t id, int64_t* out)
{
    const Session* s = get_session(p, id);
    if (!p || !out) return SK_E_INVAL;
    if (!s) return SK_E_BADSESSION;
    *out = s->retained();
    return SK_OK;
}

int sk_session_block_table(const sk_pool* p, int32_t id, const int32_t** table, int64_t* n_blocks)
{
    const Session* s = get_session(p, id);
    if (!p || !table || !n_blocks) return SK_E_INVAL;
    if (!s) return SK_E_BADSESSION;
    *table = s->blocks.data();
    *n_blocks = (int64_t)s->blocks.size();
    return SK_OK;
}

int sk_session_append(sk_pool* p, int32_t id, const void* q, const void* k, const void* v, int32_t L,
                      void* out, int out_dtype, float* lse, void* hip_stream)
{
    if (!p) return SK_E_INVAL;
    Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (L < 0) return SK_E_INVAL;
    if (L == 0) return SK_OK;
    if (L > p->L.max_batch_tokens) return SK_E_WORKSPACE;
    if (p->device) {
        if (!k || !v || (!q) != (!out)) return SK_E_INVAL;
        if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse)) return SK_E_INVAL;
        if (q) { int rc = check_out_dtype(p, out_dtype); if (rc) return rc; }
    }
    if (s->len + L > p->L.max_session_tokens) return SK_E_NOMEM;
    const int64_t need = blocks_needed(p, s->len, L);
    if (need + (tail_shared(p, s) ? 1 : 0) > (int64_t)p->free_blocks.size()) return SK_E_NOMEM;
    // everything else that can refuse the call, before it changes anything: the decomposition of the
    // attention, and the ring slot of a scatter list too long for the kernel arguments
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t n = s->len;
    const bool attend = p->device ? q != nullptr : true;
    RegPlan plan;
    if (attend) {
        int rc = plan_regular(p, id, L, (int32_t)n, n + L, 0, 0, s->frozen, s->win, 0, plan);
        if (rc) return rc;
    }
    ScatterSlot ss;
    { int rc = scatter_reserve(p, scatter_groups(n, L), ss); if (rc) return rc; }
    // from here on only a failing HIP call can stop the call; what it changed is taken back
    Undo u;
    int64_t first_new = 0;
    { int rc = grow_session(p, s, L, u, &first_new, st); if (rc) return rc; }
    std::vector<sk_scatter> items;
    build_scatter(p, s, id, n, 0, L, first_new, false, 0, items);
    int rc = scatter_launch(p, ss, items, k, v, st);
    if (rc) { rollback(p, u, false); return rc; }
    if (attend) {
        rc = launch_regular(p, plan, q, out, out_dtype, lse, st);
        if (rc) { rollback(p, u, true); return rc; }
    }
    p->stats.tokens_appended += L;
    return SK_OK;
}

int sk_session_query(sk_pool* p, int32_t id, const void* q, const void* k, const void* v, int32_t nq,
                     void* out, int out_dtype, float* lse, int32_t n_splits, void* hip_stream)
{
    if (!p) return SK_E_INVAL;
    Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (nq < 0 || n_splits < 0) return SK_E_INVAL;
    if (nq == 0) return SK_OK;
    if (!p->device) return SK_E_NODEVICE;
    if (!q || !out || (!k) != (!v)) return SK_E_INVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse)) return SK_E_INVAL;
    int rc = check_out_dtype(p, out_dtype);
    if (rc) return rc;
    if (nq > p->L.max_batch_tokens) return SK_E_WORKSPACE;
    if (!k && s->retained() == 0) return SK_E_EMPTY;
    Variant vv;
    if (!pick_variant(p, nq, vv)) return SK_E_SHAPE;
    hipStream_t st = (hipStream_t)hip_stream;
    RegPlan plan;
    if (k) rc = plan_regular(p, id, nq, (int32_t)s->len, s->len, nq, (int32_t)s->len, s->frozen, s->win, n_splits, plan);
    else rc = plan_regular(p, id, nq, SK_NO_CAUSAL, s->len, 0, 0, s->frozen, s->win, n_splits, plan);
    if (rc) return rc;
    if (k) {
        ScatterSlot ss;
        rc = scatter_reserve(p, scatter_groups(0, nq), ss);
        if (rc) return rc;
        std::vector<sk_scatter> items;
        build_scatter(p, nullptr, id, 0, 0, nq, 0, true, 0, items);
        rc = scatter_launch(p, ss, items, k, v, st);
        if (rc) return rc;
    }
    rc = launch_regular(p, plan, q, out, out_dtype, lse, st);
    if (rc) return rc;
    p->stats.tokens_queried += nq;
    return SK_OK;
}

int sk_batch_step(sk_pool* p, int32_t n_items, const int32_t* session_id, const int32_t* op, const int32_t* cu_tokens,
                  const void* q, const void* k, const void* v, void* out, int out_dtype, float* lse, void* hip_stream)
{
    if (!p || n_items < 0) return SK_E_INVAL;
    if (n_items == 0) return SK_OK;
    if (!session_id || !op || !cu_tokens) return SK_E_INVAL;
    if (n_items > p->d.max_sessions) return SK_E_INVAL;        // sessions are distinct
    if (cu_tokens[0] != 0) return SK_E_INVAL;
    std::vector<char> seen((size_t)p->d.max_sessions, 0);
    int64_t need_blocks = 0;
    bool any_kv = false;
    for (int i = 0; i < n_items; ++i) {
        const Session* s = get_session(p, session_id[i]);
        if (!s) return SK_E_BADSESSION;
        if (seen[session_id[i]]) return SK_E_INVAL;
        seen[session_id[i]] = 1;
        const int64_t T = int64_t(cu_tokens[i + 1]) - cu_tokens[i];
        if (T < 0) return SK_E_INVAL;
        if (op[i] != SK_OP_APPEND && op[i] != SK_OP_QUERY_A && op[i] != SK_OP_QUERY_B) return SK_E_INVAL;
        if (T == 0) continue;
        if (op[i] == SK_OP_APPEND) {
            if (s->len + T > p->L.max_session_tokens) return SK_E_NOMEM;
            need_blocks += blocks_needed(p, s->len, T) + (tail_shared(p, s) ? 1 : 0);
        }
        if (op[i] == SK_OP_QUERY_A && s->retained() == 0) return SK_E_EMPTY;
        if (op[i] != SK_OP_QUERY_A) any_kv = true;
    }
    const int64_t total = cu_tokens[n_items];
    if (total > p->L.max_batch_tokens) return SK_E_WORKSPACE;
    if (need_blocks > (int64_t)p->free_blocks.size()) return SK_E_NOMEM;
    {   // staging blocks of the queries that bring their own K/V
        int64_t eph_need = 0;
        for (int i = 0; i < n_items; ++i)
            if (op[i] == SK_OP_QUERY_B) eph_need += (int64_t(cu_tokens[i + 1]) - cu_tokens[i] + 15) / 16;
        if (eph_need > p->L.eph_blocks) return SK_E_WORKSPACE;
    }
    if (p->device) {
        if (!q || !out || (any_kv && (!k || !v))) return SK_E_INVAL;
        if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse)) return SK_E_INVAL;
        int rc = check_out_dtype(p, out_dtype);
        if (rc) return rc;
        Variant vv;
        if (!pick_variant(p, 1, vv)) return SK_E_SHAPE;
    }
    // From here on the sessions change; whatever stops the call afterwards (the lists do not fit the
    // workspace, a HIP call fails) takes every change back, in reverse order.
    ScatterBatch sb;
    sb.k = k; sb.v = v;
    ListGroup groups[3];
    const bool allow_256 = !p->no_256;
    int64_t eph_cursor = 0;
    std::vector<Undo> undo;
    int64_t appended = 0, queried = 0;
    auto take_back = [&](bool keep_copies) {
        for (size_t i = undo.size(); i-- > 0;) rollback(p, undo[i], keep_copies);
    };
    hipStream_t st = (hipStream_t)hip_stream;
    for (int i = 0; i < n_items; ++i) {
        Session* s = get_session(p, session_id[i]);
        const int32_t T = cu_tokens[i + 1] - cu_tokens[i];
        if (T == 0) continue;
        const int32_t id = session_id[i];
        const int64_t n = s->len;
        const int32_t tbl_off = int32_t(int64_t(id) * p->L.max_blocks_per_session);
        TileReq base = {};
        base.tbl_off = tbl_off;
        base.hole_lo = (int32_t)s->frozen; base.hole_hi = (int32_t)s->win;
        if (op[i] == SK_OP_APPEND) {
            Undo u;
            int64_t first_new = 0;
            int rc = grow_session(p, s, T, u, &first_new, st);
            if (rc) { take_back(false); return rc; }
            undo.push_back(u);
            appended += T;
            build_scatter(p, s, id, n, cu_tokens[i], T, first_new, false, 0, sb.items);
            base.pos0 = (int32_t)n; base.kv_vis = int32_t(n + T);
        } else {
            queried += T;
            if (op[i] == SK_OP_QUERY_B) {
                build_scatter(p, nullptr, id, 0, cu_tokens[i], T, 0, true, eph_cursor, sb.items);
                base.pos0 = (int32_t)n; base.kv_vis = (int32_t)n;
                base.eph_blk[0] = (int32_t)eph_cursor; base.eph_cnt[0] = T; base.eph_pos0[0] = (int32_t)n;
                eph_cursor += (T + 15) / 16;
            } else {
                base.pos0 = SK_NO_CAUSAL; base.kv_vis = (int32_t)n;
            }
        }
        // items of more than 128 rows per KV head (the appends) go to the 256-row kernel, which is
        // launched first; then the 128-row items, then the small ones
        Variant vv;
        if (!pick_variant(p, T, vv, allow_256)) { take_back(false); return SK_E_SHAPE; }
        ListGroup& g = groups[vv.id == SK_KV_MFMA64 ? 2 : vv.id == SK_KV_MFMA128 ? 1 : 0];
        g.v = vv; g.q = q; g.out = out; g.lse = lse;
        add_tiles(g, base, cu_tokens[i], T);
    }
    ListPlan plan;
    int rc = plan_list(p, &sb, 1, groups, 3, plan);
    if (rc) { take_back(false); return rc; }
    rc = launch_list(p, plan, &sb, 1, groups, 3, out_dtype, st);
    if (rc) { take_back(plan.scatter_enqueued); return rc; }
    p->stats.tokens_appended += appended;
    p->stats.tokens_queried += queried;
    return SK_OK;
}

int sk_session_query_shared_prefix(sk_pool* p, int32_t id, const void* qp, const void* kp, const void* vp, int32_t P,
                                   const void* qs, const void* ks, const void* vs, int32_t NQ, int32_t Sfx,
                                   void* out_prefix, void* out_suffix, int out_dtype,
                                   float* lse_prefix, float* lse_suffix, void* hip_stream)
{
    if (!p) return SK_E_INVAL;
    Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (P < 0 || NQ < 0 || Sfx < 0) return SK_E_INVAL;
    if (P == 0 && (NQ == 0 || Sfx == 0)) return SK_OK;
    if (!p->device) return SK_E_NODEVICE;
    if (P > 0 && (!qp || !kp || !vp || !out_prefix)) return SK_E_INVAL;
    const bool has_sfx = NQ > 0 && Sfx > 0;
    if (has_sfx && (!qs || !ks || !vs || !out_suffix)) return SK_E_INVAL;
    if (!aligned16(qp) || !aligned16(kp) || !aligned16(vp) || !aligned16(qs) || !aligned16(ks) || !aligned16(vs) ||
        !aligned16(out_prefix) || !aligned16(out_suffix) || !aligned16(lse_prefix) || !aligned16(lse_suffix)) return SK_E_INVAL;
    int rc = check_out_dtype(p, out_dtype);
    if (rc) return rc;
    const int64_t total = int64_t(P) + (has_sfx ? int64_t(NQ) * Sfx : 0);
    const int64_t sfx_blocks = (Sfx + 15) / 16, pre_blocks = (P + 15) / 16;
    if (total > p->L.max_batch_tokens || pre_blocks + (has_sfx ? NQ * sfx_blocks : 0) > p->L.eph_blocks) return SK_E_WORKSPACE;
    Variant vtest;
    if (!pick_variant(p, 1, vtest)) return SK_E_SHAPE;
    const int64_t n = s->len;
    const int32_t tbl_off = int32_t(int64_t(id) * p->L.max_blocks_per_session);
    ScatterBatch sb[2];
    ListGroup groups[2];
    if (P > 0) {
        sb[0].k = kp; sb[0].v = vp;
        build_scatter(p, nullptr, id, 0, 0, P, 0, true, 0, sb[0].items);
        TileReq base = {};
        base.tbl_off = tbl_off; base.pos0 = (int32_t)n; base.kv_vis = (int32_t)n;
        base.hole_lo = (int32_t)s->frozen; base.hole_hi = (int32_t)s->win;
        base.eph_blk[0] = 0; base.eph_cnt[0] = P; base.eph_pos0[0] = (int32_t)n;
        pick_variant(p, P, groups[0].v);
        groups[0].q = qp; groups[0].out = out_prefix; groups[0].lse = lse_prefix;
        add_tiles(groups[0], base, 0, P);
    }
    if (has_sfx) {
        sb[1].k = ks; sb[1].v = vs;
        pick_variant(p, Sfx, groups[1].v);
        groups[1].q = qs; groups[1].out = out_suffix; groups[1].lse = lse_suffix;
        // Short suffixes are packed: several questions share one 256-row tile of the eight-wave
        // kernel (their rows see the same cache and prefix; each sees its own suffix), when a
        // question's rows are a multiple of a wave's 32 and divide 256.
        const int64_t rows_q = int64_t(Sfx) * p->L.G;
        const bool pack = groups[1].v.id != SK_KV_SIMPLE && p->d.head_dim == 128 && rows_q < 256 && rows_q % 32 == 0 &&
                          256 % rows_q == 0 && NQ > 1 && !p->no_pack;
        const int32_t per_tile = pack ? int32_t(256 / rows_q) : 1;
        if (pack) groups[1].v = Variant{SK_KV_MFMA256, 256, 256 / p->L.G};
        for (int32_t j = 0; j < NQ; ++j)
            build_scatter(p, nullptr, id, 0, j * Sfx, Sfx, 0, true, pre_blocks + j * sfx_blocks, sb[1].items);
        for (int32_t j = 0; j < NQ; j += per_tile) {
            const int32_t nq_tile = std::min(per_tile, NQ - j);
            TileReq base = {};
            base.tbl_off = tbl_off; base.pos0 = int32_t(n + P); base.kv_vis = (int32_t)n;
            base.hole_lo = (int32_t)s->frozen; base.hole_hi = (int32_t)s->win;
            base.eph_blk[0] = 0; base.eph_cnt[0] = P; base.eph_pos0[0] = (int32_t)n;
            base.eph_blk[1] = int32_t(pre_blocks + j * sfx_blocks); base.eph_cnt[1] = Sfx; base.eph_pos0[1] = int32_t(n + P);
            if (pack) {
                base.tok_period = Sfx; base.sub_blocks = (int32_t)sfx_blocks;
                base.q_tok0 = j * Sfx; base.n_tok = nq_tile * Sfx;
                groups[1].tiles.push_back(base);
            } else add_tiles(groups[1], base, j * Sfx, Sfx);
        }
    }
    ListPlan plan;
    rc = plan_list(p, sb, 2, groups, 2, plan);
    if (rc) return rc;
    rc = launch_list(p, plan, sb, 2, groups, 2, out_dtype, (hipStream_t)hip_stream);
    if (rc) return rc;
    p->stats.tokens_queried += total;
    return SK_OK;
}

int sk_session_gather(const sk_pool* p, int32_t id, int64_t first, int64_t count, void* k_out, void* v_out, void* hip_stream)
{
    if (!p) return SK_E_INVAL;
    const Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (!p->device) return SK_E_NODEVICE;
    if (first < 0 || count < 0 || first + count > s->retained()) return SK_E_INVAL;
    if (count == 0) return SK_OK;
    if (!k_out || !v_out || !aligned16(k_out) || !aligned16(v_out)) return SK_E_INVAL;
    // retained tokens [first, first+count) = a piece of [0, frozen) followed by a piece of [win, len)
    const int32_t tbl_off = int32_t(int64_t(id) * p->L.max_blocks_per_session);
    const int64_t row_bytes = int64_t(p->d.n_kv_heads) * p->d.head_dim * p->L.elem;
    const int64_t n_a = std::max<int64_t>(0, std::min(first + count, s->frozen) - first);
    if (n_a > 0) {
        int e = sk_launch_gather(p->geom, tbl_off, first, n_a, k_out, v_out, hip_stream);
        if (e) { g_last_hip = e; return SK_E_HIP; }
    }
    if (count > n_a) {
        const int64_t first_b = std::max(first, s->frozen) - s->frozen + s->win;
        int e = sk_launch_gather(p->geom, tbl_off, first_b, count - n_a, (unsigned char*)k_out + n_a * row_bytes,
                                 (unsigned char*)v_out + n_a * row_bytes, hip_stream);
        if (e) { g_last_hip = e; return SK_E_HIP; }
    }
    return SK_OK;
}

int sk_session_truncate(sk_pool* p, int32_t id, int64_t new_length)
{
    if (!p) return SK_E_INVAL;
    Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (new_length < 0 || new_length > s->retained()) return SK_E_INVAL;
    if (new_length <= s->frozen) { s->frozen = new_length; s->win = new_length; s->len = new_length; }
    else s->len = s->win + (new_length - s->frozen);
    const int64_t B = p->d.block_tokens;
    const size_t keep = size_t((s->len + B - 1) / B);
    while (s->blocks.size() > keep) {
        release_block(p, s->blocks.back());
        s->blocks.pop_back();
    }
    return SK_OK;
}

int sk_session_freeze(sk_pool* p, int32_t id, int64_t n_frozen)
{
    if (!p) return SK_E_INVAL;
    Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (s->win != s->frozen) return SK_E_INVAL;           // tokens behind the frozen region were already evicted
    if (n_frozen < s->frozen || n_frozen > s->len) return SK_E_INVAL;
    s->frozen = n_frozen; s->win = n_frozen;
    return SK_OK;
}

int sk_session_evict_oldest(sk_pool* p, int32_t id, int64_t n_tokens, void* hip_stream)
{
    if (!p) return SK_E_INVAL;
    Session* s = get_session(p, id);
    if (!s) return SK_E_BADSESSION;
    if (n_tokens < 0 || n_tokens > s->len - s->win) return SK_E_INVAL;
    if (n_tokens == 0) return SK_OK;
    // blocks that lie entirely inside the hole go back to the pool; storage indices behind them move down
    const int64_t B = p->d.block_tokens;
    const int64_t win = s->win + n_tokens;
    const int64_t b0 = (s->frozen + B - 1) / B, b1 = win / B;
    if (b1 <= b0) {                  // no whole block is freed: the window start moves, nothing else
        s->win = win;
        p->stats.tokens_evicted += n_tokens;
        return SK_OK;
    }
    // The moved tail of the session's device block table is rewritten (ordered on the caller's
    // stream); the host side changes only once that copy is enqueued, so a failure leaves the
    // session as it was.
    const size_t n_moved = s->blocks.size() - (size_t)b1;
    if (n_moved > 0) {
        int slot; unsigned char* host;
        int rc = ring_acquire(p, &slot, &host);
        if (rc) return rc;
        const size_t bytes = n_moved * sizeof(int32_t);
        if (host) memcpy(host, s->blocks.data() + b1, bytes);
        int32_t* dev_tbl = p->device ? (int32_t*)((unsigned char*)p->d.workspace + p->L.off_tables) + int64_t(id) * p->L.max_blocks_per_session + b0
                                     : nullptr;
        rc = ring_copy(p, slot, dev_tbl, bytes, (hipStream_t)hip_stream);
        if (rc) return rc;
    }
    const int64_t k = b1 - b0;
    for (int64_t b = b0; b < b1; ++b) release_block(p, s->blocks[(size_t)b]);
    s->blocks.erase(s->blocks.begin() + b0, s->blocks.begin() + b1);
    s->win = win - k * B; s->len -= k * B;
    p->stats.tokens_evicted += n_tokens;
    return SK_OK;
}

int sk_session_fork(sk_pool* p, int32_t src_id, int64_t n_prefix, int32_t* out_id, void* hip_stream)
{
    if (!p || !out_id) return SK_E_INVAL;
    Session* src = get_session(p, src_id);
    if (!src) return SK_E_BADSESSION;
    if (n_prefix < 0 || n_prefix > src->retained()) return SK_E_INVAL;
    if (p->free_ids.empty()) return SK_E_NOMEM;
    // storage layout of the new session: the same hole as the source if the prefix reaches behind it
    const int64_t B = p->d.block_tokens;
    int64_t frozen, win, len;
    if (n_prefix <= src->frozen) frozen = win = len = n_prefix;
    else { frozen = src->frozen; win = src->win; len = src->win + (n_prefix - src->frozen); }
    const int64_t n_blk = (len + B - 1) / B;
    const bool tail_partial = len % B != 0;      // the new session will write into its last block: it gets a copy
    if (tail_partial && p->free_blocks.empty()) return SK_E_NOMEM;
    const int32_t id = p->free_ids.back();
    std::vector<int32_t> blocks(src->blocks.begin(), src->blocks.begin() + n_blk);
    int32_t tail_src = -1;
    if (tail_partial) { tail_src = blocks.back(); blocks.back() = p->free_blocks.front(); }
    // Device work first (the new session's block table, then the copy of the partly filled last block,
    // all KV heads), into places no live session reads; the host side changes only when both are
    // enqueued, so a failure leaves the pool as it was.
    hipStream_t st = (hipStream_t)hip_stream;
    if (n_blk > 0) {
        int slot; unsigned char* host;
        int rc = ring_acquire(p, &slot, &host);
        if (rc) return rc;
        const size_t bytes = (size_t)n_blk * sizeof(int32_t);
        if (host) memcpy(host, blocks.data(), bytes);
        int32_t* dev_tbl = p->device ? (int32_t*)((unsigned char*)p->d.workspace + p->L.off_tables) + int64_t(id) * p->L.max_blocks_per_session
                                     : nullptr;
        rc = ring_copy(p, slot, dev_tbl, bytes, st);
        if (rc) return rc;
        if (tail_partial) {
            if (inject(p, SK_SITE_BLOCK_COPY)) return SK_E_HIP;
            if (p->device) {
                int e = sk_launch_copy_block(p->geom, (unsigned char*)p->d.kv_mem, tail_src, blocks.back(), st);
                if (e) { g_last_hip = e; return SK_E_HIP; }
            }
        }
    }
    p->free_ids.pop_back();
    Session& d = p->sessions[id];
    d.live = true; d.frozen = frozen; d.win = win; d.len = len;
    d.blocks.swap(blocks);
    for (int64_t i = 0; i < n_blk - (tail_partial ? 1 : 0); ++i) p->refcnt[(size_t)d.blocks[(size_t)i]]++;
    if (tail_partial) {
        p->refcnt[(size_t)d.blocks.back()] = 1;
        p->free_blocks.pop_front();
        p->blocks_in_use++;
    }
    *out_id = id;
    p->stats.forks++;
    return SK_OK;
}

int sk_pool_inject_failure(sk_pool* p, int32_t site, int32_t countdown)
{
    if (!p || site < 0 || site > SK_SITE_PLAN || countdown < 0) return SK_E_INVAL;
    p->inject_site = countdown > 0 ? site : 0;
    p->inject_countdown = countdown;
    return SK_OK;
}

int sk_pool_set_profiling(sk_pool* p, int enable)
{
    if (!p || !p->device) return p ? SK_E_NODEVICE : SK_E_INVAL;
    p->profiling = enable != 0;
    return SK_OK;
}

int sk_pool_read_profile(sk_pool* p, sk_profile* out, float* attn_pc, float* comb_pc, int32_t capacity)
{
    if (!p || !out) return SK_E_INVAL;
    out->calls = p->prof_calls; out->attention_ms = 0; out->combine_ms = 0;
    for (int32_t i = 0; i < p->prof_calls && i < capacity; ++i) {
        if (attn_pc) attn_pc[i] = 0.f;
        if (comb_pc) comb_pc[i] = 0.f;
    }
    int rc = SK_OK;
    for (size_t i = 0; i < p->prof_used && rc == SK_OK; ++i) {
        const sk_pool::ProfRec& r = p->prof[i];
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) { rc = SK_E_HIP; break; }
        if (r.kind == 0) { out->attention_ms += ms; if (attn_pc && r.call < capacity) attn_pc[r.call] += ms; }
        else { out->combine_ms += ms; if (comb_pc && r.call < capacity) comb_pc[r.call] += ms; }
    }
    p->prof_used = 0; p->prof_calls = 0;
    return rc;
}

int64_t sk_pool_element_offset(const sk_pool* p, int64_t block, int32_t kv_head, int32_t is_v, int32_t slot, int32_t dim)
{
    if (!p || block < 0 || block >= p->d.n_blocks || kv_head < 0 || kv_head >= p->d.n_kv_heads ||
        slot < 0 || slot >= p->d.block_tokens || dim < 0 || dim >= p->d.head_dim) return -1;
    int64_t off = block * p->L.blk_stride + int64_t(kv_head) * p->L.head_stride;
    if (!is_v) return off + (int64_t(slot) * p->d.head_dim + dim) * p->L.elem;
    off += p->L.v_off;
    if (p->d.dtype == SK_BF16) return off + ((int64_t(slot >> 4) * p->d.head_dim + dim) * 16 + (slot & 15)) * p->L.elem;
    return off + (int64_t(slot) * p->d.head_dim + dim) * p->L.elem;
}

int sk_pool_get_stats(const sk_pool* p, sk_pool_stats* out)
{
    if (!p || !out) return SK_E_INVAL;
    *out = p->stats;
    return SK_OK;
}

int sk_pool_last_launch(const sk_pool* p, sk_launch_info* out)
{
    if (!p || !out) return SK_E_INVAL;
    *out = p->last;
    return SK_OK;
}

const char* sk_strerror(int status)
{
    switch (status) {
    case SK_OK: return "ok";
    case SK_E_INVAL: return "invalid argument";
    case SK_E_SHAPE: return "unsupported shape";
    case SK_E_DTYPE: return "unsupported element type";
    case SK_E_NOMEM: return "pool exhausted";
    case SK_E_BADSESSION: return "no such session";
    case SK_E_EMPTY: return "softmax over zero keys";
    case SK_E_WORKSPACE: return "buffer too small for this call";
    case SK_E_HIP: return "HIP runtime error";
    case SK_E_NODEVICE: return "metadata-only pool";
    default: return "unknown status";
    }
}

int sk_last_hip_error(void) { return g_last_hip; }
int sk_version(void) { return 2; }

}  // extern "C"
