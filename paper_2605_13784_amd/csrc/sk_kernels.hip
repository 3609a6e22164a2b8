// HIP kernels for gfx950 (CDNA4, wave64): K/V commit (scatter), attention over a paged
// session cache (bf16 MFMA kernel and an fp32 FMA kernel), cross-split log-sum-exp combine,
// gather.  What they compute is defined in include/sk.h; the data layout in sk_internal.h.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "sk_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define SK_NEG_INF (-__builtin_inff())
#define SK_LN2 0.6931471805599453f

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float sk_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float sk_log2(float x) { return __builtin_amdgcn_logf(x); }

// Value of lane (i ^ 32) next to the lane's own, with one v_permlane32_swap (no LDS round trip):
// swapping a register with a copy of itself leaves {x[i % 32], x[i % 32 + 32]} in every lane.
struct sk_halves { float lo, hi; };
__device__ __forceinline__ sk_halves sk_both_halves(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return sk_halves{__uint_as_float(r[0]), __uint_as_float(r[1])};
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{   // round to nearest even; NaN stays NaN
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Work item of workgroup b.  Regular mode derives it from the launch parameters: consecutive
// workgroups differ in KV head first (so with 8 KV heads a head stays on one XCD and its K/V
// stay in that XCD's L2), then in row tile, then in split.
__device__ __forceinline__ int sk_tile_parts(const sk_launch& P, int tok0, int ntok, int* kv_vis_out)
{
    int kv_vis = P.kv_len;
    if (P.pos0 < SK_NO_CAUSAL) {
        int last = P.pos0 + tok0 + ntok;       // last position + 1
        kv_vis = last < kv_vis ? last : kv_vis;
    }
    *kv_vis_out = kv_vis;
    int np = (kv_vis + P.chunk - 1) / P.chunk;
    if (P.eph_cnt[0] > 0 || P.eph_cnt[1] > 0) np += 1;      // uncommitted tokens: own part
    return np < 1 ? 1 : np;
}

__device__ __forceinline__ bool sk_decode_work(const sk_launch& P, int b, sk_work& w)
{
    if (P.mode == SK_MODE_LIST) { w = P.work[b]; return true; }
    const int Hkv = P.g.Hkv;
    int head = b % Hkv, rest = b / Hkv;
    int tile = rest % P.n_tiles, split = rest / P.n_tiles;
    int tok0 = tile * P.tok_per_tile;
    int ntok = P.n_tok - tok0; ntok = ntok < P.tok_per_tile ? ntok : P.tok_per_tile;
    int kv_vis;
    int np = sk_tile_parts(P, tok0, ntok, &kv_vis);
    if (split >= np) return false;
    bool has_eph = (P.eph_cnt[0] > 0 || P.eph_cnt[1] > 0);
    bool eph_part = has_eph && (split == np - 1);
    w.tbl_off = P.tbl_off; w.kv_head = head; w.q_tok0 = tok0; w.n_tok = ntok; w.pos0 = P.pos0 < SK_NO_CAUSAL ? P.pos0 + tok0 : P.pos0;
    w.kv_step = 0;
    if (eph_part) { w.kv_begin = 0; w.kv_end = 0; }
    else if (P.interleave) {          // every split's first piece exists: the host keeps splits <= kv_len / 256
        w.kv_begin = split * 64;
        w.kv_end = kv_vis;
        w.kv_step = (np - (has_eph ? 1 : 0)) * 64;
    } else {
        w.kv_begin = split * P.chunk;
        int e = w.kv_begin + P.chunk;
        w.kv_end = e < kv_vis ? e : kv_vis;
    }
    w.part = (P.n_splits == 1) ? -1 : (tile * P.n_splits + split) * Hkv + head;
    w.unit = tile * Hkv + head; w.part0 = tile * P.n_splits * Hkv + head; w.n_parts = np;
    w.hole_lo = P.hole_lo; w.hole_hi = P.hole_hi;
    w.tok_period = 0; w.sub_blocks = 0;
    for (int i = 0; i < 2; ++i) {
        w.eph_blk[i] = P.eph_blk[i]; w.eph_cnt[i] = eph_part ? P.eph_cnt[i] : 0; w.eph_pos0[i] = P.eph_pos0[i];
    }
    return true;
}

// A run of keys the kernel walks through in 16-token groups: either cached tokens of a session
// (through its block table) or an uncommitted segment in the staging area (through a slice of
// an identity table, so both kinds are addressed the same way).
struct sk_seg {
    const unsigned char* base;   // + head offset already applied
    const int32_t* table;        // block of token t = table[t >> log2B]
    int64_t blk_stride;
    int32_t v_off, B, log2B;
    int32_t begin, end;          // token indices; begin is a multiple of 16
    int32_t step;                // iteration i covers the 64 keys from begin + i * step (64: one contiguous run)
    int32_t pos_shift;           // absolute position = token index + pos_shift
    int32_t hole_lo, hole_n;     // tokens [hole_lo, hole_lo + hole_n) are evicted: streamed, never attended to
    int32_t once;                // 1: no other workgroup of the launch reads these keys (load them non-temporal)
};

// Segment s of a work item: 0 = cached tokens, 1 = first uncommitted segment, 2 + k = second
// uncommitted segment of sub-sequence k (k = 0 unless the tile packs several sequences).
__device__ __forceinline__ sk_seg sk_make_seg(const sk_launch& P, const sk_work& w, int s)
{
    sk_seg g;
    if (s == 0) {
        g.base = P.g.kv + (int64_t)w.kv_head * P.g.head_stride;
        g.table = P.g.tables + w.tbl_off; g.blk_stride = P.g.blk_stride;
        g.v_off = P.g.v_off; g.B = P.g.B; g.log2B = P.g.log2B;
        g.begin = w.kv_begin; g.end = w.kv_end; g.pos_shift = 0;
        g.step = w.kv_step > 0 ? w.kv_step : 64;
        g.hole_lo = w.hole_lo; g.hole_n = w.hole_hi - w.hole_lo;
        g.once = P.kv_once;
    } else {
        g.base = P.g.eph + (int64_t)w.kv_head * P.g.eph_head_stride;
        g.table = P.g.eph_ident + (s == 1 ? w.eph_blk[0] : w.eph_blk[1] + (s - 2) * w.sub_blocks); g.blk_stride = P.g.eph_blk_stride;
        g.v_off = P.g.eph_v_off; g.B = 16; g.log2B = 4;
        g.begin = 0; g.end = (s == 1 ? w.eph_cnt[0] : w.eph_cnt[1]); g.pos_shift = (s == 1 ? w.eph_pos0[0] : w.eph_pos0[1]);
        g.step = 64;
        g.hole_lo = 0; g.hole_n = 0;
        g.once = 0;
    }
    return g;
}

__device__ __forceinline__ const unsigned char* sk_group_base(const sk_seg& g, int tg)
{   // base of the block holding the 16-token group that starts at token tg (tg < g.end)
    // Block tables are only written by the commit kernel of an earlier launch, so inside an
    // attention kernel they are constant: reading them through the constant address space makes
    // the lookup a scalar load (it must not count as a vector memory operation, see below).
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    const int blk = ((const_i32_ptr)(uintptr_t)g.table)[tg >> g.log2B];
    return g.base + (int64_t)blk * g.blk_stride;
}

// One wave merges the split partials of one output row (partial row prow0 of the first split, the
// others pstride rows apart):
//   M = max_s m_s ; w_s = 2^(m_s - M) ; O = sum_s O_s w_s / sum_s l_s w_s ; LSE = (M + log2 sum_s lx_s w_s) ln 2
// Lane s holds the statistics of splits s, s + 64, ..; every lane two output dimensions (one when
// d = 64).  The splits are added in index order whoever calls this (the combine kernel, or a
// workgroup of the attention kernel), with explicit FMAs, so the result depends on the partials only.
// Rows are read BATCH splits at a time, the next batch requested before the current one is used.
// COHERENT: the partials were written by other workgroups of the same launch (with write-through
// stores); they are read with device-scope loads, which see them wherever the reader runs, so the
// reader needs no cache invalidate (measured at over 10 us when every workgroup issues one).
template <bool COHERENT>
__device__ __forceinline__ float sk_ld_partial(const float* p)
{
    if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

template <bool COHERENT, int BATCH>
__device__ __forceinline__ void sk_merge_row(const sk_launch& P, const size_t prow0, const size_t pstride, const int n_parts,
                                             const size_t orow, const int lane)
{
    const int d = P.g.d;
    const bool two = d == 128;
    // dimensions of a lane: COHERENT (32-bit loads) lane and lane + 64; else (64-bit loads) 2 lane, 2 lane + 1
    const int d0 = COHERENT ? lane : (two ? 2 * lane : lane);
    const int d1 = COHERENT ? lane + 64 : 2 * lane + 1;
    const float* obase = P.part_o + prow0 * d + d0;
    const size_t ostride = pstride * d;
    const float* mlbase = P.part_ml + prow0 * 4;
    const size_t mlstride = pstride * 4;
    auto load_o = [&](const int s, float& x0, float& x1) __attribute__((always_inline)) {
        const float* op = obase + (size_t)s * ostride;
        if (COHERENT) { x0 = sk_ld_partial<true>(op); x1 = two ? sk_ld_partial<true>(op + 64) : 0.f; }
        else if (two) { const float2 t = *(const float2*)op; x0 = t.x; x1 = t.y; }
        else { x0 = *op; x1 = 0.f; }
    };
    float M = SK_NEG_INF;
    if (n_parts > 64) {              // rare: the maximum needs its own pass
        for (int s = lane; s < n_parts; s += 64) M = fmaxf(M, sk_ld_partial<COHERENT>(mlbase + (size_t)s * mlstride));
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    }
    float L = 0.f, Lx = 0.f, a0 = 0.f, a1 = 0.f;
    for (int base = 0; base < n_parts; base += 64) {
        const int cnt = n_parts - base < 64 ? n_parts - base : 64;
        float x0[BATCH], x1[BATCH], y0[BATCH], y1[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            x0[j] = 0.f; x1[j] = 0.f;
            if (j < cnt) load_o(base + j, x0[j], x1[j]);
        }
        float m_s = SK_NEG_INF, l_s = 0.f, lx_s = 0.f;
        if (lane < cnt) {
            const float* mp = mlbase + (size_t)(base + lane) * mlstride;
            if (COHERENT) { m_s = sk_ld_partial<true>(mp); l_s = sk_ld_partial<true>(mp + 1); lx_s = sk_ld_partial<true>(mp + 2); }
            else { const float4 t = *(const float4*)mp; m_s = t.x; l_s = t.y; lx_s = t.z; }
        }
        if (n_parts <= 64) {
            M = m_s;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
        }
        const float wgt = (m_s == SK_NEG_INF) ? 0.f : sk_exp2(m_s - M);
        L = fmaf(l_s, wgt, L); Lx = fmaf(lx_s, wgt, Lx);
        for (int j0 = 0; j0 < cnt; j0 += BATCH) {
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {           // request the next batch
                y0[j] = 0.f; y1[j] = 0.f;
                if (j0 + BATCH + j < cnt) load_o(base + j0 + BATCH + j, y0[j], y1[j]);
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const float wj = __shfl(wgt, j0 + j, 64);    // 0 for splits past the end
                a0 = fmaf(x0[j], wj, a0); a1 = fmaf(x1[j], wj, a1);
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) { x0[j] = y0[j]; x1[j] = y1[j]; }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { L += __shfl_xor(L, off, 64); Lx += __shfl_xor(Lx, off, 64); }
    const float inv = 1.0f / L;
    if (P.out_dtype == 0) {
        float* o = (float*)P.out + orow * d;
        if (COHERENT || !two) { o[d0] = a0 * inv; if (two) o[d1] = a1 * inv; }
        else *(float2*)(o + d0) = make_float2(a0 * inv, a1 * inv);
    } else {
        uint16_t* o = (uint16_t*)P.out + orow * d;
        if (COHERENT || !two) { o[d0] = f32_to_bf16_bits(a0 * inv); if (two) o[d1] = f32_to_bf16_bits(a1 * inv); }
        else *(uint32_t*)(o + d0) = f32_to_bf16_bits(a0 * inv) | ((uint32_t)f32_to_bf16_bits(a1 * inv) << 16);
    }
    if (P.lse && lane == 0) P.lse[orow] = (M + sk_log2(Lx)) * SK_LN2;
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA attention kernel, head_dim D = 128 (described below) or 64 (the same with four instead
// of eight 16-dim slices of the first contraction and two instead of four 32-dim blocks of the
// second, in the same LDS layout, half filled; the free-running instances only).
//
// Workgroup = NRG row groups x NPH key phases = 4 or 8 waves: a row group owns 32 query rows, a
// phase owns every NPH-th key tile.  Instances: <4,1,2> 128-row tile; <2,2,2> 64-row tile, the two
// phases merged through LDS at the end; <4,2,2> 128-row tile, eight waves as four row groups x two
// phases; <8,1,4> 256-row tile, eight waves in two groups that take turns on the matrix pipe and
// the vector ALU (described at the segment loop).
//
// Keys move HBM -> LDS with direct-to-LDS loads (global_load_lds_dwordx4), never through
// registers, into a ring of NSS iterations of two 32-key tiles (K 8 KiB + V^T 8 KiB each): 64 KiB
// with two workgroups per CU, or 128 KiB with one.  One iteration consumes two tiles (64 keys:
// both by every wave when NPH = 1, one per phase when NPH = 2) while the others are in flight,
// which is what covers the HBM latency.  A direct-to-LDS load writes lane i's 16 bytes at
// base + 16 i, so the bank swizzle is applied to the *source* address each lane picks:
//   K   : LDS row rho holds global 16-byte chunk (c ^ (rho & 15)) at chunk position c,
//   V^T : LDS row dd of a 16-key group holds the two 8-key halves swapped when bit 3 of dd is set.
// The sixteen loads of one tile are issued by four waves (4 instructions each); a wave waits on
// its own vmcnt and a workgroup barrier publishes the tile.  Nothing else in the loop is a vector
// memory instruction (block-table entries are scalar loads), so the outstanding-load count a
// wave waits for is exact.
// Tiles past the end of a segment re-read its last 16-key group (always valid memory); their
// keys are masked by position.  The commit kernel zero-fills V behind the last committed key of
// a 16-key group, so a masked key never contributes 0 * garbage.
//
// Per 32 keys a wave issues
//   S^T[32 keys][32 rows]  = K[32][128] * Q^T[128][32]        8 x mfma_f32_32x32x16_bf16
//   O^T[128][32 rows]     += V^T[128][32 keys] * P^T[32][32]  8 x mfma_f32_32x32x16_bf16
// With S transposed a lane owns one query row (lane % 32) and 16 keys of it, so the row maximum
// and sum need one cross-lane exchange (lane ^ 32, v_permlane32_swap) and P feeds the second contraction straight
// from registers.  Key row rho of the first product is loaded from key tau(rho) (bits 2 and 3
// swapped) so that the 8 P values a lane hands to one PV instruction belong to 8 consecutive
// keys, which are one 16-byte read of V^T.
// Softmax runs in the log2 domain in fp32; the running maximum is only raised when a tile
// exceeds it by more than SK_RESCALE_SLACK, which keeps exp2 arguments <= the slack and makes
// accumulator rescaling rare; the result is the same up to rounding.
// ---------------------------------------------------------------------------------------------
#define SK_TILE 32                 // keys per tile
#define SK_TILE_BYTES 16384        // K 8 KiB | V^T 8 KiB
#define SK_RESCALE_SLACK 8.0f

template <int N> struct sk_int { static constexpr int value = N; };
typedef __attribute__((address_space(3))) void* sk_lds_ptr;
// LDS operand addresses are kept in the LDS address space explicitly: through a generic pointer
// the compiler may fall back to flat loads, which also count as vector memory operations.
typedef const __attribute__((address_space(3))) unsigned char* sk_lds_cptr;
typedef __attribute__((ext_vector_type(4))) unsigned sk_u32x4;       // one 16-byte MFMA operand
typedef const __attribute__((address_space(3))) sk_u32x4* sk_lds_u4ptr;
typedef const __attribute__((address_space(1))) void* sk_glb_ptr;

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt = simm16[3:0] | simm16[15:14] << 4)
#define SK_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for every
// outstanding global load, i.e. drain the ring of tiles in flight.
__device__ __forceinline__ void sk_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One direct-to-LDS load of 16 bytes per lane: lane i's data lands at lds_addr + IMM + 16 i.
// Written as inline assembly so that the compiler's automatic wait insertion does not drain the
// tiles in flight before every LDS read; the waits are placed by hand (SK_WAIT_VMCNT).
template <unsigned IMM, bool STREAM>
__device__ __forceinline__ void sk_dma16(const void* base, unsigned lane_off, unsigned lds_addr)
{   // address = base (scalar registers) + lane_off (one VGPR, unsigned)
    // STREAM marks the data as used once (cache policy "non-temporal"): it passes through the caches
    // without displacing what other kernels left there.
    if (STREAM)
        asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                     : : "s"(lds_addr), "v"(lane_off), "s"(base), "n"(IMM) : "memory", "m0", "scc");
    else
        asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2"
                     : : "s"(lds_addr), "v"(lane_off), "s"(base), "n"(IMM) : "memory", "m0", "scc");
}

// 16-byte store that is written through to memory at once (cache policy "system coherent"), so that
// the split partials never sit as dirty lines in one XCD's L2: the workgroups that merge them may run
// on another XCD, and a release fence wide enough for that would have to walk the whole L2 for dirty
// lines (measured: about 25 us per kernel).  Written as inline assembly (the compiler has no store
// with these bits outside atomics), so the caller waits for it by hand (SK_WAIT_VMCNT(0)).
typedef __attribute__((ext_vector_type(4))) float sk_f32x4;
__device__ __forceinline__ void sk_store16_through(float* p, const float4 v)
{
    const sk_f32x4 x = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(x) : "memory");
}

// Pool blocks holding the two 16-key groups of the tile that starts at key t0 (scalar loads).
// Groups past the end of the segment fall back to its last group.
struct sk_tile_blocks { uint32_t blk[2]; };
__device__ __forceinline__ sk_tile_blocks sk_lookup_tile(const sk_seg& g, int t0, int last_group)
{
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    sk_tile_blocks b;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int tg = t0 + 16 * j;
        tg = tg < last_group ? tg : last_group;
        b.blk[j] = (uint32_t)((const_i32_ptr)(uintptr_t)g.table)[(unsigned)tg >> g.log2B];
    }
    return b;
}

// Issues the four direct-to-LDS loads with which one of four waves contributes to one tile: a K
// and a V^T load for each of the tile's two 16-key groups.  The address arithmetic per load is
// kept short, because a wave issues it in between its vector or matrix work: the block's byte
// offset is a shift (a block of this kernel holds B * 512 bytes per head), the lane-dependent
// part of the address is one VGPR per kind of load, the same for every tile of a segment:
//   K   : the wave fills LDS rows 16 j + 4 sub .. + 3 of group j; lane -> (row rr, chunk position),
//         source chunk (position ^ rr):        koff = rr * 256 + ((lane & 15) ^ rr) * 16
//   V^T : the wave fills dims 32 sub .. + 31 of group j; lane -> (dim dd, half position),
//         source half (position ^ bit 3 of dd): voff = V offset in the block + dd * 32 + (half ^ ((dd >> 3) & 1)) * 16
// and the 16-key group's offset inside a block of more than 16 tokens is added to those.
// In LDS the sixteen 1 KiB units of a tile (K units 0-7, V^T units 8-15) lie US bytes apart, with
// the same unit of the other tiles of the ring in between; `unit_addr` is the address of unit `sub`.
// With head_dim 64 a tile has half the bytes.  K: rows of 128 bytes, eight to a 1 KiB unit, units
// 0-3; one load per wave and tile (wave sub loads rows 8 (sub & 1) .. + 7 of group sub >> 1, `k_group`,
// into unit sub).  V^T: the same units as with head_dim 128, of which 64 dims fill two per group, so
// only the waves with sub < 2 load it (`v_wave`).
template <unsigned US, int J, int D>
__device__ __forceinline__ void sk_issue_group(const sk_seg& g, int t0, int last_group, uint32_t blk,
                                               unsigned unit_addr, unsigned koff, unsigned voff, int k_group, bool v_wave)
{
    constexpr int LOG2_TOK_BYTES = D == 128 ? 8 : 7;       // K bytes per token and head = V^T bytes per token
    int tg = t0 + 16 * J;
    tg = tg < last_group ? tg : last_group;
    const unsigned char* bb = g.base + ((uint64_t)blk << (g.log2B + LOG2_TOK_BYTES + 1));
    if (g.B > 16) {
        const unsigned slot0 = (unsigned)tg & (unsigned)(g.B - 1);
        koff += slot0 << LOG2_TOK_BYTES;          // K: 256 (128) bytes per token
        voff += slot0 << LOG2_TOK_BYTES;          // V^T: 4 (2) KiB per 16-token group
    }
    if (g.once) {       // uniform over the workgroup
        if (D == 128) sk_dma16<J * 4 * US, true>(bb, koff, unit_addr);
        else if (k_group == J) sk_dma16<0, true>(bb, koff, unit_addr);
        if (D == 128 || v_wave) sk_dma16<(8 + J * 4) * US, true>(bb, voff, unit_addr);
    } else {
        if (D == 128) sk_dma16<J * 4 * US, false>(bb, koff, unit_addr);
        else if (k_group == J) sk_dma16<0, false>(bb, koff, unit_addr);
        if (D == 128 || v_wave) sk_dma16<(8 + J * 4) * US, false>(bb, voff, unit_addr);
    }
}
template <unsigned US, int D>
__device__ __forceinline__ void sk_issue_tile(const sk_seg& g, int t0, int last_group, const sk_tile_blocks& tb,
                                              unsigned unit_addr, unsigned koff, unsigned voff, int k_group, bool v_wave)
{
    sk_issue_group<US, 0, D>(g, t0, last_group, tb.blk[0], unit_addr, koff, voff, k_group, v_wave);
    sk_issue_group<US, 1, D>(g, t0, last_group, tb.blk[1], unit_addr, koff, voff, k_group, v_wave);
}

template <int NRG, int NPH, int NSS, int D>
__device__ __forceinline__ void sk_attn_bf16_body(const sk_launch P)
{
    static_assert(D == 128 || (D == 64 && NSS == 2 && !(NRG == 8 && NPH == 1)),
                  "head_dim 128, or 64 on the free-running instances (whose waits are all for every load)");
    constexpr int NKS = D / 16;              // 16-dim slices of the QK^T contraction
    constexpr int NMT = D / 32;              // 32-dim blocks of the output
    constexpr int NW = NRG * NPH;            // waves: 4 or 8
    constexpr int TPI = 2;                   // tiles per iteration (64 keys)
    constexpr int TPW = TPI / NPH;           // tiles per wave per iteration
    // eight waves either as two groups of row groups that take turns (LOCKSTEP, 256 rows), or as two key
    // phases per row group running freely (128 rows: half the arithmetic per wave of the four-wave
    // 128-row instance, two waves per SIMD)
    constexpr bool LOCKSTEP = NW == 8 && NPH == 1;
    constexpr int NLG = NW / 4;              // groups of four waves; each loads whole tiles
    static_assert(NW == 4 || (LOCKSTEP && NSS == 4) || (NW == 8 && NPH == 2 && NSS == 2), "four waves, or eight as described");
    static_assert(NSS == 2 || NSS == 4, "ring depth in iterations: 64 KiB (two workgroups per CU) or 128 KiB (one)");
    static_assert(NSS * TPI >= (NPH == 1 ? NW : NRG), "the epilogue transposes one 16 KiB tile per wave (per row group with two phases) in the ring");
    // The ring holds NSS iterations of TPI tiles.  Its 1 KiB units are interleaved: unit u of tile t
    // of ring slot s sits at (u * TPI * NSS + t * NSS + s) KiB, so that from a lane's per-unit base
    // address every tile of the ring is within reach of the 16-bit offset field of an LDS read.
    constexpr unsigned US = TPI * NSS * 1024;                 // bytes from unit u to unit u + 1
#define SK_SLOT_OFF(s, t) (((t) * NSS + (s)) * 1024)          // tile t of ring slot s, relative to unit bases
    // (with two key phases the merge of the phases needs 17 KiB per row group: 68 KiB for four row groups)
    constexpr unsigned RING_BYTES = NSS * TPI * SK_TILE_BYTES;
    constexpr unsigned XCH_BYTES = NPH > 1 ? NRG * 17 * 64 * 16 : 0;
    __shared__ __attribute__((aligned(16))) unsigned char lds[RING_BYTES > XCH_BYTES ? RING_BYTES : XCH_BYTES];

    sk_work w;
    if (!sk_decode_work(P, blockIdx.x, w)) return;

    const unsigned lds_base = (unsigned)(uintptr_t)(sk_lds_ptr)lds;   // LDS byte address of the ring
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // in a scalar register
    const int rg = wave % NRG, ph = wave / NRG;
    // Eight waves work as two groups of four that alternate between the matrix pipe and the vector
    // ALU (see the segment loop).  Waves i and i + 4 of a workgroup share a SIMD, so a SIMD holds
    // one wave of each group.  `sub` is the wave's index among the four that load a tile.
    const int grp = LOCKSTEP ? (wave >> 2) : 0;
    const int lg = NLG == 1 ? 0 : (wave >> 2);                     // which tiles of an iteration this wave helps to load (free-running path)
    const int sub = wave & 3;
    const unsigned unit_base = lds_base + sub * US;                // LDS address of this wave's unit of ring slot 0, tile 0
    const int r = lane & 31, kg = lane >> 5;
    // Row i of a tile is head i % G of token i / G (any group size up to 128; rows past the last
    // whole token of a tile are idle).  Rows are below 256, so the division is a multiplication by
    // ceil(2^16 / G) and a shift, exactly.
    const int G = P.g.G;
    const unsigned g_magic = (65536u + (unsigned)G - 1u) / (unsigned)G;
    auto div_g = [&](const int row) __attribute__((always_inline)) { return (int)(((unsigned)row * g_magic) >> 16); };
    const int row_in_tile = rg * 32 + r;
    const int tok_local = div_g(row_in_tile);
    const int hq = w.kv_head * G + (row_in_tile - tok_local * G);
    const bool row_valid = tok_local < w.n_tok;
    // positions of the first and last valid token of this wave (wave-uniform); with a group size that
    // does not divide 32 a token's rows can lie in two waves
    const int wave_tok_first = div_g(rg * 32);
    int wave_tok_last = div_g(rg * 32 + 31);
    if (wave_tok_last > w.n_tok - 1) wave_tok_last = w.n_tok - 1;
    const bool wave_has_rows = wave_tok_first < w.n_tok;
    const bool causal = w.pos0 < SK_NO_CAUSAL;
    // A tile may pack several sequences of tok_period tokens each (questions of a batch): token t of
    // the tile is token t % tok_period of sequence t / tok_period, all sequences start at pos0, and
    // each has its own second uncommitted segment.  A wave's rows belong to one sequence (the host
    // only packs when 32 rows divide a sequence's rows).
    const unsigned period = w.tok_period > 0 ? (unsigned)w.tok_period : 0x7fffffffu;
    const int n_sub = w.tok_period > 0 ? (w.n_tok + w.tok_period - 1) / w.tok_period : 1;
    const int wave_sub = (int)((unsigned)wave_tok_first / period);
    const int p_row = causal ? w.pos0 + (int)((unsigned)(row_valid ? tok_local : wave_tok_last) % period) : 0x7fffffff;
    const int p_wave_min = causal ? w.pos0 + (int)((unsigned)wave_tok_first % period) : 0x7fffffff;
    const int p_wave_max = causal ? w.pos0 + (int)((unsigned)wave_tok_last % period) : 0x7fffffff;

    // Q^T operand: lane (row r, k-group kg) keeps Q[row][16*ks + 8*kg .. +7] for ks = 0..7
    bf16x8 qreg[8];
    {
        uint4 z = make_uint4(0, 0, 0, 0);
        const uint4* qp = (const uint4*)((const unsigned char*)P.q +
                          ((size_t)(w.q_tok0 + (row_valid ? tok_local : 0)) * P.g.Hq + hq) * (D * 2));
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 x = z;
            if (ks < NKS) {
                x = qp[ks * 2 + kg];                   // rows past the tile re-read row 0, then zeroed
                if (!row_valid) x = z;
            }
            qreg[ks] = __builtin_bit_cast(bf16x8, x);
        }
    }

    f32x16 oacc[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[mt][v] = 0.f;
    float m_ref = SK_NEG_INF, l_run = 0.f;
    float lx_run = 0.f;                  // sum of the weights before rounding: what the log-sum-exp is taken from
    const float c_scale = P.g.scale_log2e;
    // key tau(rho): swap bits 2 and 3 of the S^T row index
    const int tau = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);

    // lane-dependent LDS addresses of the MFMA operands inside a tile (the XOR swizzles make them
    // irregular in ks, so they are kept in registers; tile and ring-slot offsets are immediates)
    sk_lds_cptr kptr[8];
    sk_lds_cptr vptr[4];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)       // K row tau is row tau % 4 of unit tau / 4 (head_dim 64: row tau % 8 of unit tau / 8)
        kptr[ks] = D == 128 ? (sk_lds_cptr)lds + SK_SLOT_OFF(0, ph * TPW) + (tau >> 2) * US + (tau & 3) * 256 + (((ks * 2 + kg) ^ (tau & 15)) << 4)
                            : (sk_lds_cptr)lds + SK_SLOT_OFF(0, ph * TPW) + (tau >> 3) * US + (tau & 7) * 128 + (((ks * 2 + kg) ^ (tau & 7)) << 4);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int dd = mt * 32 + r;
        vptr[mt] = (sk_lds_cptr)lds + SK_SLOT_OFF(0, ph * TPW) + (8 + mt) * US + r * 32 + ((kg ^ ((dd >> 3) & 1)) << 4);   // 16-key group q: + 4 q units
    }

#pragma unroll 1
    for (int s = 0; s < 2 + n_sub; ++s) {
        sk_seg g = sk_make_seg(P, w, s);
        if (g.end <= g.begin) continue;
        const int niter = (g.end - g.begin + g.step - 1) / g.step;      // iteration i: keys from g.begin + i * g.step
        const int last_group = (g.end - 1) & ~15;
        // last position of the segment this wave's rows may see; nothing of another sequence's segment
        const int seg_last_pos = (s >= 2 && s - 2 != wave_sub) ? (int)0x80000000 : g.end - 1 + g.pos_shift;
        const int lim_wave_min = p_wave_min < seg_last_pos ? p_wave_min : seg_last_pos;
        const int lim_wave_max = p_wave_max < seg_last_pos ? p_wave_max : seg_last_pos;
        const int lim_row = p_row < seg_last_pos ? p_row : seg_last_pos;

        // lane-dependent parts of the DMA source addresses for this segment
        // (head_dim 64: lane -> (row rr of eight, chunk position of eight), source chunk (position ^ rr),
        // the wave's rows being 8 (sub & 1) .. + 7 of group sub >> 1; V^T has dims for the first two waves only)
        const int krow = D == 128 ? sub * 4 + (lane >> 4) : (sub & 1) * 8 + (lane >> 3);
        const unsigned koff = D == 128 ? (unsigned)(krow * 256 + (((lane & 15) ^ krow) << 4))
                                       : (unsigned)(krow * 128 + (((lane & 7) ^ (krow & 7)) << 4));
        const int k_group = sub >> 1;
        const int vdd = sub * 32 + (lane >> 1);
        const unsigned voff = (unsigned)(g.v_off + vdd * 32 + ((((lane & 1) ^ ((vdd >> 3) & 1))) << 4));
        const bool v_wave = sub < NMT;

        // ---- the three steps of one iteration (64 keys) for this wave; the ring slot is a
        // compile-time constant so that it folds into the offset field of the LDS instructions ----
        f32x16 sacc[TPW];          // S^T of the iteration in flight
        sk_u32x4 va[TPW][2][4];       // its V^T operands (four waves)
        sk_u32x4 va0[4];              // V^T operands of the first 16 keys (eight waves)
        bf16x8 pb[TPW][2];         // its P^T operands

        // first key position of the wave's tiles of iteration `it`, and whether it has work there
        auto first_pos = [&](const int it) __attribute__((always_inline)) { return g.begin + it * g.step + ph * TPW * SK_TILE + g.pos_shift; };
        auto is_active = [&](const int it) __attribute__((always_inline)) {
            return wave_has_rows && g.begin + it * g.step + ph * TPW * SK_TILE < g.end && first_pos(it) <= lim_wave_max;
        };

        // S^T = K Q^T, TPW independent accumulator chains
        // (`soff`: byte offset of the ring slot read, a constant when the loop is unrolled over the slots)
        auto step_scores = [&](const int soff) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[t][v] = 0.f;
            sk_u32x4 ka[TPW][NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int t = 0; t < TPW; ++t)
                    ka[t][ks] = *(sk_lds_u4ptr)(kptr[ks] + soff + SK_SLOT_OFF(0, t));
            __builtin_amdgcn_s_setprio(2);     // the wave feeding the matrix pipe goes first
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int t = 0; t < TPW; ++t)
                    sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[t][ks]), qreg[ks], sacc[t], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
            // all LDS reads first, then the MFMAs back to back (two independent chains)
            __builtin_amdgcn_sched_group_barrier(0x100, NKS * TPW, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, NKS * TPW, 0);
        };
        auto load_v_tile = [&](const int t, const int soff) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int mt = 0; mt < NMT; ++mt)
                    va[t][q][mt] = *(sk_lds_u4ptr)(vptr[mt] + soff + SK_SLOT_OFF(0, t) + q * 4 * US);
        };
        // mask (only tiles that cross a limit), row maximum, P = exp2(s * scale - m), row sums
        auto step_softmax = [&](const int it) __attribute__((always_inline)) {
            const int pos_first = first_pos(it);
            // a tile is masked when it crosses a causal or end-of-segment limit, or touches evicted tokens
            const bool need_mask = pos_first + TPW * SK_TILE - 1 > lim_wave_min ||
                                   (pos_first < g.hole_lo + g.hole_n && pos_first + TPW * SK_TILE > g.hole_lo);
            // the maximum is taken on the raw scores; the softmax scale is applied inside the
            // exponent below (one FMA per score)
            float mt_ = SK_NEG_INF;
            if (need_mask) {
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int pos = pos_first + t * SK_TILE + 16 * (v >> 3) + 8 * kg + (v & 7);
                        const bool vis = pos <= lim_row && (unsigned)(pos - g.hole_lo) >= (unsigned)g.hole_n;
                        const float x = vis ? sacc[t][v] : SK_NEG_INF;
                        sacc[t][v] = x;
                        mt_ = fmaxf(mt_, x);
                    }
            } else {
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mt_ = fmaxf(mt_, sacc[t][v]);
            }
            { const sk_halves h = sk_both_halves(mt_); mt_ = fmaxf(h.lo, h.hi) * c_scale; }      // log2 units (c_scale > 0)
            const bool raise = mt_ > m_ref + SK_RESCALE_SLACK;
            if (__any(raise)) {
                const float alpha = raise ? sk_exp2(m_ref - mt_) : 1.0f;
                l_run *= alpha; lx_run *= alpha;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[mt][v] *= alpha;
                m_ref = raise ? mt_ : m_ref;
            }
            const float neg_m = (m_ref == SK_NEG_INF) ? 0.f : -m_ref;
            float lx0 = 0.f, lx1 = 0.f;
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float p0 = sk_exp2(fmaf(sacc[t][v], c_scale, neg_m)), p1 = sk_exp2(fmaf(sacc[t][8 + v], c_scale, neg_m));
                    pb[t][0][v] = (__bf16)p0;
                    pb[t][1][v] = (__bf16)p1;
                    lx0 += p0; lx1 += p1;
                }
            lx_run += lx0 + lx1;
            // The row sum that normalises the output is taken over the weights as the matrix pipe sees
            // them (rounded to bf16), two per instruction with fp32 accumulation: numerator and
            // denominator of the output then carry the same weights, so a row that one key dominates
            // keeps that key's value to fp32 accuracy whatever the rounding of its weight (with the lazy
            // maximum that weight is not 1).  The log-sum-exp is taken from the unrounded weights
            // (lx_run, above), so it does not carry the rounding.
            const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
            float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    ls0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[t][q], pb[t][q], 0, 1), ones, ls0, false);
                    ls1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[t][q], pb[t][q], 2, 3), ones, ls1, false);
                    ls0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[t][q], pb[t][q], 4, 5), ones, ls0, false);
                    ls1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pb[t][q], pb[t][q], 6, 7), ones, ls1, false);
                }
            l_run += ls0 + ls1;
        };
        // O^T += V^T P^T for one tile
        auto pv_tile = [&](const int t) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int mt = 0; mt < NMT; ++mt)
                    oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[t][q][mt]), pb[t][q], oacc[mt], 0, 0, 0);
        };

        sk_lds_barrier();                      // ring free (previous segment fully consumed)
        // The query operand must have arrived before the loop (a wait for it placed by the
        // compiler inside the loop would drain the ring on every iteration).
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) asm volatile("" : : "v"(qreg[ks]));

        if constexpr (!LOCKSTEP) {
            // ---- free-running waves: every wave walks S, softmax, PV of an iteration in turn; overlap of
            // matrix and vector work comes from the other wave of the SIMD (the other workgroup on the
            // CU for the four-wave instances, the other key phase for the eight-wave one) ----
            constexpr int LPW = 4 * TPI / NLG;   // direct-to-LDS loads per wave per iteration (tile p is loaded by wave group p % NLG)
            // prologue: iterations 0 .. NSS-2
#pragma unroll
            for (int a = 0; a < NSS - 1; ++a) {
                if (a < niter) {
#pragma unroll
                    for (int p = 0; p < TPI; ++p) {
                        if (NLG > 1 && (p % NLG) != lg) continue;
                        const int t0 = g.begin + a * g.step + p * SK_TILE;
                        const sk_tile_blocks tb = sk_lookup_tile(g, t0, last_group);
                        sk_issue_tile<US, D>(g, t0, last_group, tb, unit_base + SK_SLOT_OFF(a, p), koff, voff, k_group, v_wave);
                    }
                }
            }
            // block ids of the next refill are looked up one iteration ahead of their use
            sk_tile_blocks nb[TPI];
#pragma unroll
            for (int p = 0; p < TPI; ++p)
                nb[p] = sk_lookup_tile(g, g.begin + (NSS - 1) * g.step + p * SK_TILE, last_group);

            // `slot` is the ring slot the iteration reads; the slot read by the previous iteration is
            // refilled with iteration it + NSS - 1.  With the two-slot ring the loop is unrolled over the
            // slots (the slot offsets fold into the LDS instructions); a four-slot ring takes the slot at
            // run time (one copy of the loop body).  The four-wave instances in use have two slots: with
            // four (three iterations in flight, 128 KiB, one workgroup per CU) a query measured slower
            // (32 tokens at 32K: 38 against 33 us; 16 tokens at 128K: 103 against 98 us).
            auto iteration = [&](const int it, const int slot) __attribute__((always_inline)) {
                // this wave's loads of iteration `it` have landed: everything but the loads of the
                // (at most NSS - 2) later iterations already issued
                const int later = niter - 1 - it;
                if (NSS == 2 || later <= 0) SK_WAIT_VMCNT(0);
                else if (later == 1) SK_WAIT_VMCNT(LPW);
                else SK_WAIT_VMCNT(2 * LPW);
                sk_lds_barrier();
                if (it + NSS - 1 < niter) {
#pragma unroll
                    for (int p = 0; p < TPI; ++p) {
                        if (NLG > 1 && (p % NLG) != lg) continue;
                        sk_issue_tile<US, D>(g, g.begin + (it + NSS - 1) * g.step + p * SK_TILE, last_group, nb[p],
                                                       unit_base + SK_SLOT_OFF((slot + NSS - 1) % NSS, p), koff, voff, k_group, v_wave);
                    }
                    if (it + NSS < niter) {
#pragma unroll
                        for (int p = 0; p < TPI; ++p)
                            nb[p] = sk_lookup_tile(g, g.begin + (it + NSS) * g.step + p * SK_TILE, last_group);
                    }
                }
                if (!is_active(it)) return;
                step_scores(slot * 1024);
#pragma unroll
                for (int t = 0; t < TPW; ++t) load_v_tile(t, slot * 1024);   // requested now: their LDS latency hides behind the softmax
                step_softmax(it);
#pragma unroll
                for (int t = 0; t < TPW; ++t) pv_tile(t);
            };
            if constexpr (NSS == 2) {
                for (int it = 0; it < niter; it += 2) {
                    iteration(it, 0);
                    if (it + 1 < niter) iteration(it + 1, 1);
                }
            } else {
#pragma unroll 1
                for (int it = 0; it < niter; ++it) iteration(it, it & (NSS - 1));
            }
        } else {
            // ---- eight waves in two groups of four that take turns.  Every wave alternates between
            // a matrix slot (P V of iteration j-1, then S of iteration j) and a vector slot (softmax
            // of iteration j), with a workgroup barrier in front of each; group 1 runs the same
            // sequence one barrier behind group 0, so that whenever one group is in a matrix slot the
            // other is in a vector slot.  A SIMD holds one wave of each group: its matrix pipe and
            // its vector ALU are busy at the same time.
            //   barrier number    2j              2j+1            2j+2
            //   group 0           | PV(j-1) S(j)  | softmax(j)    | PV(j) S(j+1)
            //   group 1           | softmax(j-1)  | PV(j-1) S(j)  | softmax(j)
            // Iteration i lives in ring slot i % 4 and is read between barriers 2i and 2i+4.  Group
            // 0 loads the second tile of every iteration, group 1 the first; a wave issues the loads
            // of iteration j + 2 + grp at the start of its vector slot j (after barrier 2j+1+grp >=
            // 2(j + grp - 2) + 4, so the ring slot is free) and waits for its loads of iteration i
            // before its barrier number 2i, after which the whole iteration is in LDS.
            // The ring slot is a run-time value here (one copy of the loop body): the operand
            // addresses of the current slot are rebuilt from the per-unit bases once per iteration.
            // Every wave does every iteration (rows or keys that do not count are masked): the slots
            // are synchronised, so skipping work would not save time.
            constexpr int LPW = 4;               // direct-to-LDS loads per wave per iteration (one tile)
            const int my_tile = 1 - grp;
            const int ahead = 2 + grp;           // iterations loaded before the loop
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                if (a < ahead && a < niter) {
                    const int t0 = g.begin + a * g.step + my_tile * SK_TILE;
                    const sk_tile_blocks tb = sk_lookup_tile(g, t0, last_group);
                    sk_issue_tile<US, D>(g, t0, last_group, tb, unit_base + SK_SLOT_OFF(a, my_tile), koff, voff, k_group, v_wave);
                }
            }
            sk_tile_blocks nb = sk_lookup_tile(g, g.begin + ahead * g.step + my_tile * SK_TILE, last_group);
            {   // iteration 0 has landed: all but the loads of the later iterations issued above
                const int issued = niter < ahead ? niter : ahead;
                if (issued >= 3) SK_WAIT_VMCNT(2 * LPW); else if (issued == 2) SK_WAIT_VMCNT(LPW); else SK_WAIT_VMCNT(0);
            }
            if (grp == 1) sk_lds_barrier();      // group 1 stays one barrier behind
            // wait for this wave's loads of iteration i; those of iteration i + 1 may still be in flight
            auto wait_iteration = [&](const int i) __attribute__((always_inline)) {
                if (i + 1 < niter) SK_WAIT_VMCNT(LPW); else SK_WAIT_VMCNT(0);
            };
            auto refill = [&](const int j) __attribute__((always_inline)) {
                const int i = j + ahead;
                if (i < niter) {
                    sk_issue_tile<US, D>(g, g.begin + i * g.step + my_tile * SK_TILE, last_group, nb,
                                                   unit_base + SK_SLOT_OFF(i & 3, my_tile), koff, voff, k_group, v_wave);
                    if (i + 1 < niter) nb = sk_lookup_tile(g, g.begin + (i + 1) * g.step + my_tile * SK_TILE, last_group);
                }
            };
            // Matrix slot: eight groups of four matrix instructions, P V of the previous iteration
            // (V^T through vp, the pointers of its ring slot) and S of the current one (K through
            // kc).  Operands stream from LDS two groups ahead of their use, into the registers that
            // earlier groups have released (the scheduling barriers keep that order); the first
            // group's were read in the vector slot.  KIND 0: first slot of a segment, S only;
            // 2: last slot, P V only.
            auto matrix_slot = [&](auto kind_const, const int j, const sk_lds_cptr (&kc)[8], const sk_lds_cptr (&vp)[4])
                                   __attribute__((always_inline)) {
                constexpr int KIND = decltype(kind_const)::value;
                auto ld_v = [&](sk_u32x4 (&o)[4], const int t, const int q) __attribute__((always_inline)) {
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) o[mt] = *(sk_lds_u4ptr)(vp[mt] + SK_SLOT_OFF(0, t) + q * 4 * US);
                };
                auto mm_v = [&](const sk_u32x4 (&o)[4], const int t, const int q) __attribute__((always_inline)) {
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt)
                        oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o[mt]), pb[t][q], oacc[mt], 0, 0, 0);
                };
                auto ld_k = [&](sk_u32x4 (&o)[4], const int kk) __attribute__((always_inline)) {      // ks = 2 kk, 2 kk + 1; both tiles
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = *(sk_lds_u4ptr)(kc[kk * 2 + (i >> 1)] + SK_SLOT_OFF(0, i & 1));
                };
                auto mm_k = [&](const sk_u32x4 (&o)[4], const int kk) __attribute__((always_inline)) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        sacc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o[i]), qreg[kk * 2 + (i >> 1)], sacc[i & 1], 0, 0, 0);
                };
                auto clear_scores = [&]() __attribute__((always_inline)) {
#pragma unroll
                    for (int t = 0; t < 2; ++t)
#pragma unroll
                        for (int v = 0; v < 16; ++v) sacc[t][v] = 0.f;
                };
#define SK_SB __builtin_amdgcn_sched_barrier(0)
                sk_u32x4 o1[4], o2[4], o3[4], o4[4], o5[4], o6[4], o7[4];
                if (KIND == 1) {
                    ld_v(o1, 0, 1); ld_v(o2, 1, 0); SK_SB;
                    mm_v(va0, 0, 0); SK_SB; ld_v(o3, 1, 1); SK_SB;
                    mm_v(o1, 0, 1); SK_SB; ld_k(o4, 0); SK_SB;
                    mm_v(o2, 1, 0); SK_SB; ld_k(o5, 1); SK_SB;
                    mm_v(o3, 1, 1); SK_SB; ld_k(o6, 2); SK_SB;
                    clear_scores(); mm_k(o4, 0); SK_SB; ld_k(o7, 3); SK_SB;
                    mm_k(o5, 1); SK_SB;
                    mm_k(o6, 2); SK_SB;
                    mm_k(o7, 3);
                } else if (KIND == 0) {
                    ld_k(o4, 0); ld_k(o5, 1); ld_k(o6, 2); ld_k(o7, 3);
                    clear_scores();
                    mm_k(o4, 0); mm_k(o5, 1); mm_k(o6, 2); mm_k(o7, 3);
                } else {
                    ld_v(o1, 0, 1); ld_v(o2, 1, 0); ld_v(o3, 1, 1);
                    mm_v(va0, 0, 0); mm_v(o1, 0, 1); mm_v(o2, 1, 0); mm_v(o3, 1, 1);
                }
#undef SK_SB
            };
            // Vector slot: softmax of iteration j, and the operands of the first group of matrix
            // instructions of the slot that follows (V^T, first 16 keys of the iteration).
            auto vector_slot = [&](const int j, const sk_lds_cptr (&vc)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) va0[mt] = *(sk_lds_u4ptr)(vc[mt]);
                step_softmax(j);
            };
            sk_lds_cptr kc[8];          // K operand addresses in the ring slot of the current iteration
            sk_lds_cptr vc[4];          // V^T operand addresses in it (the next matrix slot reads them as "previous")
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) kc[ks] = kptr[ks];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) vc[mt] = vptr[mt];
            // slots of iteration 0 (ring slot 0): S only
            sk_lds_barrier();
            matrix_slot(sk_int<0>{}, 0, kc, vc);
            if (grp == 1 && 1 < niter) wait_iteration(1);
            sk_lds_barrier();
            refill(0);
            vector_slot(0, vc);
#pragma unroll 1
            for (int j = 1; j < niter; ++j) {
                sk_lds_cptr vp[4];
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) { vp[mt] = vc[mt]; vc[mt] = vptr[mt] + (j & 3) * 1024; }
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) kc[ks] = kptr[ks] + (j & 3) * 1024;
                if (grp == 0) wait_iteration(j);
                    sk_lds_barrier();                                  // barrier 2j (group 0), 2j+1 (group 1)
                matrix_slot(sk_int<1>{}, j, kc, vp);
                if (grp == 1 && j + 1 < niter) wait_iteration(j + 1);
                sk_lds_barrier();                                  // barrier 2j+1 (group 0), 2j+2 (group 1)
                refill(j);
                vector_slot(j, vc);
            }
            // slots after the last iteration: P V only
            sk_lds_barrier();
            matrix_slot(sk_int<2>{}, niter, kc, vc);
            sk_lds_barrier();
            if (grp == 0) sk_lds_barrier();      // the barrier group 1 took first
        }
    }

    float l_tot; { const sk_halves h = sk_both_halves(l_run); l_tot = h.lo + h.hi; }
    float lx_tot; { const sk_halves h = sk_both_halves(lx_run); lx_tot = h.lo + h.hi; }

    if (NPH > 1) {
        // merge the key phases of each row group through LDS: per row group 17 x 64 float4 (lane-major, so a
        // wave's 16-byte accesses are conflict-free): entries 0..15 the accumulators, entry 16 = (m, l, lx, -)
        __syncthreads();                                  // every wave is done reading key tiles
        float4* xch = (float4*)lds + rg * (17 * 64) + lane;
        if (ph == 1) {
#pragma unroll
            for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    xch[(mt * 4 + q4) * 64] = make_float4(oacc[mt][q4 * 4 + 0], oacc[mt][q4 * 4 + 1], oacc[mt][q4 * 4 + 2], oacc[mt][q4 * 4 + 3]);
            xch[16 * 64] = make_float4(m_ref, l_tot, lx_tot, 0.f);
        }
        __syncthreads();
        if (ph == 0) {
            const float4 s1 = xch[16 * 64];
            const float m1 = s1.x, l1 = s1.y, lx1 = s1.z;
            const float M = fmaxf(m_ref, m1);
            const float a0 = (m_ref == SK_NEG_INF) ? 0.f : sk_exp2(m_ref - M);
            const float a1 = (m1 == SK_NEG_INF) ? 0.f : sk_exp2(m1 - M);
#pragma unroll
            for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const float4 x = xch[(mt * 4 + q4) * 64];
                    oacc[mt][q4 * 4 + 0] = oacc[mt][q4 * 4 + 0] * a0 + x.x * a1;
                    oacc[mt][q4 * 4 + 1] = oacc[mt][q4 * 4 + 1] * a0 + x.y * a1;
                    oacc[mt][q4 * 4 + 2] = oacc[mt][q4 * 4 + 2] * a0 + x.z * a1;
                    oacc[mt][q4 * 4 + 3] = oacc[mt][q4 * 4 + 3] * a0 + x.w * a1;
                }
            l_tot = l_tot * a0 + l1 * a1;
            lx_tot = lx_tot * a0 + lx1 * a1;
            m_ref = M;
        }
        __syncthreads();                                  // the exchange area is read; the transposes reuse it
    }

    // ---- epilogue: rows go out through LDS so that every store instruction writes whole rows ----
    // A lane holds 4-float pieces of ONE row (its accumulators are O^T); written as they are, a store
    // instruction would touch 64 different 128-byte lines.  Each wave transposes its 32 x 128 tile in
    // 16 KiB of the (now idle) ring, XOR-swizzled by row so both directions are conflict-free (the
    // ring holds one such tile per wave: 64 KiB for four waves, 128 KiB for eight).
    if (NPH == 1) __syncthreads();                    // every wave is done reading key tiles
    const bool direct = w.part < 0;
    if (NPH == 1 || ph == 0) {                        // with two key phases, phase 0 holds the merged rows
        const float inv = direct ? 1.0f / l_tot : 1.0f;
        float* tr = (float*)lds + (NPH == 1 ? wave : rg) * 4096;
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int c4 = mt * 8 + q4 * 2 + kg;
                *(float4*)(tr + r * 128 + ((c4 ^ r) & 31) * 4) =
                    make_float4(oacc[mt][q4 * 4 + 0] * inv, oacc[mt][q4 * 4 + 1] * inv, oacc[mt][q4 * 4 + 2] * inv, oacc[mt][q4 * 4 + 3] * inv);
            }
        const size_t orow_lane = ((size_t)(w.q_tok0 + tok_local) * P.g.Hq + hq);
        if (row_valid && kg == 0) {
            if (direct) { if (P.lse) P.lse[orow_lane] = (m_ref + sk_log2(lx_tot)) * SK_LN2; }
            else sk_store16_through(P.part_ml + ((size_t)w.part * P.rows_per_slot + row_in_tile) * 4, make_float4(m_ref, l_tot, lx_tot, 0.f));
        }
        // a row is D / 4 chunks of four floats: a store instruction writes two rows (four at head_dim 64)
        constexpr int CPR = D / 4, RPI = 64 / CPR, NIT = 32 / RPI;
        const int c4 = lane & (CPR - 1);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            // the row order is rotated by the workgroup index: workgroups that finish together (short
            // contexts) would otherwise all write the same offset of their partial slots, which lie a
            // power of two apart, at the same time, and crowd onto a few memory channels
            const int row = ((it + blockIdx.x) & (NIT - 1)) * RPI + lane / CPR;
            const float4 val = *(const float4*)(tr + row * 128 + ((c4 ^ row) & 31) * 4);
            const int rit = rg * 32 + row;                 // row inside the tile
            const int tok2 = div_g(rit);
            if (tok2 >= w.n_tok) continue;
            if (direct) {
                const size_t orow = ((size_t)(w.q_tok0 + tok2) * P.g.Hq + w.kv_head * G + (rit - tok2 * G));
                if (P.out_dtype == 0) *(float4*)((float*)P.out + orow * D + c4 * 4) = val;
                else {
                    const uint32_t lo = f32_to_bf16_bits(val.x) | ((uint32_t)f32_to_bf16_bits(val.y) << 16);
                    const uint32_t hi = f32_to_bf16_bits(val.z) | ((uint32_t)f32_to_bf16_bits(val.w) << 16);
                    *(uint2*)((uint16_t*)P.out + orow * D + c4 * 4) = make_uint2(lo, hi);
                }
            } else {
                sk_store16_through(P.part_o + ((size_t)w.part * P.rows_per_slot + rit) * D + c4 * 4, val);
            }
        }
    }
    SK_WAIT_VMCNT(0);                                 // the partial's stores (inline assembly) have completed
    if (direct || !P.fuse) return;

    // ---- in-kernel merge of the split partials ----
    // The workgroups of one (row tile, KV head) are a unit.  Each has written its partial above; it
    // now arrives at the unit's counter and waits, for a bounded number of polls, until all have
    // arrived; then every workgroup of the unit merges its own share of the tile's rows (split k the
    // rows k * rps ..), reading the other partials through the L2.  A workgroup that gives up waiting
    // says so in the counter's high bits and leaves; the last workgroup to arrive (which never waits,
    // so the scheme needs no two workgroups to be resident together) then merges every share.  Who
    // merges a row does not change its value: sk_merge_row adds the splits in index order.
    __syncthreads();                                  // the whole partial is written (and LDS is free again)
    volatile int* flag = (volatile int*)lds;
    uint32_t* cnt = P.sync + 2 * (size_t)w.unit;
    uint32_t left = 0;
    // Release: every thread has waited for its write-through stores and passed the barrier above, so
    // the partial is in memory before the arrival below.  Acquire: the merge reads the partials with
    // device-scope loads, issued after the counter has said that everybody has arrived (the fence below
    // only keeps the compiler and this workgroup's waves from reading earlier).
    if (tid == 0) {
        if (P.merge_fences) __threadfence();
        const uint32_t np = (uint32_t)w.n_parts;
        const uint32_t old = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int state;                                    // 0: leave, 1: merge the own share, 2: merge every share
        if ((old & 0xffffu) + 1u == np) state = (old >> 16) ? 2 : 1;
        else {
            state = 0;
            for (int i = 0; i < P.wait_polls; ++i) {
                __builtin_amdgcn_s_sleep(4);
                if ((__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xffffu) == np) { state = 1; break; }
            }
            if (state == 0) {
                // gave up.  The mark and the last arrival are atomic operations on one word: either the last
                // arriver sees the mark (and merges this share), or this sees that everybody has arrived.
                const uint32_t o2 = __hip_atomic_fetch_add(cnt, 0x10000u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((o2 & 0xffffu) == np) state = 1;
            }
        }
        if (P.merge_fences) __threadfence(); else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        // departure (this workgroup will not look at the arrival counter again), requested now so that
        // its round trip runs beside the merge; the answer is needed at the very end only
        left = __hip_atomic_fetch_add(cnt + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = state;
    }
    __syncthreads();
    const int state = *flag;
    if (state != 0) {
        const int nrows = w.n_tok * G;
        const int rps = (nrows + w.n_parts - 1) / w.n_parts;
        const int k_own = (w.part - w.part0) / P.g.Hkv;
        const int k_lo = state == 2 ? 0 : k_own, k_hi = state == 2 ? w.n_parts : k_own + 1;
        for (int k = k_lo; k < k_hi; ++k) {
            const int row_end = (k + 1) * rps < nrows ? (k + 1) * rps : nrows;
            for (int row = k * rps + wave; row < row_end; row += NW) {
                const int tok3 = div_g(row);
                const size_t orow = (size_t)(w.q_tok0 + tok3) * P.g.Hq + w.kv_head * G + (row - tok3 * G);
                sk_merge_row<true, 16>(P, (size_t)w.part0 * P.rows_per_slot + row, (size_t)P.g.Hkv * P.rows_per_slot, w.n_parts, orow, lane);
            }
        }
    }
    // the last workgroup of the unit to depart clears the counters for the next launch
    if (tid == 0) {
        if (left + 1u == (uint32_t)w.n_parts) {
            __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(cnt + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// The kernels proper: head_dim 128 (all four instances) and head_dim 64 (the free-running ones).
template <int NRG, int NPH, int NSS>
__global__ __launch_bounds__(64 * NRG * NPH, NRG * NPH == 8 ? 1 : 2) void sk_attn_bf16_d128(const sk_launch P)
{
    sk_attn_bf16_body<NRG, NPH, NSS, 128>(P);
}
template <int NRG, int NPH, int NSS>
__global__ __launch_bounds__(64 * NRG * NPH, NRG * NPH == 8 ? 1 : 2) void sk_attn_bf16_d64(const sk_launch P)
{
    sk_attn_bf16_body<NRG, NPH, NSS, 64>(P);
}

// ---------------------------------------------------------------------------------------------
// fp32-arithmetic attention kernel (fp32 pools, and bf16 pools whose shape the MFMA kernel does
// not take).  Tile of up to 16 query rows x 32 keys; every product and sum is an fp32 FMA.
// Thread (r = tid/16, c = tid%16): scores of row r for keys c and c+16; output
// dimensions c + 16 j of row r.
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void sk_attn_simple(const sk_launch P)
{
    constexpr int DMAX = 128;
    __shared__ float Qs[16][DMAX + 1];
    __shared__ float Ks[32][DMAX + 1];
    __shared__ float Vs[32][DMAX + 1];
    __shared__ float Ps[16][32 + 1];

    sk_work w;
    if (!sk_decode_work(P, blockIdx.x, w)) return;
    const int tid = threadIdx.x, r = tid >> 4, c = tid & 15;
    const int d = P.g.d, G = P.g.G, Hq = P.g.Hq;
    const int nrows = w.n_tok * G;
    const bool row_valid = r < nrows;
    const int tok_local = row_valid ? r / G : 0;
    const int hq = w.kv_head * G + (row_valid ? r % G : 0);
    const bool causal = w.pos0 < SK_NO_CAUSAL;
    const int p_row = causal ? w.pos0 + tok_local : 0x7fffffff;
    const float c_scale = P.g.scale_log2e;
    const int nd = d >> 4;          // output dims per thread

    for (int idx = tid; idx < 16 * d; idx += 256) {
        int rr = idx / d, t = idx % d;
        float x = 0.f;
        if (rr < nrows) {
            size_t off = ((size_t)(w.q_tok0 + rr / G) * Hq + (w.kv_head * G + rr % G)) * d + t;
            x = BF16 ? bf16_bits_to_f32(((const uint16_t*)P.q)[off]) : ((const float*)P.q)[off];
        }
        Qs[rr][t] = x;
    }
    float o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = 0.f;
    float m_run = SK_NEG_INF, l_run = 0.f;

    for (int s = 0; s < 3; ++s) {
        sk_seg g = sk_make_seg(P, w, s);
        for (int t0 = g.begin; t0 < g.end; t0 += 32) {
            __syncthreads();
            // stage 32 keys and values as fp32, zero past the end
            for (int idx = tid; idx < 32 * d; idx += 256) {
                int tt = idx / d, t = idx % d;
                int tok = t0 + tt;
                float kx = 0.f, vx = 0.f;
                if (tok < g.end) {
                    const unsigned char* bb = sk_group_base(g, tok & ~15);
                    int slot = tok & (g.B - 1);
                    if (BF16) {
                        kx = bf16_bits_to_f32(((const uint16_t*)bb)[(size_t)slot * d + t]);
                        vx = bf16_bits_to_f32(((const uint16_t*)(bb + g.v_off))[((size_t)(slot >> 4) * d + t) * 16 + (slot & 15)]);
                    } else {
                        kx = ((const float*)bb)[(size_t)slot * d + t];
                        vx = ((const float*)(bb + g.v_off))[(size_t)slot * d + t];
                    }
                }
                Ks[tt][t] = kx; Vs[tt][t] = vx;
            }
            __syncthreads();
            const int seg_last_pos = g.end - 1 + g.pos_shift;
            const int lim = p_row < seg_last_pos ? p_row : seg_last_pos;
            float sc[2];
            float mt_ = SK_NEG_INF;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int tt = c + 16 * j;
                float acc = 0.f;
                for (int t = 0; t < d; ++t) acc = fmaf(Qs[r][t], Ks[tt][t], acc);
                float x = acc * c_scale;
                x = (t0 + tt + g.pos_shift <= lim && (unsigned)(t0 + tt - g.hole_lo) >= (unsigned)g.hole_n) ? x : SK_NEG_INF;
                sc[j] = x;
                mt_ = fmaxf(mt_, x);
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) mt_ = fmaxf(mt_, __shfl_xor(mt_, off, 64));
            const float m_new = fmaxf(m_run, mt_);
            const float m_use = (m_new == SK_NEG_INF) ? 0.f : m_new;
            const float alpha = (m_run == SK_NEG_INF) ? 0.f : sk_exp2(m_run - m_use);
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float p = sk_exp2(sc[j] - m_use);
                Ps[r][c + 16 * j] = p;
                psum += p;
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) psum += __shfl_xor(psum, off, 64);
            l_run = l_run * alpha + psum;
            m_run = m_new;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j < nd) {
                    float acc = o[j] * alpha;
                    const int t = c + 16 * j;
                    for (int tt = 0; tt < 32; ++tt) acc = fmaf(Ps[r][tt], Vs[tt][t], acc);
                    o[j] = acc;
                }
            }
        }
    }
    if (!row_valid) return;
    const size_t orow = ((size_t)(w.q_tok0 + tok_local) * Hq + hq);
    if (w.part < 0) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < nd) {
                const int t = c + 16 * j;
                if (P.out_dtype == 0) ((float*)P.out)[orow * d + t] = o[j] * inv;
                else ((uint16_t*)P.out)[orow * d + t] = f32_to_bf16_bits(o[j] * inv);
            }
        }
        if (P.lse && c == 0) P.lse[orow] = (m_run + sk_log2(l_run)) * SK_LN2;
    } else {
        const size_t prow = (size_t)w.part * P.rows_per_slot + r;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < nd) P.part_o[prow * d + c + 16 * j] = o[j];
        if (c == 0) *((float4*)P.part_ml + prow) = make_float4(m_run, l_run, l_run, 0.f);
    }
}

// ---------------------------------------------------------------------------------------------
// Cross-split combine: one wave per output row.
//   M = max_s m_s ; L = sum_s l_s 2^(m_s - M) ; O = sum_s O_s 2^(m_s - M) / L
//   LSE = (M + log2 sum_s lx_s 2^(m_s - M)) ln 2       (lx: the row sums before bf16 rounding)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sk_combine(const sk_launch P)
{
    const int groups_per_tile = P.rows_per_slot >> 2;
    const int item = blockIdx.x / groups_per_tile;
    const int row = (blockIdx.x % groups_per_tile) * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    sk_comb cb;
    if (P.mode == SK_MODE_LIST) cb = P.comb[item];
    else {
        const int Hkv = P.g.Hkv;
        int head = item % Hkv, tile = item / Hkv;
        int tok0 = tile * P.tok_per_tile;
        int ntok = P.n_tok - tok0; ntok = ntok < P.tok_per_tile ? ntok : P.tok_per_tile;
        int kv_vis;
        cb.n_parts = sk_tile_parts(P, tok0, ntok, &kv_vis);
        cb.part0 = tile * P.n_splits * Hkv + head; cb.part_stride = Hkv;
        cb.q_tok0 = tok0; cb.n_tok = ntok; cb.kv_head = head;
    }
    const int G = P.g.G;
    if (row >= cb.n_tok * G) return;
    const size_t orow = ((size_t)(cb.q_tok0 + row / G) * P.g.Hq + cb.kv_head * G + row % G);
    sk_merge_row<false, 8>(P, (size_t)cb.part0 * P.rows_per_slot + row, (size_t)cb.part_stride * P.rows_per_slot, cb.n_parts, orow, lane);
}

// ---------------------------------------------------------------------------------------------
// K/V commit.  One workgroup per (destination 16-token group, KV head).  Pure bit copies through
// integer lanes.  K rows are copied as 16-byte chunks; V is copied likewise for f32 pools and
// transposed through LDS for bf16 pools ([dim][token] within each 16-token group).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void sk_scatter_item(const sk_geom& g, const void* k, const void* v, const sk_scatter& it,
                                                const int head, int32_t* tables_rw, unsigned char* kv_rw, unsigned char* eph_rw)
{
    __shared__ uint16_t vt[16][128 + 2];
    const int tid = threadIdx.x;
    const int d = g.d, elem = g.elem;
    const int rowbytes = d * elem;
    unsigned char* dst = (it.to_eph ? eph_rw : kv_rw) + it.dst_off +
                         (int64_t)head * (it.to_eph ? g.eph_head_stride : g.head_stride);
    const int v_off = it.to_eph ? g.eph_v_off : g.v_off;
    if (it.tbl_index >= 0 && head == 0 && tid == 0) tables_rw[it.tbl_index] = it.block_id;

    const int cpr = rowbytes >> 4;                 // 16-byte chunks per row
    const int total = it.count * cpr;
    for (int cidx = tid; cidx < total; cidx += 256) {
        const int row = cidx / cpr, cc = cidx % cpr;
        const size_t src = ((size_t)(it.src_tok0 + row) * g.Hkv + head) * rowbytes + cc * 16;
        uint4 x = *(const uint4*)((const unsigned char*)k + src);
        *(uint4*)(dst + (size_t)(it.dst_slot0 + row) * rowbytes + cc * 16) = x;
        if (elem == 4) {
            uint4 y = *(const uint4*)((const unsigned char*)v + src);
            *(uint4*)(dst + v_off + (size_t)(it.dst_slot0 + row) * rowbytes + cc * 16) = y;
        }
    }
    if (elem == 2) {
        for (int idx = tid; idx < it.count * d; idx += 256) {
            const int row = idx / d, t = idx % d;
            vt[row][t] = ((const uint16_t*)v)[((size_t)(it.src_tok0 + row) * g.Hkv + head) * d + t];
        }
        __syncthreads();
        // Slots of the 16-token group behind the last committed token are zero-filled, so that a
        // key the attention kernel masks out never multiplies 0 by leftover bits.
        const int first = it.dst_slot0 & 15;            // position inside the 16-token group
        uint16_t* vd = (uint16_t*)(dst + v_off) + (size_t)(it.dst_slot0 >> 4) * d * 16;     // the group's [dim][16 tokens]
        if (first == 0) {
            // from the start of the group: 2 lanes per dimension, 8 tokens (16 bytes) each
            for (int idx = tid; idx < 2 * d; idx += 256) {
                const int t = idx >> 1, half = idx & 1;
                uint32_t wv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int s0 = half * 8 + 2 * j;
                    const uint32_t lo = s0 < it.count ? vt[s0][t] : 0u;
                    const uint32_t hi = s0 + 1 < it.count ? vt[s0 + 1][t] : 0u;
                    wv[j] = lo | (hi << 16);
                }
                *(uint4*)(vd + (size_t)t * 16 + half * 8) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
            }
        } else {
            const int span = 16 - first;                 // slots first..15: tokens, then zeros
            for (int idx = tid; idx < span * d; idx += 256) {
                const int t = idx / span, jj = idx % span;
                vd[(size_t)t * 16 + first + jj] = jj < it.count ? vt[jj][t] : (uint16_t)0;
            }
        }
    }
}

// Items read from a list in the workspace (batched steps) ...
__global__ __launch_bounds__(256) void sk_scatter_kernel(const sk_geom g, const void* k, const void* v,
                                                         const sk_scatter* items, int32_t* tables_rw,
                                                         unsigned char* kv_rw, unsigned char* eph_rw)
{
    const sk_scatter it = items[blockIdx.x / g.Hkv];
    sk_scatter_item(g, k, v, it, blockIdx.x % g.Hkv, tables_rw, kv_rw, eph_rw);
}
// ... or carried in the kernel arguments (single-session calls: no host-to-device copy in front)
__global__ __launch_bounds__(256) void sk_scatter_kernel_args(const sk_geom g, const void* k, const void* v,
                                                              const sk_scatter_list items, int32_t* tables_rw,
                                                              unsigned char* kv_rw, unsigned char* eph_rw)
{
    sk_scatter_item(g, k, v, items.item[blockIdx.x / g.Hkv], blockIdx.x % g.Hkv, tables_rw, kv_rw, eph_rw);
}


// Reads committed K/V back in token order (bit copy).  One thread per element pair is enough:
// this is a verification / export path.
__global__ __launch_bounds__(256) void sk_gather_kernel(const sk_geom g, int32_t tbl_off, int64_t first,
                                                        int64_t count, void* k_out, void* v_out)
{
    const int d = g.d;
    const int64_t total = count * g.Hkv * d;
    for (int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int t = (int)(idx % d);
        const int head = (int)((idx / d) % g.Hkv);
        const int64_t tok = first + idx / ((int64_t)d * g.Hkv);
        const int blk = g.tables[tbl_off + (tok >> g.log2B)];
        const int slot = (int)(tok & (g.B - 1));
        const unsigned char* bb = g.kv + (int64_t)blk * g.blk_stride + (int64_t)head * g.head_stride;
        if (g.elem == 2) {
            ((uint16_t*)k_out)[idx] = ((const uint16_t*)bb)[(size_t)slot * d + t];
            ((uint16_t*)v_out)[idx] = ((const uint16_t*)(bb + g.v_off))[((size_t)(slot >> 4) * d + t) * 16 + (slot & 15)];
        } else {
            ((uint32_t*)k_out)[idx] = ((const uint32_t*)bb)[(size_t)slot * d + t];
            ((uint32_t*)v_out)[idx] = ((const uint32_t*)(bb + g.v_off))[(size_t)slot * d + t];
        }
    }
}

// Copies pool block `src` to block `dst`, all KV heads (the one block a fork or a copy-on-write
// duplicates).  Offsets are formed in 64 bits: a head's blocks lie head_stride bytes apart, which
// exceeds 2 GiB in large pools.
__global__ __launch_bounds__(256) void sk_copy_block_kernel(const sk_geom g, unsigned char* kv_rw, int32_t src, int32_t dst)
{
    const int head = blockIdx.y;
    const int64_t n16 = g.blk_stride >> 4;
    const uint4* s4 = (const uint4*)(kv_rw + (int64_t)head * g.head_stride + (int64_t)src * g.blk_stride);
    uint4* d4 = (uint4*)(kv_rw + (int64_t)head * g.head_stride + (int64_t)dst * g.blk_stride);
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x) d4[i] = s4[i];
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
int sk_launch_scatter(const sk_geom& g, const void* k, const void* v, const sk_scatter* items,
                      int32_t n_items, int32_t* tables_rw, unsigned char* kv_rw, unsigned char* eph_rw,
                      void* stream)
{
    if (n_items <= 0) return 0;
    hipLaunchKernelGGL(sk_scatter_kernel, dim3(n_items * g.Hkv), dim3(256), 0, (hipStream_t)stream,
                       g, k, v, items, tables_rw, kv_rw, eph_rw);
    return (int)hipGetLastError();
}

int sk_launch_scatter_args(const sk_geom& g, const void* k, const void* v, const sk_scatter_list& items,
                           int32_t n_items, int32_t* tables_rw, unsigned char* kv_rw, unsigned char* eph_rw,
                           void* stream)
{
    if (n_items <= 0) return 0;
    hipLaunchKernelGGL(sk_scatter_kernel_args, dim3(n_items * g.Hkv), dim3(256), 0, (hipStream_t)stream,
                       g, k, v, items, tables_rw, kv_rw, eph_rw);
    return (int)hipGetLastError();
}

// The two launchers below take an optional pair of events that the runtime fills with the
// dispatch's own start and end time stamps (the figures a profiler reports for the kernel), for
// sk_pool_set_profiling; without them they are plain launches.
#define SK_LAUNCH(kernel, grid, block)                                                                              \
    do {                                                                                                            \
        if (ev_start) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, (hipEvent_t)ev_start, (hipEvent_t)ev_stop, 0, L); \
        else hipLaunchKernelGGL(kernel, grid, block, 0, st, L);                                                     \
    } while (0)

int sk_launch_attention(const sk_launch& L, int variant, int32_t n_workgroups, void* stream, void* ev_start, void* ev_stop)
{
    if (n_workgroups <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    if (variant != SK_KV_SIMPLE && L.g.d != 128 && !(L.g.d == 64 && variant != SK_KV_MFMA256)) return (int)hipErrorInvalidValue;
    const bool d64 = L.g.d == 64;
    switch (variant) {
    case SK_KV_MFMA256:      SK_LAUNCH((sk_attn_bf16_d128<8, 1, 4>), dim3(n_workgroups), dim3(512)); break;
    case SK_KV_MFMA128:
        if (d64) SK_LAUNCH((sk_attn_bf16_d64<4, 1, 2>), dim3(n_workgroups), dim3(256));
        else SK_LAUNCH((sk_attn_bf16_d128<4, 1, 2>), dim3(n_workgroups), dim3(256));
        break;
    case SK_KV_MFMA64:
        if (d64) SK_LAUNCH((sk_attn_bf16_d64<2, 2, 2>), dim3(n_workgroups), dim3(256));
        else SK_LAUNCH((sk_attn_bf16_d128<2, 2, 2>), dim3(n_workgroups), dim3(256));
        break;
    case SK_KV_MFMA128P:
        if (d64) SK_LAUNCH((sk_attn_bf16_d64<4, 2, 2>), dim3(n_workgroups), dim3(512));
        else SK_LAUNCH((sk_attn_bf16_d128<4, 2, 2>), dim3(n_workgroups), dim3(512));
        break;
    default:
        if (L.g.elem == 2) SK_LAUNCH(sk_attn_simple<true>, dim3(n_workgroups), dim3(256));
        else SK_LAUNCH(sk_attn_simple<false>, dim3(n_workgroups), dim3(256));
    }
    return (int)hipGetLastError();
}

int sk_launch_combine(const sk_launch& L, int32_t n_row_tiles, void* stream, void* ev_start, void* ev_stop)
{
    if (n_row_tiles <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    SK_LAUNCH(sk_combine, dim3(n_row_tiles * (L.rows_per_slot >> 2)), dim3(256));
    return (int)hipGetLastError();
}
#undef SK_LAUNCH

int sk_launch_gather(const sk_geom& g, int32_t tbl_off, int64_t first, int64_t count,
                     void* k_out, void* v_out, void* stream)
{
    if (count <= 0) return 0;
    int64_t total = count * g.Hkv * g.d;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65535) blocks = 65535;
    hipLaunchKernelGGL(sk_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       g, tbl_off, first, count, k_out, v_out);
    return (int)hipGetLastError();
}

int sk_launch_copy_block(const sk_geom& g, unsigned char* kv_rw, int32_t src, int32_t dst, void* stream)
{
    const int64_t n16 = g.blk_stride >> 4;
    int64_t bx = (n16 + 255) / 256;
    if (bx > 64) bx = 64;
    hipLaunchKernelGGL(sk_copy_block_kernel, dim3((unsigned)bx, (unsigned)g.Hkv), dim3(256), 0, (hipStream_t)stream, g, kv_rw, src, dst);
    return (int)hipGetLastError();
}
