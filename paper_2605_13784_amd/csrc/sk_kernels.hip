// HIP kernels for gfx950 (CDNA4, wave64): K/V commit (scatter), attention over a paged
// session cache (bf16 MFMA kernel and an fp32 FMA kernel), cross-split log-sum-exp combine,
// gather.  What they compute is defined in include/sk.h; the data layout in sk_internal.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "sk_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define SK_NEG_INF (-__builtin_inff())
#define SK_LN2 0.6931471805599453f

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float sk_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float sk_log2(float x) { return __builtin_amdgcn_logf(x); }

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
    if (eph_part) { w.kv_begin = 0; w.kv_end = 0; }
    else {
        w.kv_begin = split * P.chunk;
        int e = w.kv_begin + P.chunk;
        w.kv_end = e < kv_vis ? e : kv_vis;
    }
    w.part = (P.n_splits == 1) ? -1 : (tile * P.n_splits + split) * Hkv + head;
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
    int32_t pos_shift;           // absolute position = token index + pos_shift
};

__device__ __forceinline__ sk_seg sk_make_seg(const sk_launch& P, const sk_work& w, int s)
{
    sk_seg g;
    if (s == 0) {
        g.base = P.g.kv + (int64_t)w.kv_head * P.g.head_stride;
        g.table = P.g.tables + w.tbl_off; g.blk_stride = P.g.blk_stride;
        g.v_off = P.g.v_off; g.B = P.g.B; g.log2B = P.g.log2B;
        g.begin = w.kv_begin; g.end = w.kv_end; g.pos_shift = 0;
    } else {
        g.base = P.g.eph + (int64_t)w.kv_head * P.g.eph_head_stride;
        g.table = P.g.eph_ident + (s == 1 ? w.eph_blk[0] : w.eph_blk[1]); g.blk_stride = P.g.eph_blk_stride;
        g.v_off = P.g.eph_v_off; g.B = 16; g.log2B = 4;
        g.begin = 0; g.end = (s == 1 ? w.eph_cnt[0] : w.eph_cnt[1]); g.pos_shift = (s == 1 ? w.eph_pos0[0] : w.eph_pos0[1]);
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

// ---------------------------------------------------------------------------------------------
// bf16 MFMA attention kernel, head_dim 128.
//
// Workgroup = 4 waves, arranged as NRG row groups x NPH key phases (NRG * NPH = 4): a row group
// owns 32 query rows, a phase owns every NPH-th key tile.
//
// Keys move HBM -> LDS with direct-to-LDS loads (global_load_lds_dwordx4), never through
// registers, into a ring of four 32-key tiles (K 8 KiB + V^T 8 KiB each).  One iteration
// consumes two tiles (64 keys: both by every wave when NPH = 1, one per phase when NPH = 2)
// while the other two are in flight, 32 KiB per workgroup and 64 KiB per CU, which is what
// covers the HBM latency.  A direct-to-LDS load writes lane i's 16 bytes at
// base + 16 i, so the bank swizzle is applied to the *source* address each lane picks:
//   K   : LDS row rho holds global 16-byte chunk (c ^ (rho & 15)) at chunk position c,
//   V^T : LDS row dd of a 16-key group holds the two 8-key halves swapped when bit 3 of dd is set.
// The loads of one tile are issued by all four waves (4 instructions each); a wave waits on its
// own vmcnt and a workgroup barrier publishes the tile.  Nothing else in the loop is a vector
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
// and sum need one cross-lane exchange (lane ^ 32) and P feeds the second contraction straight
// from registers.  Key row rho of the first product is loaded from key tau(rho) (bits 2 and 3
// swapped) so that the 8 P values a lane hands to one PV instruction belong to 8 consecutive
// keys, which are one 16-byte read of V^T.
// Softmax runs in the log2 domain in fp32; the running maximum is only raised when a tile
// exceeds it by more than SK_RESCALE_SLACK, which keeps exp2 arguments <= the slack and makes
// accumulator rescaling rare; the result is the same up to rounding.
// ---------------------------------------------------------------------------------------------
#define SK_TILE 32                 // keys per tile
#define SK_TILE_BYTES 16384        // K 8 KiB | V^T 8 KiB
#ifndef SK_NST
#define SK_NST 4                   // ring depth in tiles
#endif
#ifndef SK_WGS_PER_CU
#define SK_WGS_PER_CU 2            // workgroups per CU the register budget is sized for
#endif
#define SK_RESCALE_SLACK 8.0f

template <int N> struct sk_int { static constexpr int value = N; };
typedef __attribute__((address_space(3))) void* sk_lds_ptr;
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

// One direct-to-LDS load of 16 bytes per lane: lane i's data lands at lds_addr + 16 i.
// Written as inline assembly so that the compiler's automatic wait insertion does not drain the
// tiles in flight before every LDS read; the waits are placed by hand (SK_WAIT_VMCNT).
__device__ __forceinline__ void sk_dma16(const void* base, unsigned lane_off, unsigned lds_addr)
{   // address = base (scalar registers) + lane_off (one VGPR, unsigned)
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}

// Pool blocks holding the two 16-key groups of the tile that starts at key t0 (scalar loads).
// Groups past the end of the segment fall back to its last group.
struct sk_tile_blocks { int32_t blk[2]; };
__device__ __forceinline__ sk_tile_blocks sk_lookup_tile(const sk_seg& g, int t0, int last_group)
{
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    sk_tile_blocks b;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int tg = t0 + 16 * j;
        tg = tg < last_group ? tg : last_group;
        b.blk[j] = ((const_i32_ptr)(uintptr_t)g.table)[tg >> g.log2B];
    }
    return b;
}

// Issues the four direct-to-LDS loads with which this wave contributes to one tile.  The part of
// every source address that depends on the lane is the same for all tiles of a segment (koff,
// voff); the rest is uniform and stays in scalar registers.
//   K   : this wave fills LDS rows 16 j + 4 wave .. + 3 of group j; lane -> (row rr, chunk position),
//         source chunk (position ^ rr):        koff = rr * 256 + ((lane & 15) ^ rr) * 16
//   V^T : this wave fills dims 32 wave .. + 31 of group j; lane -> (dim dd, half position),
//         source half (position ^ bit 3 of dd): voff = dd * 2B + (half ^ ((dd >> 3) & 1)) * 16
__device__ __forceinline__ void sk_issue_tile(const sk_seg& g, int t0, int last_group, const sk_tile_blocks& tb,
                                              unsigned stage, int wave, unsigned koff, unsigned voff)
{
#pragma unroll
    for (int j = 0; j < 2; ++j) {            // j = 16-key group of the tile
        int tg = t0 + 16 * j;
        tg = tg < last_group ? tg : last_group;
        const unsigned char* bb = g.base + (int64_t)tb.blk[j] * g.blk_stride;
        const int slot0 = tg & (g.B - 1);
        sk_dma16(bb + (size_t)slot0 * 256, koff, stage + (j * 4 + wave) * 1024);
        sk_dma16(bb + g.v_off + slot0 * 2, voff, stage + 8192 + (j * 4 + wave) * 1024);
    }
}

#ifdef SK_EXPERIMENT              // development builds: P.pad bit 0 = no arithmetic, bit 1 = no loads
#define SK_EXP_LOADS if (!(P.pad & 2))
#else
#define SK_EXP_LOADS
#endif

template <int NPH>
__global__ __launch_bounds__(256, SK_WGS_PER_CU) void sk_attn_bf16_d128(const sk_launch P)
{
    constexpr int NRG = 4 / NPH;
    constexpr int TPI = 2;                   // tiles per iteration (64 keys)
    constexpr int TPW = TPI / NPH;           // tiles per wave per iteration
    constexpr int NSS = SK_NST / TPI;        // ring depth in iterations
    constexpr int LP = 4 * TPI;              // loads per wave per iteration
    static_assert(SK_NST % TPI == 0 && NSS >= 2, "ring depth");
    __shared__ __attribute__((aligned(16))) unsigned char lds[SK_NST * SK_TILE_BYTES];

    sk_work w;
    if (!sk_decode_work(P, blockIdx.x, w)) return;

#ifdef SK_EXPERIMENT
    if (P.pad & 4) return;                     // launch overhead only
#endif
    const unsigned lds_base = (unsigned)(uintptr_t)(sk_lds_ptr)lds;   // LDS byte address of the ring
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // in a scalar register
    const int rg = wave % NRG, ph = wave / NRG;
    const int r = lane & 31, kg = lane >> 5;
    const int log2G = P.g.log2G, G = P.g.G;
    const int row_in_tile = rg * 32 + r;
    const int tok_local = row_in_tile >> log2G;
    const int hq = w.kv_head * G + (row_in_tile & (G - 1));
    const bool row_valid = tok_local < w.n_tok;
    const int tok_per_rg = 32 >> log2G;
    // positions of the first and last valid token of this wave (wave-uniform)
    const int wave_tok_first = rg * tok_per_rg;
    int wave_tok_last = wave_tok_first + tok_per_rg - 1;
    if (wave_tok_last > w.n_tok - 1) wave_tok_last = w.n_tok - 1;
    const bool wave_has_rows = wave_tok_first < w.n_tok;
    const bool causal = w.pos0 < SK_NO_CAUSAL;
    const int p_row = causal ? w.pos0 + (row_valid ? tok_local : wave_tok_last) : 0x7fffffff;
    const int p_wave_min = causal ? w.pos0 + wave_tok_first : 0x7fffffff;
    const int p_wave_max = causal ? w.pos0 + wave_tok_last : 0x7fffffff;

    // Q^T operand: lane (row r, k-group kg) keeps Q[row][16*ks + 8*kg .. +7] for ks = 0..7
    bf16x8 qreg[8];
    {
        uint4 z = make_uint4(0, 0, 0, 0);
        const uint4* qp = (const uint4*)((const unsigned char*)P.q +
                          ((size_t)(w.q_tok0 + (row_valid ? tok_local : 0)) * P.g.Hq + hq) * 256);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 x = qp[ks * 2 + kg];                 // rows past the tile re-read row 0, then zeroed
            if (!row_valid) x = z;
            qreg[ks] = __builtin_bit_cast(bf16x8, x);
        }
    }

    f32x16 oacc[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[mt][v] = 0.f;
    float m_ref = SK_NEG_INF, l_run = 0.f;
    const float c_scale = P.g.scale_log2e;
    // key tau(rho): swap bits 2 and 3 of the S^T row index
    const int tau = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);

    // lane-dependent LDS addresses of the MFMA operands inside a tile (the XOR swizzles make them
    // irregular in ks, so they are kept in registers; tile and ring-half offsets are immediates)
    const unsigned char* kptr[8];
    const unsigned char* vptr[4];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kptr[ks] = lds + ph * TPW * SK_TILE_BYTES + tau * 256 + (((ks * 2 + kg) ^ (tau & 15)) << 4);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int dd = mt * 32 + r;
        vptr[mt] = lds + ph * TPW * SK_TILE_BYTES + 8192 + dd * 32 + ((kg ^ ((dd >> 3) & 1)) << 4);
    }
    static_assert(NSS == 2, "the iteration body is unrolled over the two ring halves");

#pragma unroll 1
    for (int s = 0; s < 3; ++s) {
        sk_seg g = sk_make_seg(P, w, s);
        if (g.end <= g.begin) continue;
        const int ntiles = (g.end - g.begin + SK_TILE - 1) / SK_TILE;
        const int niter = (ntiles + TPI - 1) / TPI;
        const int last_group = (g.end - 1) & ~15;
        const int seg_last_pos = g.end - 1 + g.pos_shift;
        const int lim_wave_min = p_wave_min < seg_last_pos ? p_wave_min : seg_last_pos;
        const int lim_wave_max = p_wave_max < seg_last_pos ? p_wave_max : seg_last_pos;
        const int lim_row = p_row < seg_last_pos ? p_row : seg_last_pos;

        // lane-dependent parts of the DMA source addresses for this segment
        const unsigned koff = (unsigned)((wave * 4 + (lane >> 4)) * 256 + (((lane & 15) ^ (wave * 4 + (lane >> 4))) << 4));
        const int vdd = wave * 32 + (lane >> 1);
        const unsigned voff = (unsigned)(vdd * (2 * g.B) + ((((lane & 1) ^ ((vdd >> 3) & 1))) << 4));

        sk_lds_barrier();                      // ring free (previous segment fully consumed)
        // prologue: iteration 0
        if (niter > 0) {
#pragma unroll
            for (int p = 0; p < TPI; ++p) {
                const int t0 = g.begin + p * SK_TILE;
                const sk_tile_blocks tb = sk_lookup_tile(g, t0, last_group);
                SK_EXP_LOADS sk_issue_tile(g, t0, last_group, tb, lds_base + p * SK_TILE_BYTES, wave, koff, voff);
            }
        }
        // block ids of the next refill are looked up one iteration ahead of their use
        sk_tile_blocks nb[TPI];
#pragma unroll
        for (int p = 0; p < TPI; ++p)
            nb[p] = sk_lookup_tile(g, g.begin + (TPI + p) * SK_TILE, last_group);
        // The query operand must have arrived before the loop (a wait for it placed by the
        // compiler inside the loop would drain the ring on every iteration).
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : : "v"(qreg[ks]));

        // One iteration (64 keys).  STAGE is the ring half it reads (a compile-time constant, so LDS
        // offsets fold into the instructions' immediate fields); the other half is being refilled.
        auto iteration = [&](const int it, auto stage_const) {
            constexpr int STAGE = decltype(stage_const)::value;
            SK_WAIT_VMCNT(0);                  // this wave's loads of iteration `it` have landed
            sk_lds_barrier();
            // refill the half consumed in iteration it-1 with iteration it+1 (its block ids were
            // looked up during the previous iteration), then look up the next ones
            if (it + 1 < niter) {
#pragma unroll
                for (int p = 0; p < TPI; ++p)
                    SK_EXP_LOADS sk_issue_tile(g, g.begin + ((it + 1) * TPI + p) * SK_TILE, last_group, nb[p],
                                               lds_base + ((1 - STAGE) * TPI + p) * SK_TILE_BYTES, wave, koff, voff);
                if (it + 2 < niter) {
#pragma unroll
                    for (int p = 0; p < TPI; ++p)
                        nb[p] = sk_lookup_tile(g, g.begin + ((it + 2) * TPI + p) * SK_TILE, last_group);
                }
            }
            // this wave's TPW consecutive tiles of the iteration
            const int tile0 = it * TPI + ph * TPW;
            const int pos_first = g.begin + tile0 * SK_TILE + g.pos_shift;
            bool active = wave_has_rows && tile0 < ntiles && pos_first <= lim_wave_max;
#ifdef SK_EXPERIMENT
            if (P.pad & 1) active = false;      // stream only: no arithmetic
#endif
            if (!active) return;
            const bool need_mask = pos_first + TPW * SK_TILE - 1 > lim_wave_min;
            constexpr int SOFF = STAGE * TPI * SK_TILE_BYTES;       // byte offset of this ring half

            // S^T = K Q^T, TPW independent accumulator chains
            f32x16 sacc[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[t][v] = 0.f;
            {
                uint4 ka[TPW][8];
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
                        ka[t][ks] = *(const uint4*)(kptr[ks] + SOFF + t * SK_TILE_BYTES);
                __builtin_amdgcn_s_setprio(2);     // the wave feeding the matrix pipe goes first
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
                        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[t][ks]), qreg[ks], sacc[t], 0, 0, 0);
                __builtin_amdgcn_s_setprio(0);
                // all LDS reads first, then the MFMAs back to back (two independent chains)
                __builtin_amdgcn_sched_group_barrier(0x100, 8 * TPW, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 8 * TPW, 0);
            }
            // V^T operands are requested now, so that their LDS latency hides behind the softmax
            uint4 va[TPW][2][4];
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt)
                        va[t][q][mt] = *(const uint4*)(vptr[mt] + SOFF + t * SK_TILE_BYTES + q * 4096);
            // mask (only tiles that cross a limit) and row maximum, on the raw scores; the softmax
            // scale is applied inside the exponent below (one FMA per score)
            float mt_ = SK_NEG_INF;
            if (need_mask) {
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int pos = pos_first + t * SK_TILE + 16 * (v >> 3) + 8 * kg + (v & 7);
                        const float x = (pos <= lim_row) ? sacc[t][v] : SK_NEG_INF;
                        sacc[t][v] = x;
                        mt_ = fmaxf(mt_, x);
                    }
            } else {
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mt_ = fmaxf(mt_, sacc[t][v]);
            }
            mt_ = fmaxf(mt_, __shfl_xor(mt_, 32, 64)) * c_scale;      // log2 units (c_scale > 0)
            const bool raise = mt_ > m_ref + SK_RESCALE_SLACK;
            if (__any(raise)) {
                const float alpha = raise ? sk_exp2(m_ref - mt_) : 1.0f;
                l_run *= alpha;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[mt][v] *= alpha;
                m_ref = raise ? mt_ : m_ref;
            }
            const float neg_m = (m_ref == SK_NEG_INF) ? 0.f : -m_ref;
            // P = exp2(s * scale - m), row sums, O^T += V^T P^T
            bf16x8 pb[TPW][2];
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float p0 = sk_exp2(fmaf(sacc[t][v], c_scale, neg_m)), p1 = sk_exp2(fmaf(sacc[t][8 + v], c_scale, neg_m));
                    l_run += p0 + p1;
                    pb[t][0][v] = (__bf16)p0;
                    pb[t][1][v] = (__bf16)p1;
                }
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt)
                        oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[t][q][mt]), pb[t][q], oacc[mt], 0, 0, 0);
        };
        for (int it = 0; it < niter; it += 2) {
            iteration(it, sk_int<0>{});
            if (it + 1 < niter) iteration(it + 1, sk_int<1>{});
        }
    }

    float l_tot = l_run + __shfl_xor(l_run, 32, 64);

    if (NPH > 1) {
        // merge the key phases of each row group through LDS: [value index][lane], value 64 = m, 65 = l
        __syncthreads();
        float* xch = (float*)&lds[0] + rg * (66 * 64);
        if (ph == 1) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) xch[(mt * 16 + v) * 64 + lane] = oacc[mt][v];
            xch[64 * 64 + lane] = m_ref;
            xch[65 * 64 + lane] = l_tot;
        }
        __syncthreads();
        if (ph == 1) return;
        const float m1 = xch[64 * 64 + lane], l1 = xch[65 * 64 + lane];
        const float M = fmaxf(m_ref, m1);
        const float a0 = (m_ref == SK_NEG_INF) ? 0.f : sk_exp2(m_ref - M);
        const float a1 = (m1 == SK_NEG_INF) ? 0.f : sk_exp2(m1 - M);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[mt][v] = oacc[mt][v] * a0 + xch[(mt * 16 + v) * 64 + lane] * a1;
        l_tot = l_tot * a0 + l1 * a1;
        m_ref = M;
    }

    // ---- epilogue: rows go out through LDS so that every store instruction writes whole rows ----
    // A lane holds 4-float pieces of ONE row (its accumulators are O^T); written as they are, a store
    // instruction would touch 64 different 128-byte lines.  Each wave transposes its 32 x 128 tile in
    // its own 16 KiB of the (now idle) ring, XOR-swizzled by row so both directions are conflict-free.
    if (NPH == 1) __syncthreads();                    // every wave is done reading key tiles
#ifdef SK_EXPERIMENT
    if (P.pad & 8) return;                     // no output
#endif
    const bool direct = w.part < 0;
    const float inv = direct ? 1.0f / l_tot : 1.0f;
    float* tr = (float*)lds + (NPH == 1 ? wave : rg * 2) * 4096;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int c4 = mt * 8 + q4 * 2 + kg;
            *(float4*)(tr + r * 128 + ((c4 ^ r) & 31) * 4) =
                make_float4(oacc[mt][q4 * 4 + 0] * inv, oacc[mt][q4 * 4 + 1] * inv, oacc[mt][q4 * 4 + 2] * inv, oacc[mt][q4 * 4 + 3] * inv);
        }
    const size_t orow_lane = ((size_t)(w.q_tok0 + tok_local) * P.g.Hq + hq);
    if (row_valid && kg == 0) {
        if (direct) { if (P.lse) P.lse[orow_lane] = (m_ref + sk_log2(l_tot)) * SK_LN2; }
        else *(float2*)(P.part_ml + ((size_t)w.part * P.rows_per_slot + row_in_tile) * 2) = make_float2(m_ref, l_tot);
    }
    const int c4 = lane & 31;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int row = it * 2 + (lane >> 5);
        const float4 val = *(const float4*)(tr + row * 128 + ((c4 ^ row) & 31) * 4);
        const int rit = rg * 32 + row;                 // row inside the tile
        const int tok2 = rit >> log2G;
        if (tok2 >= w.n_tok) continue;
        if (direct) {
            const size_t orow = ((size_t)(w.q_tok0 + tok2) * P.g.Hq + w.kv_head * G + (rit & (G - 1)));
            if (P.out_dtype == 0) *(float4*)((float*)P.out + orow * 128 + c4 * 4) = val;
            else {
                const uint32_t lo = f32_to_bf16_bits(val.x) | ((uint32_t)f32_to_bf16_bits(val.y) << 16);
                const uint32_t hi = f32_to_bf16_bits(val.z) | ((uint32_t)f32_to_bf16_bits(val.w) << 16);
                *(uint2*)((uint16_t*)P.out + orow * 128 + c4 * 4) = make_uint2(lo, hi);
            }
        } else {
            *(float4*)(P.part_o + ((size_t)w.part * P.rows_per_slot + rit) * 128 + c4 * 4) = val;
        }
    }
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
                        vx = bf16_bits_to_f32(((const uint16_t*)(bb + g.v_off))[(size_t)t * g.B + slot]);
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
                x = (t0 + tt + g.pos_shift <= lim) ? x : SK_NEG_INF;
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
        if (c == 0) { P.part_ml[prow * 2] = m_run; P.part_ml[prow * 2 + 1] = l_run; }
    }
}

// ---------------------------------------------------------------------------------------------
// Cross-split combine: one wave per output row.
//   M = max_s m_s ; L = sum_s l_s 2^(m_s - M) ; O = sum_s O_s 2^(m_s - M) / L ; LSE = (M + log2 L) ln 2
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
    const int G = P.g.G, d = P.g.d;
    if (row >= cb.n_tok * G) return;
    const int tok_local = row / G;
    const int hq = cb.kv_head * G + row % G;
    const size_t prow0 = (size_t)cb.part0 * P.rows_per_slot + row;
    const size_t pstride = (size_t)cb.part_stride * P.rows_per_slot;
    // Lane s owns (m, l) of part base+s; rows are read in batches of eight parts, the next
    // batch requested before the current one is used, so one memory latency covers the kernel.
    const int per_lane = d >> 6;     // 1 (d=64) or 2 (d=128)
    const float* obase = P.part_o + prow0 * d + per_lane * lane;
    const size_t ostride = pstride * d;
    float M = SK_NEG_INF;
    if (cb.n_parts > 64) {           // rare: the maximum needs its own pass
        for (int s = lane; s < cb.n_parts; s += 64) M = fmaxf(M, P.part_ml[(prow0 + s * pstride) * 2]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    }
    float L = 0.f, a0 = 0.f, a1 = 0.f;
    for (int base = 0; base < cb.n_parts; base += 64) {
        const int cnt = cb.n_parts - base < 64 ? cb.n_parts - base : 64;
        float2 ml = make_float2(SK_NEG_INF, 0.f);
        if (lane < cnt) ml = *(const float2*)(P.part_ml + (prow0 + (base + lane) * pstride) * 2);
        float2 x[8], y[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = make_float2(0.f, 0.f);
            if (j < cnt) {
                const float* op = obase + (size_t)(base + j) * ostride;
                if (per_lane == 2) x[j] = *(const float2*)op; else x[j].x = *op;
            }
        }
        if (cb.n_parts <= 64) {
            M = ml.x;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
        }
        const float wgt = (ml.x == SK_NEG_INF) ? 0.f : sk_exp2(ml.x - M);
        L += ml.y * wgt;
        for (int j0 = 0; j0 < cnt; j0 += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {           // request the next batch
                y[j] = make_float2(0.f, 0.f);
                if (j0 + 8 + j < cnt) {
                    const float* op = obase + (size_t)(base + j0 + 8 + j) * ostride;
                    if (per_lane == 2) y[j] = *(const float2*)op; else y[j].x = *op;
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float wj = __shfl(wgt, j0 + j, 64);    // 0 for parts past the end
                a0 += x[j].x * wj; a1 += x[j].y * wj;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = y[j];
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) L += __shfl_xor(L, off, 64);
    const float inv = 1.0f / L;
    const size_t orow = ((size_t)(cb.q_tok0 + tok_local) * P.g.Hq + hq);
    if (P.out_dtype == 0) {
        float* o = (float*)P.out + orow * d;
        if (per_lane == 2) *(float2*)(o + 2 * lane) = make_float2(a0 * inv, a1 * inv);
        else o[lane] = a0 * inv;
    } else {
        uint16_t* o = (uint16_t*)P.out + orow * d;
        if (per_lane == 2) *(uint32_t*)(o + 2 * lane) = f32_to_bf16_bits(a0 * inv) | ((uint32_t)f32_to_bf16_bits(a1 * inv) << 16);
        else o[lane] = f32_to_bf16_bits(a0 * inv);
    }
    if (P.lse && lane == 0) P.lse[orow] = (M + sk_log2(L)) * SK_LN2;
}

// ---------------------------------------------------------------------------------------------
// K/V commit.  One workgroup per (destination 16-token group, KV head).  Pure bit copies through
// integer lanes.  K rows are copied as 16-byte chunks; V is copied likewise for f32 pools and
// transposed through LDS for bf16 pools ([dim][token]).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sk_scatter_kernel(const sk_geom g, const void* k, const void* v,
                                                         const sk_scatter* items, int32_t* tables_rw,
                                                         unsigned char* kv_rw, unsigned char* eph_rw)
{
    __shared__ uint16_t vt[16][128 + 2];
    const int item = blockIdx.x / g.Hkv, head = blockIdx.x % g.Hkv;
    const sk_scatter it = items[item];
    const int tid = threadIdx.x;
    const int d = g.d, elem = g.elem;
    const int rowbytes = d * elem;
    const int Bd = it.to_eph ? 16 : g.B;
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
        uint16_t* vd = (uint16_t*)(dst + v_off) + (it.dst_slot0 - first);
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
                *(uint4*)(vd + (size_t)t * Bd + half * 8) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
            }
        } else {
            const int span = 16 - first;                 // slots first..15: tokens, then zeros
            for (int idx = tid; idx < span * d; idx += 256) {
                const int t = idx / span, jj = idx % span;
                vd[(size_t)t * Bd + first + jj] = jj < it.count ? vt[jj][t] : (uint16_t)0;
            }
        }
    }
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
            ((uint16_t*)v_out)[idx] = ((const uint16_t*)(bb + g.v_off))[(size_t)t * g.B + slot];
        } else {
            ((uint32_t*)k_out)[idx] = ((const uint32_t*)bb)[(size_t)slot * d + t];
            ((uint32_t*)v_out)[idx] = ((const uint32_t*)(bb + g.v_off))[(size_t)slot * d + t];
        }
    }
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

int sk_launch_attention(const sk_launch& L, int variant, int32_t n_workgroups, void* stream)
{
    if (n_workgroups <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    switch (variant) {
    case SK_KV_MFMA128: hipLaunchKernelGGL(sk_attn_bf16_d128<1>, dim3(n_workgroups), dim3(256), 0, st, L); break;
    case SK_KV_MFMA64:  hipLaunchKernelGGL(sk_attn_bf16_d128<2>, dim3(n_workgroups), dim3(256), 0, st, L); break;
    default:
        if (L.g.elem == 2) hipLaunchKernelGGL(sk_attn_simple<true>, dim3(n_workgroups), dim3(256), 0, st, L);
        else hipLaunchKernelGGL(sk_attn_simple<false>, dim3(n_workgroups), dim3(256), 0, st, L);
    }
    return (int)hipGetLastError();
}

int sk_launch_combine(const sk_launch& L, int32_t n_row_tiles, void* stream)
{
    if (n_row_tiles <= 0) return 0;
    hipLaunchKernelGGL(sk_combine, dim3(n_row_tiles * (L.rows_per_slot >> 2)), dim3(256), 0, (hipStream_t)stream, L);
    return (int)hipGetLastError();
}

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
