// Greedy sampling with a confidence gap on the device (Sec. 3.8: argmax over the logit row without
// copying it to the host; Sec. 3.9.2 / 3.9.4: the gap between the two largest logits), gfx950.
// What it computes is defined in include/sk.h (sk_top2).  Bound by reading the logits once.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include <mutex>
#include "../../include/sk.h"

// First-pass pairs of sk_top2_static: part of the device image, so no call ever allocates it.  In
// host code this name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[SK_TOP2_STATIC_BYTES];

namespace {

struct Top2 { float v1; int32_t i1; float v2; int32_t i2; };

// a before b: larger value, or equal value and lower index
__device__ __forceinline__ bool before(float va, int32_t ia, float vb, int32_t ib)
{
    return va > vb || (va == vb && ia < ib);
}
// Adds entry (v, i) to a thread's running pair (v1, i1, v2, i2).  A thread visits its entries in
// increasing index order, so an entry only goes in front of one it strictly exceeds.  Written on
// scalars with min/max and selects so that it compiles to straight-line code (2 compares, 3
// min/max, 4 selects per logit), which keeps the scan below the time the logits take to arrive
// from HBM.  An entry of -inf never displaces the initial (-inf, INT_MAX); the final kernel
// resolves those.
#define SK_TOP2_PUSH(v, i) do {                                   \
        const float v_ = (v); const int32_t i_ = (i);             \
        const bool g1_ = v_ > v1, g2_ = v_ > v2;                  \
        const int32_t j2_ = g2_ ? i_ : i2;                        \
        i2 = g1_ ? i1 : j2_;                                      \
        i1 = g1_ ? i_ : i1;                                       \
        v2 = fmaxf(v2, fminf(v1, v_));                            \
        v1 = fmaxf(v1, v_);                                       \
    } while (0)

// Merges pair b into pair a (any index order: equal logits go by index).  Selects only.
__device__ __forceinline__ void merge(float& v1, int32_t& i1, float& v2, int32_t& i2,
                                      const float bv1, const int32_t bi1, const float bv2, const int32_t bi2)
{
    const bool af = before(v1, i1, bv1, bi1);
    const float w1v = af ? v1 : bv1, l1v = af ? bv1 : v1, o2v = af ? v2 : bv2;
    const int32_t w1i = af ? i1 : bi1, l1i = af ? bi1 : i1, o2i = af ? i2 : bi2;
    const bool sf = before(o2v, o2i, l1v, l1i);
    v1 = w1v; i1 = w1i;
    v2 = sf ? o2v : l1v; i2 = sf ? o2i : l1i;
}
// reduction over the 256 threads of a workgroup; the result is valid in thread 0
__device__ __forceinline__ void block_reduce(float& v1, int32_t& i1, float& v2, int32_t& i2)
{
    __shared__ float pv1[4], pv2[4];
    __shared__ int32_t pi1[4], pi2[4];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const float bv1 = __shfl_xor(v1, m, 64), bv2 = __shfl_xor(v2, m, 64);
        const int32_t bi1 = __shfl_xor(i1, m, 64), bi2 = __shfl_xor(i2, m, 64);
        merge(v1, i1, v2, i2, bv1, bi1, bv2, bi2);
    }
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { pv1[w] = v1; pi1[w] = i1; pv2[w] = v2; pi2[w] = i2; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 1; k < 4; ++k) merge(v1, i1, v2, i2, pv1[k], pi1[k], pv2[k], pi2[k]);
    }
}

constexpr int kChunk = 8192;      // logits per workgroup of the first pass (32 KiB)

// pass 1: workgroup (chunk c, row r) -> partial[r][c]
__global__ __launch_bounds__(256) void sk_top2_partial(const float* __restrict__ logits, int64_t row_stride, int32_t vocab,
                                                       int32_t n_chunks, Top2* __restrict__ partial)
{
    const int c = blockIdx.x, r = blockIdx.y;
    const float* row = logits + (int64_t)r * row_stride;
    const int begin = c * kChunk;
    const int end = min(begin + kChunk, vocab);
    float v1 = -__builtin_inff(), v2 = -__builtin_inff();
    int32_t i1 = INT_MAX, i2 = INT_MAX;
    // float4 loads over the aligned body (rows are 16-byte aligned, chunk starts are multiples of 4);
    // a full chunk is eight loads per thread, all issued before the first comparison
    const int n4 = (end - begin) >> 2;
    const float4* row4 = (const float4*)(row + begin);
    if (n4 == kChunk / 4) {
        // the logits are read once: non-temporal loads (the plain-read probe gains 8 % by them)
        typedef __attribute__((ext_vector_type(4))) float f32x4;
        f32x4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = __builtin_nontemporal_load((const f32x4*)row4 + threadIdx.x + 256 * u);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = begin + 4 * (threadIdx.x + 256 * u);
            SK_TOP2_PUSH(x[u].x, i); SK_TOP2_PUSH(x[u].y, i + 1); SK_TOP2_PUSH(x[u].z, i + 2); SK_TOP2_PUSH(x[u].w, i + 3);
        }
    } else {
        for (int j = threadIdx.x; j < n4; j += 256) {
            const float4 x = row4[j];
            const int i = begin + 4 * j;
            SK_TOP2_PUSH(x.x, i); SK_TOP2_PUSH(x.y, i + 1); SK_TOP2_PUSH(x.z, i + 2); SK_TOP2_PUSH(x.w, i + 3);
        }
        for (int i = begin + 4 * n4 + threadIdx.x; i < end; i += 256) SK_TOP2_PUSH(row[i], i);
    }
    block_reduce(v1, i1, v2, i2);
    if (threadIdx.x == 0) partial[(int64_t)r * n_chunks + c] = Top2{v1, i1, v2, i2};
}

// pass 2: one workgroup per row merges its partials
__global__ __launch_bounds__(256) void sk_top2_final(const Top2* __restrict__ partial, int32_t n_chunks,
                                                     int32_t* idx1, int32_t* idx2, float* val1, float* val2, float* gap)
{
    const int r = blockIdx.x;
    float v1 = -__builtin_inff(), v2 = -__builtin_inff();
    int32_t i1 = INT_MAX, i2 = INT_MAX;
    for (int c = threadIdx.x; c < n_chunks; c += 256) {
        const Top2 b = partial[(int64_t)r * n_chunks + c];
        merge(v1, i1, v2, i2, b.v1, b.i1, b.v2, b.i2);
    }
    block_reduce(v1, i1, v2, i2);
    if (threadIdx.x == 0) {
        // places still held by the initial pair: every entry that could stand there is -inf, and
        // the lowest index not taken yet is the answer
        if (i1 == INT_MAX) { i1 = 0; i2 = 1; }
        else if (i2 == INT_MAX) i2 = i1 == 0 ? 1 : 0;
        const Top2 t = {v1, i1, v2, i2};
        idx1[r] = t.i1; idx2[r] = t.i2;
        if (val1) val1[r] = t.v1;
        if (val2) val2[r] = t.v2;
        if (gap) gap[r] = t.v1 - t.v2;
    }
}

}  // namespace

extern "C" {

size_t sk_top2_workspace_bytes(int32_t rows, int32_t vocab)
{
    if (rows <= 0 || vocab < 2) return 0;
    const int64_t n_chunks = (int64_t(vocab) + kChunk - 1) / kChunk;
    return size_t(rows) * size_t(n_chunks) * sizeof(Top2);
}

int sk_top2(const float* logits, int32_t rows, int32_t vocab, int64_t row_stride, void* workspace, size_t workspace_bytes,
            int32_t* idx1, int32_t* idx2, float* val1, float* val2, float* gap, void* hip_stream)
{
    if (rows < 0 || vocab < 2 || row_stride < vocab) return SK_E_INVAL;
    if (rows == 0) return SK_OK;
    if (rows > 65535) return SK_E_INVAL;
    if (!logits || !idx1 || !idx2 || !workspace) return SK_E_INVAL;
    if ((uintptr_t)logits % 16 || row_stride % 4 || (uintptr_t)workspace % 16) return SK_E_INVAL;
    if (workspace_bytes < sk_top2_workspace_bytes(rows, vocab)) return SK_E_WORKSPACE;
    const int32_t n_chunks = int32_t((int64_t(vocab) + kChunk - 1) / kChunk);
    hipStream_t st = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(sk_top2_partial, dim3(n_chunks, rows), dim3(256), 0, st, logits, row_stride, vocab, n_chunks, (Top2*)workspace);
    hipLaunchKernelGGL(sk_top2_final, dim3(rows), dim3(256), 0, st, (const Top2*)workspace, n_chunks, idx1, idx2, val1, val2, gap);
    return hipGetLastError() == hipSuccess ? SK_OK : SK_E_HIP;
}

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(void** out)
{
    constexpr int kMaxDevices = 64;
    static void* ptr_of[kMaxDevices];
    static std::mutex mu;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SK_E_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SK_E_HIP;
        ptr_of[dev] = ptr;
    }
    *out = ptr_of[dev];
    return SK_OK;
}

int sk_top2_static(const float* logits, int32_t rows, int32_t vocab, int64_t row_stride,
                   int32_t* idx1, int32_t* idx2, float* val1, float* val2, float* gap, void* hip_stream)
{
    if (rows < 0 || vocab < 2 || row_stride < vocab) return SK_E_INVAL;
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != SK_OK) return rc;
    if (rows == 0) return SK_OK;
    if (rows > 65535) return SK_E_INVAL;
    if (sk_top2_workspace_bytes(rows, vocab) > (size_t)SK_TOP2_STATIC_BYTES) return SK_E_WORKSPACE;
    return sk_top2(logits, rows, vocab, row_stride, ptr, (size_t)SK_TOP2_STATIC_BYTES, idx1, idx2, val1, val2, gap, hip_stream);
}

}  // extern "C"
