// Two measurement probes for benchmarks on gfx950: what a plain streaming read of a buffer takes
// (the ceiling of the query path, which is bound by reading the cache once) and what the matrix
// pipe sustains on bf16 32x32x16 products with operands that toggle like real data (the ceiling of
// the append path).  Declared in include/sk.h; no part of the attention path calls them.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/sk.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Every thread reads 16-byte pieces `stride` apart and folds them into one word; the word is stored
// only if it equals a value that the host picks at random, so the loads cannot be dropped and the
// store practically never happens.  NT: the loads carry the non-temporal cache policy.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
template <bool NT>
__device__ __forceinline__ uint32_t sk_probe_ld(const u32x4* p)
{
    const u32x4 a = NT ? __builtin_nontemporal_load(p) : *p;
    return a.x ^ a.y ^ a.z ^ a.w;
}
template <bool NT>
__global__ __launch_bounds__(256) void sk_probe_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t never, uint32_t* sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {          // eight independent loads in flight per thread
        uint32_t x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = sk_probe_ld<NT>(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= x[u];
    }
    for (; i < n16; i += stride) acc ^= sk_probe_ld<NT>(src + i);
    if (acc == never) sink[0] = acc;
}

// Every wave runs `iters` rounds of eight independent 32x32x16 bf16 products (two operand sets, four
// accumulators) on register operands: taken from `operands` (4 KiB per wave, any bf16 data the caller
// wants the pipe to chew on: how much the operand bits toggle decides the power drawn and with it the
// clock), or, without it, from a hash of the lane index (+-[0.5, 1) with random mantissas).
__global__ __launch_bounds__(512) void sk_probe_mfma_kernel(int iters, uint32_t never, float* sink, const uint4* operands, uint32_t n_vec)
{
    uint32_t h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
    bf16x8 a[2], b[2];
    if (operands) {
        const uint32_t base = (blockIdx.x * 512u + threadIdx.x) * 4u;
        a[0] = __builtin_bit_cast(bf16x8, operands[(base + 0) % n_vec]);
        a[1] = __builtin_bit_cast(bf16x8, operands[(base + 1) % n_vec]);
        b[0] = __builtin_bit_cast(bf16x8, operands[(base + 2) % n_vec]);
        b[1] = __builtin_bit_cast(bf16x8, operands[(base + 3) % n_vec]);
    } else {
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            h = h * 1664525u + 1013904223u;
            const uint16_t ba = (uint16_t)(0x3f00u | ((h >> 9) & 0x80ffu));     // +-[0.5, 1) with a random mantissa
            h = h * 1664525u + 1013904223u;
            const uint16_t bb = (uint16_t)(0x3f00u | ((h >> 9) & 0x80ffu));
            a[k][e] = __builtin_bit_cast(__bf16, ba);
            b[k][e] = __builtin_bit_cast(__bf16, bb);
        }
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[j & 1], acc[j], 0, 0, 0);
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[(j + 1) & 1], acc[j], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    if (__float_as_uint(s) == never) sink[0] = s;
}

}  // namespace

extern "C" {

int sk_probe_read(const void* src, size_t bytes, int32_t n_workgroups, int32_t non_temporal, void* sink, void* hip_stream)
{
    if (!src || !sink || bytes < 16 || (uintptr_t)src % 16 || n_workgroups <= 0 || n_workgroups > (1 << 20)) return SK_E_INVAL;
    if (non_temporal)
        hipLaunchKernelGGL(sk_probe_read_kernel<true>, dim3((unsigned)n_workgroups), dim3(256), 0, (hipStream_t)hip_stream,
                           (const u32x4*)src, bytes / 16, 0x9e3779b9u, (uint32_t*)sink);
    else
        hipLaunchKernelGGL(sk_probe_read_kernel<false>, dim3((unsigned)n_workgroups), dim3(256), 0, (hipStream_t)hip_stream,
                           (const u32x4*)src, bytes / 16, 0x9e3779b9u, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? SK_OK : SK_E_HIP;
}

int sk_probe_mfma(int32_t n_workgroups, int32_t iters, const void* operands, size_t operand_bytes, void* sink,
                  double* flops_out, void* hip_stream)
{
    if (!sink || n_workgroups <= 0 || n_workgroups > (1 << 20) || iters <= 0) return SK_E_INVAL;
    if (operands && ((uintptr_t)operands % 16 || operand_bytes < 64)) return SK_E_INVAL;
    hipLaunchKernelGGL(sk_probe_mfma_kernel, dim3((unsigned)n_workgroups), dim3(512), 0, (hipStream_t)hip_stream,
                       (int)iters, 0x7fc12345u, (float*)sink, (const uint4*)operands, (uint32_t)(operand_bytes / 16));
    if (flops_out) *flops_out = double(n_workgroups) * 8.0 /*waves*/ * double(iters) * 8.0 /*products*/ * (2.0 * 32 * 32 * 16);
    return hipGetLastError() == hipSuccess ? SK_OK : SK_E_HIP;
}

}  // extern "C"
