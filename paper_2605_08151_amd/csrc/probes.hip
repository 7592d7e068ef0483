// Measurement probes: what this chip delivers on the two roofs the verification kernels are priced against,
// so that a report can put "fraction of the measured ceiling" beside "fraction of the datasheet peak".
//   spec_probe_read   a linear device read (every byte once, 16 bytes per lane and load, many loads in flight)
//   spec_probe_read_pages  the same bytes as whole 4 KB pages in the order of a page list (the K/V access pattern)
//   spec_probe_mfma   a loop of independent v_mfma_f32_16x16x32_bf16 on register operands, nothing else
// Neither is part of the verification path.
#include "common.h"

namespace specv {

// Every workgroup walks the buffer with a grid stride; 8 independent 16-byte loads per lane and step.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc ^= v[k];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    // data-dependent, practically never true: keeps the loads alive without a store per lane
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = acc.x;
}

// The access pattern of paged K/V: 4 KB pages read whole, in the order of a page list (a random permutation models a
// page pool after long serving).  One page per 256 threads and load, 8 pages in flight per workgroup.
__global__ __launch_bounds__(256) void probe_read_pages_kernel(const u32x4* __restrict__ src, const int32_t* __restrict__ pages,
                                                               int n_pages, uint32_t* __restrict__ sink)
{
    u32x4 acc = {0u, 0u, 0u, 0u};
    const int stride = gridDim.x;
    int i = blockIdx.x;
    for (; i + 7 * stride < n_pages; i += 8 * stride) {
        int pg[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) pg[k] = pages[i + k * stride];
        u32x4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load(src + (size_t)pg[k] * 256 + threadIdx.x);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc ^= v[k];
    }
    for (; i < n_pages; i += stride) acc ^= __builtin_nontemporal_load(src + (size_t)pages[i] * 256 + threadIdx.x);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = acc.x;
}

// NW waves per workgroup, each with 16 independent accumulators; operands rotate among 4 A and 4 B fragments per
// lane so that consecutive instructions see different bit patterns, as in a real product.  constant_operands: every
// fragment holds the same value (the chip draws less power and clocks higher).
__global__ __launch_bounds__(512, 1) void probe_mfma_kernel(int iters, int constant_operands, uint32_t seed, float* __restrict__ sink)
{
    bf16x8 a[4], b[4];
    uint32_t h = seed ^ (threadIdx.x * 0x9E3779B9u) ^ (blockIdx.x * 0x85EBCA6Bu);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        u32x4 wa, wb;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h = h * 1664525u + 1013904223u;
            // two bf16 in [-2, 2) with random mantissas: exponent bits of 1.0, sign and mantissa from the hash
            const uint32_t ra = constant_operands ? 0x3F803F80u : ((h & 0x807F807Fu) | 0x3F803F80u);
            h = h * 1664525u + 1013904223u;
            const uint32_t rb = constant_operands ? 0x3F803F80u : ((h & 0x807F807Fu) | 0x3F803F80u);
            wa[k] = ra;
            wb[k] = rb;
        }
        a[f] = __builtin_bit_cast(bf16x8, wa);
        b[f] = __builtin_bit_cast(bf16x8, wb);
    }
    f32x4 acc[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 16; ++k)
            acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[k & 3], b[(k >> 2) & 3], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) s += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    if (s == 12345.678f) sink[0] = s;                       // keeps the accumulators alive
}

// The same loop with v_mfma_f32_32x32x16_bf16 (8 independent accumulators of 16 registers): the same flops per
// instruction pair, half the operand registers read per flop.
__global__ __launch_bounds__(512, 1) void probe_mfma32_kernel(int iters, int constant_operands, uint32_t seed, float* __restrict__ sink)
{
    bf16x8 a[4], b[4];
    uint32_t h = seed ^ (threadIdx.x * 0x9E3779B9u) ^ (blockIdx.x * 0x85EBCA6Bu);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        u32x4 wa, wb;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h = h * 1664525u + 1013904223u;
            const uint32_t ra = constant_operands ? 0x3F803F80u : ((h & 0x807F807Fu) | 0x3F803F80u);
            h = h * 1664525u + 1013904223u;
            const uint32_t rb = constant_operands ? 0x3F803F80u : ((h & 0x807F807Fu) | 0x3F803F80u);
            wa[k] = ra;
            wb[k] = rb;
        }
        a[f] = __builtin_bit_cast(bf16x8, wa);
        b[f] = __builtin_bit_cast(bf16x8, wb);
    }
    f32x16 acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k & 3], b[(k >> 1) & 3], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[k][e];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace specv

extern "C" int spec_probe_read(const void* src, size_t bytes, void* sink, void* stream)
{
    using namespace specv;
    if (!src || !sink) return fail(SPEC_EINVAL, "spec_probe_read: NULL pointer argument");
    if (!aligned(src, 16) || bytes % 16 != 0) return fail(SPEC_EINVAL, "spec_probe_read: 16-byte aligned buffer and size required");
    if (bytes == 0) return SPEC_OK;
    const int grid = device_cu_count() * 8;
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, bytes / 16, (uint32_t*)sink);
    return check_launch("spec_probe_read");
}

extern "C" int spec_probe_read_pages(const void* src, const int32_t* pages, int n_pages, void* sink, void* stream)
{
    using namespace specv;
    if (!src || !pages || !sink || n_pages < 0) return fail(SPEC_EINVAL, "spec_probe_read_pages: NULL pointer or negative count");
    if (!aligned(src, 16)) return fail(SPEC_EINVAL, "spec_probe_read_pages: 16-byte aligned buffer required");
    if (n_pages == 0) return SPEC_OK;
    const int grid = device_cu_count() * 8;
    hipLaunchKernelGGL(probe_read_pages_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, pages, n_pages, (uint32_t*)sink);
    return check_launch("spec_probe_read_pages");
}

extern "C" double spec_probe_mfma(int iters, int constant_operands, void* sink, void* stream)
{
    using namespace specv;
    if (!sink || iters <= 0) { fail(SPEC_EINVAL, "spec_probe_mfma: NULL sink or iters <= 0"); return -1.0; }
    const int grid = device_cu_count();
    // bit 1 of constant_operands selects the 32x32x16 shape (8 instructions of 32768 flop per iteration instead of 16 of 16384)
    if (constant_operands & 2)
        hipLaunchKernelGGL(probe_mfma32_kernel, dim3(grid), dim3(512), 0, (hipStream_t)stream, iters, constant_operands & 1, 12345u, (float*)sink);
    else
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(512), 0, (hipStream_t)stream, iters, constant_operands & 1, 12345u, (float*)sink);
    if (check_launch("spec_probe_mfma") != SPEC_OK) return -1.0;
    // floating-point operations of the launch: workgroups x 8 waves x iters x 16 instructions x 2*16*16*32
    return (double)grid * 8.0 * (double)iters * 16.0 * 16384.0;
}
