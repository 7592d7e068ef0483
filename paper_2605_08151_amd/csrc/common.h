// Shared host-side helpers of libspecverify: error text, argument checks, device types.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "spec_verify.h"

namespace specv {

// per-thread error text behind spec_last_error_string()
char* error_buffer();

inline int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

inline int check_launch(const char* what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SPEC_EHIP, "%s: %s", what, hipGetErrorString(e));
    return SPEC_OK;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the device's copy of the code) and
// again whenever a launch needs more.  `granted` is the caller's static table, one slot per device ordinal.
constexpr int kMaxDevices = 64;
inline int ensure_dynamic_lds(const void* kernel, size_t bytes, size_t (&granted)[kMaxDevices], const char* who)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    if (granted[dev] >= bytes) return SPEC_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return fail(SPEC_EHIP, "%s: cannot reserve %zu bytes of LDS", who, bytes);
    granted[dev] = bytes;
    return SPEC_OK;
}

// fp32 -> bf16, round to nearest even (inputs here are finite)
__device__ inline uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform).
// Written as inline assembly so that the compiler does not order it against later LDS reads by draining
// the whole load queue: the kernel double-buffers and waits with explicit s_waitcnt vmcnt(n) instead.
__device__ inline void lds_dma16(const void* g, void* lds_base)
{
    const uint32_t m0v = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_base;
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0v) : "memory");
}

}  // namespace specv
