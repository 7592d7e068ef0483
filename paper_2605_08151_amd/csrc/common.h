// Shared host-side helpers of libspecverify: error text, argument checks, device types.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
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

// A launch heuristic that spec_set_tuning may override: one word, written and read atomically.
typedef std::atomic<int> Tunable;

constexpr int kMaxDevices = 64;

// Compute units of the current device (256 if the runtime cannot say), cached per device ordinal.
inline int device_cu_count()
{
    static std::atomic<int> cached[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int cus = cached[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        cached[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}

// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the device's copy of the code) and
// again whenever a launch needs more.  `granted` is the caller's static table, one slot per device ordinal; two
// threads that race here both set the attribute, which is harmless.
typedef std::atomic<size_t> LdsGrantTable[kMaxDevices];
inline int ensure_dynamic_lds(const void* kernel, size_t bytes, LdsGrantTable& granted, const char* who)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    if (granted[dev].load(std::memory_order_acquire) >= bytes) return SPEC_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return fail(SPEC_EHIP, "%s: cannot reserve %zu bytes of LDS", who, bytes);
    granted[dev].store(bytes, std::memory_order_release);
    return SPEC_OK;
}

// fp32 -> bf16, round to nearest even: the conversion instructions of gfx950 (v_cvt_pk_bf16_f32)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ inline uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.0f) & 0xFFFFu; }

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform).
// Written as inline assembly so that the compiler does not order it against later LDS reads by draining
// the whole load queue: the kernel double-buffers and waits with explicit s_waitcnt vmcnt(n) instead.
// M0 (the LDS base of the transfer) is an operand tied to that register: the compiler writes it and knows it is live.
__device__ inline void lds_dma16(const void* g, void* lds_base)
{
    const uint32_t m0v = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_base;
    asm volatile("global_load_lds_dwordx4 %0, off" ::"v"(g), "{m0}"(m0v) : "memory");
}

}  // namespace specv
