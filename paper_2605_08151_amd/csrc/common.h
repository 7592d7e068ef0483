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

// Block summaries of the large-tile LM head (lm_head_mfma.hip): what acceptance needs from a row of logits without reading it again.  A
// block is what one wave holds of a row at the end of a pass, at most 64 consecutive vocabulary entries; block index =
// (panel range * passes per range + pass) * 4 + wave, so blocks cover increasing vocabulary ranges; blk_span[2 b],
// blk_span[2 b + 1] = first entry and number of entries of block b (0 for a slot that holds nothing).  Per row and block:
// blk_max = the maximum (NaN if the block holds a NaN) and, for the rows of sampled requests (temperature T > 0),
// blk_sum = sum of 2^((l - blk_max) log2(e)/T), in fp32.  A row's request is found from qo_indptr once per workgroup.
struct LmSummary {
    const float* temperature; // [B]
    const int32_t* qo_indptr; // [B + 1]
    int B;
    float* blk_max;           // [M, blocks]
    float* blk_sum;           // [M, blocks]
    int32_t* blk_span;        // [blocks, 2]
    int blocks, passes_per_range;
};


// Reductions over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48), result in every lane, with the row-swap
// instructions of gfx950 instead of two round trips through the LDS crossbar: v_permlane32_swap exchanges the upper half
// of its first operand with the lower half of the second, v_permlane16_swap the odd rows of the first with the even rows
// of the second; fed with two copies of x they leave (x_lo, x_lo) / (x_hi, x_hi), resp. rows (0,0,2,2) / (1,1,3,3), whose
// element-wise combination is the xor-32, resp. xor-16, step of a butterfly.
// Written as assembly statements: through the compiler's builtins for these two instructions both results of a swap
// came back as the first one (seen in the generated code: max(first, second) had become a plain copy), so that
// "the maximum" was that of the first row alone.  The s_nop covers the wait states the instructions need after a
// vector instruction wrote their operands.
struct SwapPair { float first, second; };

__device__ inline SwapPair swap_halves(float x)          // (x_lo, x_lo), (x_hi, x_hi)
{
    SwapPair p{x, x};
    asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(p.first), "+v"(p.second));
    return p;
}

__device__ inline SwapPair swap_rows(float x)            // rows (0,0,2,2), rows (1,1,3,3)
{
    SwapPair p{x, x};
    asm("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(p.first), "+v"(p.second));
    return p;
}

__device__ inline float four_rows_max(float x)
{
    const SwapPair a = swap_halves(x);
    const SwapPair b = swap_rows(fmaxf(a.first, a.second));
    return fmaxf(b.first, b.second);
}

__device__ inline float four_rows_sum(float x)
{
    const SwapPair a = swap_halves(x);
    const SwapPair b = swap_rows(a.first + a.second);
    return b.first + b.second;
}

// All-reduce over the 16 lanes of a 16-lane row with data-parallel-primitive operand modifiers (rotations by 8, 4, 2, 1
// within the row): every lane ends with the combination of all 16.  (For a sum the order of the additions differs from
// lane to lane; callers that need one answer take it from one lane.)
template <int CTRL>
__device__ inline float dpp_rotated(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

__device__ inline float row16_max(float x)
{
    x = fmaxf(x, dpp_rotated<0x128>(x));              // row_ror:8
    x = fmaxf(x, dpp_rotated<0x124>(x));              // row_ror:4
    x = fmaxf(x, dpp_rotated<0x122>(x));              // row_ror:2
    return fmaxf(x, dpp_rotated<0x121>(x));           // row_ror:1
}

__device__ inline float row16_sum(float x)
{
    x += dpp_rotated<0x128>(x);
    x += dpp_rotated<0x124>(x);
    x += dpp_rotated<0x122>(x);
    return x + dpp_rotated<0x121>(x);
}

}  // namespace specv
