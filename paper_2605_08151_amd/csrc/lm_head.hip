// spec_lm_head: logits[r, v] = sum_k hidden[r, k] * W[v, k] for every candidate row (paper, Appendix
// "Target side": every position of the verification candidate is scored so that the accepted length
// can be computed).  bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation, fp32 logits.
//
// Both operands are K-contiguous ("NT" product), which is the MFMA operand order: lane l of a
// 32x32x16 step holds 8 consecutive k of row l%32 (A) or of vocabulary entry l%32 (B), k-group l/32.
#include "common.h"

namespace specv {

// ------------------------------------------------------------------------------------------------
// General tiled kernel: BM x BN output tile per workgroup, 4 waves in a 2 x 2 grid, K staged
// through LDS in slabs of 64 with register prefetch of the next slab.
// ------------------------------------------------------------------------------------------------
constexpr int kBK = 64;
constexpr int kPitch = kBK + 8;     // bf16 elements per LDS row: 144 B, keeps 16 consecutive rows on distinct banks

template <int BM, int BN>
__global__ __launch_bounds__(256) void lm_head_tiled_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W, float* __restrict__ C, int M, int H, int V)
{
    constexpr int WM = BM / 2, WN = BN / 2;           // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;         // 32x32 MFMA tiles per wave
    constexpr int A_LOADS = BM * kBK / 8 / 256;       // 16-byte loads per thread per slab
    constexpr int B_LOADS = BN * kBK / 8 / 256;
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * kPitch];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // vocabulary tiles vary fastest inside a group of row tiles so that W is streamed once
    const int tiles_m = (M + BM - 1) / BM;
    const int bm = blockIdx.x % tiles_m, bn = blockIdx.x / tiles_m;
    const int m0 = bm * BM, n0 = bn * BN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 ra[A_LOADS], rb[B_LOADS];
    const int lrow = tid >> 3, lchunk = tid & 7;       // 8 chunks of 16 B per 64-wide slab row
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            const int row = m0 + lrow + p * 32;
            ra[p] = (row < M) ? *reinterpret_cast<const u32x4*>(A + (size_t)row * H + k0 + lchunk * 8) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int row = n0 + lrow + p * 32;
            rb[p] = (row < V) ? *reinterpret_cast<const u32x4*>(W + (size_t)row * H + k0 + lchunk * 8) : u32x4{0, 0, 0, 0};
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            *reinterpret_cast<u32x4*>(sA + (lrow + p * 32) * kPitch + lchunk * 8) = ra[p];
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            *reinterpret_cast<u32x4*>(sB + (lrow + p * 32) * kPitch + lchunk * 8) = rb[p];
    };

    fetch(0);
    for (int k0 = 0; k0 < H; k0 += kBK) {
        __syncthreads();                 // previous slab fully consumed
        stash();
        __syncthreads();
        if (k0 + kBK < H) fetch(k0 + kBK);
        const int r32 = lane & 31, kg = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(sA + (wm * WM + i * 32 + r32) * kPitch + ks * 16 + kg * 8);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(sB + (wn * WN + j * 32 + r32) * kPitch + ks * 16 + kg * 8);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
    // accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile
    const int col = lane & 31, rhalf = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int gc = n0 + wn * WN + j * 32 + col;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gr = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * rhalf + (r & 3);
                if (gr < M && gc < V) C[(size_t)gr * V + gc] = acc[i][j][r];
            }
        }
}

}  // namespace specv

extern "C" int spec_lm_head(const void* hidden, const void* W, float* logits, int M, int H, int V, void* stream)
{
    using namespace specv;
    if (M < 0 || H <= 0 || V < 0) return fail(SPEC_EINVAL, "spec_lm_head: negative size (M=%d H=%d V=%d)", M, H, V);
    if (M == 0 || V == 0) return SPEC_OK;
    if (!hidden || !W || !logits) return fail(SPEC_EINVAL, "spec_lm_head: NULL pointer argument");
    if (H % 64 != 0) return fail(SPEC_ESHAPE, "spec_lm_head: H=%d must be a multiple of 64", H);
    if (!aligned(hidden, 16) || !aligned(W, 16) || !aligned(logits, 16))
        return fail(SPEC_EINVAL, "spec_lm_head: operands must be 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const uint16_t* a = (const uint16_t*)hidden;
    const uint16_t* w = (const uint16_t*)W;
    if (M <= 64) {
        const long tiles = (long)((M + 63) / 64) * ((V + 127) / 128);
        hipLaunchKernelGGL((lm_head_tiled_kernel<64, 128>), dim3((unsigned)tiles), dim3(256), 0, s, a, w, logits, M, H, V);
    } else {
        const long tiles = (long)((M + 127) / 128) * ((V + 127) / 128);
        hipLaunchKernelGGL((lm_head_tiled_kernel<128, 128>), dim3((unsigned)tiles), dim3(256), 0, s, a, w, logits, M, H, V);
    }
    return check_launch("spec_lm_head");
}
