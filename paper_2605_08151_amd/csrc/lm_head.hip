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


// ------------------------------------------------------------------------------------------------
// Weight-streaming kernel for M <= 160 rows (verify batches of a few dozen requests with a handful of drafts each):
// the roof is HBM (W is read once, 2*V*H bytes), so the layout is built around the W stream.
//   * One persistent workgroup per CU owns a contiguous range of vocabulary entries and walks it in
//     passes of 4 waves x 32 entries; the last pass is split evenly over the waves so that all CUs
//     finish together whatever V is.  Only 32 rows of W per wave are open at a time: measured on
//     MI355X, a read stream over 8 KB-strided rows reaches ~5.7 TB/s with 128 rows in flight per CU
//     but only ~4.7 TB/s with 256, against ~6.0 TB/s for a linear read.
//   * Each wave reads ITS vocabulary rows straight from HBM into registers in MFMA operand order
//     (v_mfma_f32_16x16x32_bf16, W on the A side: lane (entry l%16, k-group l/16) takes 16 B at
//     k = 32c + 8*(l/16), so the four lanes of a row cover 64 contiguous bytes per instruction).
//     The registers form a ring of 256 k that is refilled 256 k ahead, two chunks (the two halves of a
//     128-byte line) at a time, right after the MFMAs that consumed them.  No W byte touches LDS.
//     Measured with the math removed, a deeper ring does not stream faster: the rate is set by the
//     number of open rows and by the traffic through the CU's vector L1, not by the bytes in flight.
//   * hidden (all M rows, L2-resident) is staged through LDS in 128-wide k slabs shared by the waves.
//     Its L2 hits are not free: per pass every CU pulls all of hidden (1.25x the W bytes of the pass at
//     M = 160) through the same L1 port, and the time this takes adds to the W stream (measured:
//     +50 us on a 225 us stream), so the pass is as wide as the open-row limit above allows.
//   * C^T tiles come out with 4 consecutive vocabulary entries per lane: 16-byte stores along V.
// ------------------------------------------------------------------------------------------------
constexpr int kSlab = 128;                   // k per hidden slab in LDS
constexpr int kHPitch = kSlab * 2;           // bytes per hidden row in LDS; 16-byte chunk ch of row r sits at position ch ^ (r & 15)
constexpr int kPassCols = 128;               // vocabulary entries per workgroup pass (4 wave columns x 32)

// TM: 16-row tiles of hidden in total; MS: wave rows (the 4*MS waves form a 4 x MS grid: wave column = 32
// vocabulary entries, wave row = TM/MS row tiles; with MS = 2 two waves share every SIMD and hide each other's
// load latency); RS: depth of the W register ring in 128-k slabs; PAIR: refill two chunks at a time.
// STATS: also leave, per row and per pass of the workgroup (block b = workgroup * passes_per_wg + pass), the maximum
// of the block's logits and its lowest index (NaN and INT_MAX if the block holds a NaN; -inf and INT_MAX for a
// block without entries), so that greedy acceptance need not read the logits again.
template <int TM, int MS, int RS, int PAIR, bool STATS>
__global__ __launch_bounds__(256 * MS, 1) void lm_head_skinny_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W, float* __restrict__ C,
    int M, int H, int V, int cols_per_wg, bool vec_store,
    float* __restrict__ blk_max, int32_t* __restrict__ blk_arg, int nblk, int passes_per_wg)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int TN = 2;                             // 16-entry tiles of W per wave
    constexpr int kThreads = 256 * MS;
    constexpr int TMH = (TM + MS - 1) / MS;           // row tiles per wave
    constexpr int BM = TMH * MS * 16;                 // hidden rows staged in LDS (rows >= M repeat row M-1)
    constexpr int H_LOADS = (BM * 16 + kThreads - 1) / kThreads;   // 16-byte chunks of a hidden slab per thread
    constexpr int kRing = 4 * RS;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wcol = wave & 3, mh = wave >> 2;
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int c_begin = blockIdx.x * cols_per_wg;
    const int c_end = min(V, c_begin + cols_per_wg);
    if (c_begin >= c_end) return;
    int pass_index = 0;

    f32x4 acc[TN][TMH];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TMH; ++tm) acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Loads retire in order, so waiting for a young hidden load would drain the whole W ring.  The
    // hidden slab s+2 is therefore requested at the start of slab s and only stashed at the end of slab
    // s+1, when every load older than it is one the math needed anyway.
    const uint16_t* wptr[TN];
    u32x4 wreg[TN][kRing], hreg[2][H_LOADS];
    int wave_c0 = 0, wave_nc = 0;
    auto open_pass = [&](int pass0) {                 // the wave's share of a pass and its W row pointers
        const int pass_cols = min(kPassCols, c_end - pass0);
        const int per_wave = pass_cols == kPassCols ? kPassCols / 4 : (((pass_cols + 3) / 4 + 3) & ~3);
        wave_c0 = pass0 + wcol * per_wave;
        wave_nc = max(0, min(per_wave, pass_cols - wcol * per_wave));
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            // entries past the wave's range re-read its last row (branch-free loop); their results are never stored
            const int e = max(0, min(tn * 16 + l16, wave_nc - 1));
            wptr[tn] = W + (size_t)min(wave_c0 + e, V - 1) * H + kg * 8;
        }
    };
    auto fetch_w = [&](int c, int k0) {               // chunk c of the ring <- k0 + 32*(c%4) .. +32
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) wreg[tn][c] = *reinterpret_cast<const u32x4*>(wptr[tn] + k0 + (c & 3) * 32);
    };
    auto fetch_h = [&](int set, int k0) {
#pragma unroll
        for (int p = 0; p < H_LOADS; ++p) {
            // rows past M read row M-1: every output row depends on its own hidden row only
            const int idx = min(tid + p * kThreads, BM * 16 - 1), row = min(idx >> 4, M - 1), ch = idx & 15;
            hreg[set][p] = *reinterpret_cast<const u32x4*>(A + (size_t)row * H + k0 + ch * 8);
        }
    };
    auto stash_h = [&](int set, unsigned char* buf) {
#pragma unroll
        for (int p = 0; p < H_LOADS; ++p) {
            const int idx = min(tid + p * kThreads, BM * 16 - 1), row = idx >> 4, ch = idx & 15;
            *reinterpret_cast<u32x4*>(buf + row * kHPitch + ((ch ^ (row & 15)) << 4)) = hreg[set][p];
        }
    };
    // First requests of a pass, in the order of the steady state (hidden slab, then W chunks), so that the
    // wait counts the compiler derives for the loop entry are not tighter than those of the back edge.
    auto open_loads = [&]() {
        fetch_h(0, 0);
#pragma unroll
        for (int c = 0; c < 4; ++c) fetch_w(c, 0);
        fetch_h(1, kSlab);                            // slab 1, stashed at the end of slab 0
#pragma unroll
        for (int c = 4; c < kRing; ++c) fetch_w(c, (c >> 2) * kSlab);
    };

    const int nslab = H / kSlab;                      // multiple of RS
    unsigned char* buf0 = smem;
    unsigned char* buf1 = smem + BM * kHPitch;
    const int hrow0 = mh * TMH * 16 + l16;
    int pass0 = c_begin;
    open_pass(pass0);
    open_loads();
    for (;;) {
        stash_h(0, buf0);                             // every wave left the previous pass through a barrier
        __syncthreads();
        for (int sR = 0; sR < nslab; sR += RS) {
#pragma unroll
            for (int par = 0; par < RS; ++par) {
                const int s = sR + par;
                unsigned char* cur = (s & 1) ? buf1 : buf0;
                unsigned char* nxt = (s & 1) ? buf0 : buf1;   // last read in slab s-1, before the barrier that ended it
                // past the end the prefetches wrap to a valid slab (L2 hits, results unused): no branch in the loop
                const int kh = min((s + 2) * kSlab, H - kSlab);
                const int kw = min((s + RS) * kSlab, H - kSlab);
                fetch_h(s & 1, kh);
                // The scheduler must not move the loads: their program order is what the in-order wait
                // counters are derived from (see above), so every step is fenced.
                __builtin_amdgcn_sched_barrier(0);
                bf16x8 hf[2][TMH];
#pragma unroll
                for (int tm = 0; tm < TMH; ++tm)
                    hf[0][tm] = *reinterpret_cast<const bf16x8*>(cur + (hrow0 + tm * 16) * kHPitch + ((kg ^ l16) << 4));
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (c < 3) {
#pragma unroll
                        for (int tm = 0; tm < TMH; ++tm)
                            hf[(c + 1) & 1][tm] = *reinterpret_cast<const bf16x8*>(cur + (hrow0 + tm * 16) * kHPitch + ((((c + 1) * 4 + kg) ^ l16) << 4));
                    }
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const bf16x8 wf = __builtin_bit_cast(bf16x8, wreg[tn][par * 4 + c]);
#pragma unroll
                        for (int tm = 0; tm < TMH; ++tm)
                            acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, hf[c & 1][tm], acc[tn][tm], 0, 0, 0);
                    }
                    if (!PAIR) {
                        fetch_w(par * 4 + c, kw);
                    } else if (c & 1) {
                        fetch_w(par * 4 + c - 1, kw);
                        fetch_w(par * 4 + c, kw);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                stash_h((s & 1) ^ 1, nxt);            // slab s+1, requested one slab ago
                __syncthreads();
            }
        }
        // Stores and loads share the in-order queue: a wave that stored its tile first would have to see
        // those writes land before the first W chunk of the next pass counts as arrived.  So the next
        // pass is opened first and the finished tile is stored behind its loads.
        const int st_c0 = wave_c0, st_nc = wave_nc;
        pass0 += kPassCols;
        const bool more = pass0 < c_end;
        if (more) {
            open_pass(pass0);
            open_loads();
            __builtin_amdgcn_sched_barrier(0);
        }
        // acc[tn][tm][i] = C[row hrow0 + 16tm][entry st_c0 + 16tn + 4kg + i]
        if (STATS) {
            // every wave has left the last slab through a barrier, so the hidden buffers are free: buf1 takes 16
            // candidates per row (4 waves x 4 lane groups), each the best of a lane's 8 entries
            float* cand_v = reinterpret_cast<float*>(buf1);
            int* cand_i = reinterpret_cast<int*>(buf1 + BM * 16 * 4);
#pragma unroll
            for (int tm = 0; tm < TMH; ++tm) {
                float best = -INFINITY;
                int bi = 0x7FFFFFFF;
                bool nan = false;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int e = tn * 16 + kg * 4 + i;
                        const float v = acc[tn][tm][i];
                        if (e < st_nc) {
                            nan |= (v != v);
                            if (v > best) { best = v; bi = st_c0 + e; }
                        }
                    }
                const int slot = (hrow0 + tm * 16) * 16 + wave * 4 + kg;
                cand_v[slot] = nan ? __builtin_nanf("") : best;
                cand_i[slot] = bi;
            }
            __syncthreads();
            for (int r = tid; r < M; r += kThreads) {
                float best = -INFINITY;
                int bi = 0x7FFFFFFF;
                bool nan = false;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const float v = cand_v[r * 16 + q];
                    const int vi = cand_i[r * 16 + q];
                    nan |= (v != v);
                    if (v > best || (v == best && vi < bi)) { best = v; bi = vi; }
                }
                const size_t o = (size_t)r * nblk + (size_t)blockIdx.x * passes_per_wg + pass_index;
                blk_max[o] = nan ? __builtin_nanf("") : best;
                blk_arg[o] = nan ? 0x7FFFFFFF : bi;
            }
            ++pass_index;
            // (the candidates are read before the next barrier, which precedes the next write to buf1)
        }
#pragma unroll
        for (int tm = 0; tm < TMH; ++tm) {
            const int row = hrow0 + tm * 16;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {     // the two 64-byte halves of a row's 128 bytes back to back
                const int e = tn * 16 + kg * 4;
                if (row < M && e < st_nc) {
                    float* dst = C + (size_t)row * V + st_c0 + e;
                    if (vec_store && e + 3 < st_nc) {
                        *reinterpret_cast<f32x4*>(dst) = acc[tn][tm];
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (e + i < st_nc) dst[i] = acc[tn][tm][i];
                    }
                }
                acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        if (!more) break;
    }
    if (STATS) {
        // blocks of passes this workgroup did not have (the last workgroup's range may be shorter)
        const int missing = passes_per_wg - pass_index;
        for (int e = tid; e < missing * M; e += kThreads) {
            const int r = e / missing, q = e - r * missing;
            const size_t o = (size_t)r * nblk + (size_t)blockIdx.x * passes_per_wg + pass_index + q;
            blk_max[o] = -INFINITY;
            blk_arg[o] = 0x7FFFFFFF;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// MFMA-bound kernel for M > 160 rows (large or deeply speculating batches: 576 to ~1200 rows).
//   * (64*TMW) x 256 output tile per workgroup, 4 waves in a 2 x 2 grid, each wave TMW x 4 tiles of
//     v_mfma_f32_32x32x16_bf16 (up to 256 accumulator registers).
//   * K advances in slabs of 32 through a ring of 4 LDS stages filled by direct HBM/L2 -> LDS loads
//     (no staging registers): three slabs are in flight while one is multiplied, one barrier per slab.
//     Rows are 64 B in LDS with the 16-byte chunks XOR-swizzled by row pair, so the 8 lanes that read
//     8 consecutive rows at the same k hit 8 different bank groups.
//     Measured with the math removed: the direct loads deliver ~12.5 TB/s into the CUs of the chip whatever
//     the slab width or ring depth (a 256 x 256 tile needs 16 TB/s at the MFMA peak); staging through
//     registers instead (17.5 TB/s at 128 B per row) gave the same kernel time, because the time is set
//     by the waves waiting for each other's operands at the per-slab barrier, not by either pipe alone.
//   * Workgroup -> tile mapping keeps the row tiles of one vocabulary tile on the same XCD (workgroups
//     are dealt round-robin to the 8 XCDs), so a W slab is fetched into one L2 only.
// ------------------------------------------------------------------------------------------------
constexpr int kBigBN = 256, kBigBK = 32, kBigStages = 4;

// NW = 4: waves in a 2 x 2 grid, TMW x 4 tiles each; NW = 8: 2 x 4 grid, TMW x 2 tiles each, two waves per SIMD
// (<= 256 registers), so that one wave's barrier and LDS waits are covered by the other's MFMAs.
template <int TMW, int NW>
__global__ __launch_bounds__(64 * NW, 1) void lm_head_big_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W, float* __restrict__ C,
    int M, int H, int V, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * TMW;
    constexpr int kRowB = kBigBK * 2;                     // 64 bytes per LDS row
    constexpr int kRows = BM + kBigBN;
    constexpr int kStage = kRows * kRowB;                 // bytes per stage
    constexpr int kGroups = kRows / 16;                   // 16-row groups of a stage
    constexpr int kDma = (kGroups + NW - 1) / NW;         // direct loads per wave per stage; when the groups do not
                                                          // divide evenly the surplus loads repeat the last group
    constexpr int TNW = 16 / NW;                          // 32-wide vocabulary tiles per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / (NW / 2), wn = wave % (NW / 2);
    // blockIdx -> (row tile, vocabulary tile): consecutive workgroups of one XCD walk the row tiles of one vocabulary tile
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int bn = (slot / tiles_m) * 8 + xcd, bm = slot % tiles_m;
    if (bn >= tiles_n) return;
    const int m0 = bm * BM, n0 = bn * kBigBN;

    // direct-load role: instruction j of this wave fills LDS rows 16*(4j + wave) .. +15 of the stage
    // (rows 0..BM-1 = hidden, BM.. = W); lane -> (row = lane/4, position = lane%4),
    // source chunk = position ^ swizzle(row), swizzle = 2*bit1(row) + bit2(row)
    const uint16_t* src[kDma];
#pragma unroll
    for (int j = 0; j < kDma; ++j) {
        const int row = 16 * min(NW * j + wave, kGroups - 1) + (lane >> 2);
        const int ch = (lane & 3) ^ (((row >> 1) & 1) * 2 + ((row >> 2) & 1));
        // rows past M or V read the last valid row: their results are never stored
        src[j] = row < BM ? A + (size_t)min(m0 + row, M - 1) * H + ch * 8
                          : W + (size_t)min(n0 + row - BM, V - 1) * H + ch * 8;
    }
    auto issue = [&](int k0, unsigned char* stage) {
#pragma unroll
        for (int j = 0; j < kDma; ++j) lds_dma16(src[j] + k0, stage + 16 * min(NW * j + wave, kGroups - 1) * kRowB);
    };

    f32x16 acc[TMW][TNW];
#pragma unroll
    for (int i = 0; i < TMW; ++i)
#pragma unroll
        for (int j = 0; j < TNW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int r32 = lane & 31, kg = lane >> 5;
    const int swz = ((r32 >> 1) & 1) * 2 + ((r32 >> 2) & 1);
    const int nslab = H / kBigBK;                         // >= kBigStages (H >= 128)
#pragma unroll
    for (int s = 0; s < kBigStages - 1; ++s) issue(s * kBigBK, smem + s * kStage);
    for (int s = 0; s < nslab; ++s) {
        unsigned char* cur = smem + (s % kBigStages) * kStage;
        // all but the two youngest slabs of this wave's loads have landed (the tail has fewer in flight)
        if (s + 2 < nslab) __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * kDma) & 15) | (((2 * kDma) >> 4) << 14));
        else if (s + 1 < nslab) __builtin_amdgcn_s_waitcnt(0x0F70 | (kDma & 15) | ((kDma >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();                                  // everyone's part of slab s is in LDS, slab s-1 is consumed
        if (s + kBigStages - 1 < nslab) issue((s + kBigStages - 1) * kBigBK, smem + ((s + kBigStages - 1) % kBigStages) * kStage);
        const unsigned char* sa = cur + (wm * (BM / 2) + r32) * kRowB;
        const unsigned char* sb = cur + (BM + wn * (32 * TNW) + r32) * kRowB;
        bf16x8 fa[2][TMW], fb[2][TNW];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int off = ((ks * 2 + kg) ^ swz) << 4;
#pragma unroll
            for (int i = 0; i < TMW; ++i) fa[ks][i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * kRowB + off);
#pragma unroll
            for (int j = 0; j < TNW; ++j) fb[ks][j] = *reinterpret_cast<const bf16x8*>(sb + j * 32 * kRowB + off);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < TMW; ++i)
#pragma unroll
                for (int j = 0; j < TNW; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
    }
    // accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile.  The four
    // vocabulary tiles of a row are stored back to back, so that a row's 512 contiguous bytes reach the
    // memory system together (measured: the epilogue costs ~100 us instead of ~290 at M = 1024).
#pragma unroll
    for (int i = 0; i < TMW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int gr = m0 + wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
#pragma unroll
            for (int j = 0; j < TNW; ++j) {
                const int gc = n0 + wn * (32 * TNW) + j * 32 + r32;
                if (gr < M && gc < V) C[(size_t)gr * V + gc] = acc[i][j][r];
            }
        }
}

template <int TMW, int NW>
static int launch_big(const uint16_t* a, const uint16_t* w, float* c, int M, int H, int V, hipStream_t s)
{
    constexpr int BM = 64 * TMW;
    const size_t smem = (size_t)kBigStages * (BM + kBigBN) * kBigBK * 2;
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&lm_head_big_kernel<TMW, NW>), smem, granted, "spec_lm_head")) return rc;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (V + kBigBN - 1) / kBigBN;
    const long grid = (long)((tiles_n + 7) / 8) * 8 * tiles_m;
    hipLaunchKernelGGL((lm_head_big_kernel<TMW, NW>), dim3((unsigned)grid), dim3(64 * NW), smem, s, a, w, c, M, H, V, tiles_m, tiles_n);
    return SPEC_OK;
}

// ------------------------------------------------------------------------------------------------
// MFMA-bound kernel, second form: operands travel L2 -> registers -> LDS in slabs of 64 k.
//   Plain 16-byte register loads with 128 contiguous bytes per row and instruction deliver ~17.5 TB/s into the
//   CUs against ~12.5 TB/s for the direct loads above (measured with the math removed).
//   * Same tile, XCD-aware tile order and wave grids as above; LDS holds 2 stages of (BM + 256) rows x 128 B,
//     16-byte chunks XOR-swizzled by row (chunk ^ row%8): conflict-free for the 8-lanes-per-row stores and for
//     the 8-rows-per-phase fragment reads.
//   * Two slabs are in flight in registers while one is multiplied: slab s+1 is written to the idle stage in the
//     middle of iteration s and its registers immediately take slab s+3.  One barrier per slab.
//   Measured on MI355X (V = 151936, H = 4096; M = 576 / 1152): direct loads 943 / 1665 us with 4 waves and
//   957 / 1683 us with 8; this kernel 948 / 1670 us with 4 waves and 900 / 1592 us with 8, the default.  With the
//   chip power-limited to ~1.5 PFLOP/s under random bf16 data the MFMAs alone take ~930 us at M = 1152.
// ------------------------------------------------------------------------------------------------
constexpr int kB2BK = 64;

template <int TMW, int NW>
__global__ __launch_bounds__(64 * NW, 1) void lm_head_big2_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ W, float* __restrict__ C,
    int M, int H, int V, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * TMW;
    constexpr int kRowB = kB2BK * 2;                      // 128 bytes per LDS row
    constexpr int kRows = BM + kBigBN;
    constexpr int kStage = kRows * kRowB;
    constexpr int kGroups = kRows / 8;                    // 8-row groups of a slab
    constexpr int kLd = (kGroups + NW - 1) / NW;          // loads per wave per slab; surplus loads repeat the last group
    constexpr int TNW = 16 / NW;                          // 32-wide vocabulary tiles per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / (NW / 2), wn = wave % (NW / 2);
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int bn = (slot / tiles_m) * 8 + xcd, bm = slot % tiles_m;
    if (bn >= tiles_n) return;
    const int m0 = bm * BM, n0 = bn * kBigBN;

    // loader role: instruction j of this wave moves 8 rows of the slab (rows 0..BM-1 = hidden, BM.. = W);
    // lane -> (row = lane/8, 16-byte chunk = lane%8)
    const int lr = lane >> 3, lc = lane & 7;
    const uint16_t* src[kLd];
    int dst[kLd];
#pragma unroll
    for (int j = 0; j < kLd; ++j) {
        const int row = 8 * min(NW * j + wave, kGroups - 1) + lr;
        // rows past M or V read the last valid row: their results are never stored
        src[j] = row < BM ? A + (size_t)min(m0 + row, M - 1) * H + lc * 8
                          : W + (size_t)min(n0 + row - BM, V - 1) * H + lc * 8;
        dst[j] = row * kRowB + ((lc ^ lr) << 4);
    }
    u32x4 stg[2][kLd];
    auto fetch = [&](int set, int k0) {
#pragma unroll
        for (int j = 0; j < kLd; ++j) stg[set][j] = *reinterpret_cast<const u32x4*>(src[j] + k0);
    };
    auto stash = [&](int set, unsigned char* stage) {
#pragma unroll
        for (int j = 0; j < kLd; ++j) *reinterpret_cast<u32x4*>(stage + dst[j]) = stg[set][j];
    };

    f32x16 acc[TMW][TNW];
#pragma unroll
    for (int i = 0; i < TMW; ++i)
#pragma unroll
        for (int j = 0; j < TNW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int r32 = lane & 31, kg = lane >> 5;
    const int sa_off = (wm * (BM / 2) + r32) * kRowB, sb_off = (BM + wn * (32 * TNW) + r32) * kRowB;
    const int nslab = H / kB2BK;                          // >= 2 and even (H % 128 == 0)
    unsigned char* st0 = smem;
    unsigned char* st1 = smem + kStage;
    fetch(0, 0);
    fetch(1, kB2BK);
    stash(0, st0);
    fetch(0, min(2 * kB2BK, H - kB2BK));
    __syncthreads();
    for (int s2 = 0; s2 < nslab; s2 += 2) {
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            const int s = s2 + par;
            const unsigned char* cur = par ? st1 : st0;
            unsigned char* oth = par ? st0 : st1;         // held slab s-1, consumed before the last barrier
            bf16x8 fa[2][TMW], fb[2][TNW];
            auto read_frags = [&](int buf, int ks) {
                const int off = ((ks * 2 + kg) ^ (r32 & 7)) << 4;
#pragma unroll
                for (int i = 0; i < TMW; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(cur + sa_off + i * 32 * kRowB + off);
#pragma unroll
                for (int j = 0; j < TNW; ++j) fb[buf][j] = *reinterpret_cast<const bf16x8*>(cur + sb_off + j * 32 * kRowB + off);
            };
            read_frags(0, 0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < 3) read_frags((ks + 1) & 1, ks + 1);
#pragma unroll
                for (int i = 0; i < TMW; ++i)
#pragma unroll
                    for (int j = 0; j < TNW; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
                if (ks == 1) {
                    // slab s+1 (requested two iterations ago) goes to the idle stage; its registers take slab s+3
                    // (past the end: a valid slab again, never stashed)
                    if (s + 1 < nslab) stash(par ^ 1, oth);
                    fetch(par ^ 1, min((s + 3) * kB2BK, H - kB2BK));
                }
            }
            __syncthreads();                              // slab s is consumed, slab s+1 is in LDS
        }
    }
#pragma unroll
    for (int i = 0; i < TMW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int gr = m0 + wm * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
#pragma unroll
            for (int j = 0; j < TNW; ++j) {
                const int gc = n0 + wn * (32 * TNW) + j * 32 + r32;
                if (gr < M && gc < V) C[(size_t)gr * V + gc] = acc[i][j][r];
            }
        }
}

template <int TMW, int NW>
static int launch_big2(const uint16_t* a, const uint16_t* w, float* c, int M, int H, int V, hipStream_t s)
{
    constexpr int BM = 64 * TMW;
    const size_t smem = 2 * (size_t)(BM + kBigBN) * kB2BK * 2;
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&lm_head_big2_kernel<TMW, NW>), smem, granted, "spec_lm_head")) return rc;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (V + kBigBN - 1) / kBigBN;
    const long grid = (long)((tiles_n + 7) / 8) * 8 * tiles_m;
    hipLaunchKernelGGL((lm_head_big2_kernel<TMW, NW>), dim3((unsigned)grid), dim3(64 * NW), smem, s, a, w, c, M, H, V, tiles_m, tiles_n);
    return SPEC_OK;
}

Tunable g_lm_kernel_waves{8};  // benchmark hook: waves per workgroup of the MFMA-bound kernel (4 or 8)
Tunable g_lm_kernel{0};   // benchmark hook: 0 = automatic, 1 = weight-streaming, 2 = MFMA-bound with direct loads, 3 = plain tiled,
                       // 8 = MFMA-bound with register staging (the automatic choice for M > 160),
                       // 4 = weight-streaming with 8 waves (4 x 2) and a 2-slab ring, 5/6/7 = 4 waves with
                       // 4-slab ring / 4-slab ring + paired refills / 2-slab ring + paired refills (the default)

// vocabulary entries per workgroup and the grid of the weight-streaming kernel
static void skinny_geometry(int V, int* cols, int* grid)
{
    const int cus = device_cu_count();
    int c = ((V + cus - 1) / cus + 3) & ~3;
    if (c < 64) c = 64;
    *cols = c;
    *grid = (V + c - 1) / c;
}

template <int TM, int MS, int RS, int PAIR = 0, bool STATS = false>
static int launch_skinny(const uint16_t* a, const uint16_t* w, float* c, int M, int H, int V, hipStream_t s,
                         float* blk_max = nullptr, int32_t* blk_arg = nullptr)
{
    constexpr int BM = (TM + MS - 1) / MS * MS * 16;
    const size_t smem = 2 * (size_t)BM * kHPitch;
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&lm_head_skinny_kernel<TM, MS, RS, PAIR, STATS>), smem, granted, "spec_lm_head")) return rc;
    int cols, grid;
    skinny_geometry(V, &cols, &grid);
    const int ppw = (cols + kPassCols - 1) / kPassCols;
    const bool vec_store = (V % 4 == 0);
    hipLaunchKernelGGL((lm_head_skinny_kernel<TM, MS, RS, PAIR, STATS>), dim3(grid), dim3(256 * MS), smem, s, a, w, c, M, H, V, cols,
                       vec_store, blk_max, blk_arg, grid * ppw, ppw);
    return SPEC_OK;
}

template <int TM>
static int launch_skinny_auto(const uint16_t* a, const uint16_t* w, float* c, int M, int H, int V, hipStream_t s)
{
    // measured on MI355X at M = 160, V = 151936 inside the whole verify step: 4 waves with a 2-slab ring and
    // paired refills ~347 us, with a 4-slab ring and single refills ~363 us, 8 waves (two wave rows re-reading
    // the same W rows) with a 2-slab ring ~470 us
    if (g_lm_kernel == 4) return launch_skinny<TM, 2, 2>(a, w, c, M, H, V, s);
    if (g_lm_kernel == 5) return launch_skinny<TM, 1, 4>(a, w, c, M, H, V, s);
    if (g_lm_kernel == 6) return launch_skinny<TM, 1, 4, 1>(a, w, c, M, H, V, s);
    if (g_lm_kernel == 7) return launch_skinny<TM, 1, 2, 1>(a, w, c, M, H, V, s);
    return launch_skinny<TM, 1, 2, 1>(a, w, c, M, H, V, s);
}

static bool skinny_applies(int M, int H)
{
    const int force = g_lm_kernel;
    // the register ring holds 2 slabs of 128 k (4 in the variants 5 and 6): H must be a whole number of rings
    const int ring = (force == 5 || force == 6) ? 4 : 2;
    return (force == 0 || force == 1 || force >= 4) && force != 8 && M <= 160 && H % (ring * kSlab) == 0;
}

}  // namespace specv

/* blocks per row of the statistics spec_lm_head_stats writes; 0 = this shape is not served by the fused kernel */
extern "C" int spec_lm_head_stats_blocks(int M, int H, int V)
{
    using namespace specv;
    if (M <= 0 || H <= 0 || V <= 0 || !skinny_applies(M, H) || g_lm_kernel >= 4) return 0;
    int cols, grid;
    skinny_geometry(V, &cols, &grid);
    return grid * ((cols + kPassCols - 1) / kPassCols);
}

extern "C" int spec_lm_head_stats(const void* hidden, const void* W, float* logits, int M, int H, int V,
                                  float* blk_max, int32_t* blk_arg, void* stream)
{
    using namespace specv;
    const int blocks = spec_lm_head_stats_blocks(M, H, V);
    if (blocks == 0) return spec_lm_head(hidden, W, logits, M, H, V, stream);
    if (!hidden || !W || !logits || !blk_max || !blk_arg) return fail(SPEC_EINVAL, "spec_lm_head_stats: NULL pointer argument");
    if (!aligned(hidden, 16) || !aligned(W, 16) || !aligned(logits, 16))
        return fail(SPEC_EINVAL, "spec_lm_head_stats: operands must be 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const uint16_t* a = (const uint16_t*)hidden;
    const uint16_t* w = (const uint16_t*)W;
    int rc;
    if (M <= 32) rc = launch_skinny<2, 1, 2, 1, true>(a, w, logits, M, H, V, s, blk_max, blk_arg);
    else if (M <= 64) rc = launch_skinny<4, 1, 2, 1, true>(a, w, logits, M, H, V, s, blk_max, blk_arg);
    else if (M <= 96) rc = launch_skinny<6, 1, 2, 1, true>(a, w, logits, M, H, V, s, blk_max, blk_arg);
    else if (M <= 128) rc = launch_skinny<8, 1, 2, 1, true>(a, w, logits, M, H, V, s, blk_max, blk_arg);
    else rc = launch_skinny<10, 1, 2, 1, true>(a, w, logits, M, H, V, s, blk_max, blk_arg);
    if (rc != SPEC_OK) return rc;
    return check_launch("spec_lm_head_stats");
}

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
    const int force = g_lm_kernel;
    if (skinny_applies(M, H)) {
        int rc;
        if (M <= 32) rc = launch_skinny_auto<2>(a, w, logits, M, H, V, s);
        else if (M <= 64) rc = launch_skinny_auto<4>(a, w, logits, M, H, V, s);
        else if (M <= 96) rc = launch_skinny_auto<6>(a, w, logits, M, H, V, s);
        else if (M <= 128) rc = launch_skinny_auto<8>(a, w, logits, M, H, V, s);
        else rc = launch_skinny_auto<10>(a, w, logits, M, H, V, s);
        if (rc != SPEC_OK) return rc;
    } else if ((force == 8 || (force == 0 && M > 160)) && H % (2 * kB2BK) == 0) {
        const int waste192 = (M + 191) / 192 * 192 - M, waste256 = (M + 255) / 256 * 256 - M;
        int rc;
        if (g_lm_kernel_waves == 4) rc = waste192 <= waste256 ? launch_big2<3, 4>(a, w, logits, M, H, V, s) : launch_big2<4, 4>(a, w, logits, M, H, V, s);
        else rc = waste192 <= waste256 ? launch_big2<3, 8>(a, w, logits, M, H, V, s) : launch_big2<4, 8>(a, w, logits, M, H, V, s);
        if (rc != SPEC_OK) return rc;
    } else if ((force == 2 || (force == 0 && M > 160)) && H % kBigBK == 0 && H >= kBigBK * kBigStages) {   // H % 128 != 0 ends here
        // row tiles of 192 or 256: whichever wastes fewer padded rows
        const int waste192 = (M + 191) / 192 * 192 - M, waste256 = (M + 255) / 256 * 256 - M;
        int rc;
        if (g_lm_kernel_waves == 4) rc = waste192 <= waste256 ? launch_big<3, 4>(a, w, logits, M, H, V, s) : launch_big<4, 4>(a, w, logits, M, H, V, s);
        else rc = waste192 <= waste256 ? launch_big<3, 8>(a, w, logits, M, H, V, s) : launch_big<4, 8>(a, w, logits, M, H, V, s);
        if (rc != SPEC_OK) return rc;
    } else if (M <= 64) {
        const long tiles = (long)((M + 63) / 64) * ((V + 127) / 128);
        hipLaunchKernelGGL((lm_head_tiled_kernel<64, 128>), dim3((unsigned)tiles), dim3(256), 0, s, a, w, logits, M, H, V);
    } else {
        const long tiles = (long)((M + 127) / 128) * ((V + 127) / 128);
        hipLaunchKernelGGL((lm_head_tiled_kernel<128, 128>), dim3((unsigned)tiles), dim3(256), 0, s, a, w, logits, M, H, V);
    }
    return check_launch("spec_lm_head");
}
