// spec_lm_head_pack / spec_lm_head_packed: the logits of every candidate row (paper, Appendix "Target side":
// every position of the verification candidate is scored) with the vocabulary matrix stored once, at load
// time, in the order the matrix cores consume it.
//
// Why a second layout.  With W row-major the weight stream of a verify batch touches, per workgroup pass, one
// 64-byte piece of each of 128 rows that lie 2*H bytes apart; measured on MI355X that stream reaches 4.4-4.9
// TB/s, falls further when more rows are open, and the L2-resident hidden rows that every pass re-reads cost
// their transfer time on top.  Stored as below, every wave load is 1 KB of consecutive bytes, the stream runs at
// the rate of a linear read (6.0 TB/s), and because the number of open rows no longer matters a pass can be
// twice as wide, which halves the hidden re-reads.
//
// Packed layout: panels of 16 vocabulary entries; panel p, k-tile t (32 consecutive k), lane l, element j:
//     Wp[((p * (H/32) + t) * 64 + l) * 8 + j] = W[16 p + l % 16][32 t + 8 (l / 16) + j]      (0 for entries >= V)
// i.e. the A operand of v_mfma_f32_16x16x32_bf16 for that tile, lane by lane.  ceil(V/16) panels.
#include "common.h"

namespace specv {

constexpr int kPkSlab = 128;                   // k per hidden slab in LDS
constexpr int kPkHPitch = kPkSlab * 2;         // bytes per hidden row in LDS; 16-byte chunk ch of row r sits at position ch ^ (r & 15)
constexpr int kPkMaxRows = 160;                // rows of hidden per row group (one workgroup's share)

__global__ __launch_bounds__(256) void lm_head_pack_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ Wp,
                                                           int V, int H, size_t n_chunks)
{
    // one 16-byte chunk of the packed matrix per thread and step: consecutive threads write consecutive chunks
    const int ktiles = H / 32;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_chunks; o += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(o & 63);
        const size_t tile = o >> 6;
        const int t = (int)(tile % ktiles);
        const size_t p = tile / ktiles;
        const size_t entry = p * 16 + (lane & 15);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (entry < (size_t)V) v = *reinterpret_cast<const u32x4*>(W + entry * H + t * 32 + (lane >> 4) * 8);
        *reinterpret_cast<u32x4*>(Wp + o * 8) = v;
    }
}

// ------------------------------------------------------------------------------------------------
// One persistent workgroup of NW waves per CU owns a contiguous range of panels and walks it in passes of at most
// NW * TN panels (16 = 256 vocabulary entries by default), cut so that all passes of a workgroup are equally wide
// (whatever V is, every CU streams at the same rate to the end).  Inside a pass wave w takes up to TN consecutive
// panels and all rows of hidden; with NW = 8 two waves share each SIMD and one's MFMAs cover the other's waits
// (10 us of 297 at M = 160):
//   * W goes from HBM straight into registers in operand order through a ring of RS slabs of 128 k, refilled
//     right after the MFMAs that consumed a chunk pair; no W byte touches LDS.
//   * hidden is staged through LDS in 128-k slabs shared by the waves, requested two slabs ahead: loads retire
//     in order, so a younger hidden load must never be what the math waits for.
//   * the next pass's first loads are issued before the finished tile is stored, because stores share the
//     in-order queue with loads.
//   * C^T tiles come out with 4 consecutive vocabulary entries per lane and 16 rows per instruction; they are
//     turned through LDS so that a store instruction writes whole 128-byte lines (all the wave's entries of a
//     row, 128 or 256 bytes).  With one or two row groups they are stored nontemporal (nobody reads them before the
//     next kernel; 263 against 280 us at M = 160); with many groups the L2 absorbs the writes better (1351 against
//     1504 us at M = 1152).
// TM: 16-row tiles of hidden per row group (rows <= 16 TM); RS: slabs in the W register ring (1 in every launch: 2
// measured 5 us slower at M = 160 and equal above); NW: waves (4 or 8); NT: nontemporal stores of the logits;
// TN: panels per wave and pass (2 or 4: a pass is 16 NW TN entries wide);
// STATS: also leave per-block maxima for greedy acceptance.
// ------------------------------------------------------------------------------------------------
template <int TM, int RS, int NW, bool NT, int TN, bool STATS>
__global__ __launch_bounds__(64 * NW, 1) void lm_head_packed_kernel(
    const uint16_t* __restrict__ A_all, const uint16_t* __restrict__ Wp, float* __restrict__ C_all,
    int M_all, int H, int V, int n_panels, int panels_per_wg, bool vec_store, int groups, int rows_per_group,
    float* __restrict__ blk_max, int32_t* __restrict__ blk_arg, int nblk, int passes_per_range)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int kPassPanels = NW * TN;              // panels per workgroup pass
    constexpr int kThreads = 64 * NW;
    constexpr int BM = TM * 16;                       // hidden rows staged in LDS (rows >= M repeat row M-1)
    constexpr int H_LOADS = (BM * 16 + kThreads - 1) / kThreads;   // 16-byte chunks of a hidden slab per thread
    constexpr int kRing = 4 * RS;
    constexpr int kHfAhead = 4;                       // (8 is slower: 340 against 325 us at M = 160)
    constexpr int U = RS % 2 ? 2 * RS : RS;           // slabs per unrolled step: even, so that buffer parities are static
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    // Workgroup -> (row group, panel range).  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2:
    // the row groups of one panel range sit on the same XCD and are dispatched together, so that they stream the
    // same panels at the same time and all but the first read of a panel is an L2 hit.
    const int xcd = blockIdx.x & 7, dealt = blockIdx.x >> 3;
    const int group = dealt % groups, range = (dealt / groups) * 8 + xcd;
    const int M = min(rows_per_group, M_all - group * rows_per_group);              // >= 1 by the host's choice of groups
    const uint16_t* __restrict__ A = A_all + (size_t)group * rows_per_group * H;
    float* __restrict__ C = C_all + (size_t)group * rows_per_group * V;
    const int p_begin = range * panels_per_wg;
    const int p_end = min(n_panels, p_begin + panels_per_wg);
    // STATS: block b = range * passes_per_range + pass of a row holds the maximum of the logits this workgroup computed
    // for the row in that pass and its lowest index (NaN / INT_MAX if the block holds a NaN, -inf / INT_MAX for a
    // block without entries), so that greedy acceptance need not read the logits again.
    auto fill_empty_blocks = [&](int first_pass) {
        const int missing = passes_per_range - first_pass;
        for (int e = tid; e < missing * M; e += kThreads) {
            const int r = e / missing, q = e - r * missing;
            const size_t o = (size_t)(group * rows_per_group + r) * nblk + (size_t)range * passes_per_range + first_pass + q;
            blk_max[o] = -INFINITY;
            blk_arg[o] = 0x7FFFFFFF;
        }
    };
    if (p_begin >= p_end) {
        if (STATS) fill_empty_blocks(0);
        return;
    }
    const int n_own = p_end - p_begin;
    const int npass = (n_own + kPassPanels - 1) / kPassPanels;

    f32x4 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint16_t* wptr[TN];
    u32x4 wreg[TN][kRing], hreg[2][H_LOADS];
    int wave_p0 = 0, wave_np = 0;
    auto open_pass = [&](int pass) {                  // the wave's panels of a pass and their stream pointers
        const int lo = p_begin + (int)((long)pass * n_own / npass);
        const int hi = p_begin + (int)((long)(pass + 1) * n_own / npass);      // 1 <= hi - lo <= kPassPanels
        const int m = hi - lo;
        wave_p0 = lo + wave * m / NW;
        wave_np = lo + (wave + 1) * m / NW - wave_p0; // 0 .. TN; wave_p0 < hi is a panel of the matrix either way
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            // panels past the wave's share re-read its last one (branch-free loop); their results are never stored
            const int p = wave_p0 + max(0, min(tn, wave_np - 1));
            wptr[tn] = Wp + (size_t)p * 16 * H + lane * 8;
        }
    };
    auto fetch_w = [&](int c, int slab) {             // chunk c of the ring <- k-tile 4 * slab + c % 4
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
            wreg[tn][c] = *reinterpret_cast<const u32x4*>(wptr[tn] + (size_t)(slab * 4 + (c & 3)) * 512);
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
            *reinterpret_cast<u32x4*>(buf + row * kPkHPitch + ((ch ^ (row & 15)) << 4)) = hreg[set][p];
        }
    };
    const int nslab = H / kPkSlab;                    // multiple of U
    // first requests of a pass, in the order of the steady state (hidden slab, then W chunks)
    auto open_loads = [&]() {
        fetch_h(0, 0);
#pragma unroll
        for (int c = 0; c < 4; ++c) fetch_w(c, 0);
        fetch_h(1, kPkSlab);                          // slab 1, stashed at the end of slab 0
#pragma unroll
        for (int c = 4; c < kRing; ++c) fetch_w(c, c >> 2);
    };

    unsigned char* buf0 = smem;
    unsigned char* buf1 = smem + BM * kPkHPitch;
    constexpr int kPatchPitch = TN * 64 + 16;         // bytes per row of the wave's store patch: 16 rows x 16 TN entries
    unsigned char* patch = smem + 2 * BM * kPkHPitch + wave * (16 * kPatchPitch);
    // STATS: per row one candidate (value, index) from each wave, merged by the first threads after the next barrier
    float* cand_v = reinterpret_cast<float*>(smem + 2 * BM * kPkHPitch + NW * 16 * kPatchPitch);   // [BM][NW]
    int* cand_i = reinterpret_cast<int*>(cand_v + BM * NW);
    auto merge_candidates = [&](int done_pass) {          // after a barrier that follows the pass's candidate writes
        for (int r = tid; r < M; r += kThreads) {
            float best = -INFINITY;
            int bi = 0x7FFFFFFF;
            bool nan = false;
#pragma unroll
            for (int q = 0; q < NW; ++q) {
                const float v = cand_v[r * NW + q];
                const int vi = cand_i[r * NW + q];
                nan |= (v != v);
                if (v > best || (v == best && vi < bi)) { best = v; bi = vi; }
            }
            const size_t o = (size_t)(group * rows_per_group + r) * nblk + (size_t)range * passes_per_range + done_pass;
            blk_max[o] = nan ? __builtin_nanf("") : best;
            blk_arg[o] = nan ? 0x7FFFFFFF : bi;
        }
    };
    int pass = 0;
    open_pass(pass);
    open_loads();
    for (;;) {
        stash_h(0, buf0);                             // every wave left the previous pass through a barrier
        __syncthreads();
        if (STATS && pass > 0) merge_candidates(pass - 1);   // written before this barrier, rewritten 2 * nslab barriers later
        for (int sR = 0; sR < nslab; sR += U) {
#pragma unroll
            for (int par2 = 0; par2 < U; ++par2) {
                const int s = sR + par2, par = par2 % RS;
                unsigned char* cur = (s & 1) ? buf1 : buf0;
                unsigned char* nxt = (s & 1) ? buf0 : buf1;   // last read in slab s-1, before the barrier that ended it
                // past the end the prefetches wrap to a valid slab (cache hits, results unused): no branch in the loop
                const int kh = min((s + 2) * kPkSlab, H - kPkSlab);
                const int sw = min(s + RS, nslab - 1);
                fetch_h(s & 1, kh);
                // the scheduler must not move the loads: their program order is what the in-order wait counters
                // are derived from, so every step is fenced
                __builtin_amdgcn_sched_barrier(0);
                // The slab is 4 chunks x TM row tiles; each (chunk, row tile) fragment of hidden feeds the TN MFMAs of
                // the wave's panels and is read from LDS kHfAhead fragments before it is used: a short ring instead of
                // a whole chunk of fragments, which leaves the registers to the W ring.
                bf16x8 hfq[kHfAhead];
                auto hfrag = [&](int i) {
                    return *reinterpret_cast<const bf16x8*>(cur + ((i % TM) * 16 + l16) * kPkHPitch + ((((i / TM) * 4 + kg) ^ l16) << 4));
                };
#pragma unroll
                for (int i = 0; i < kHfAhead; ++i) hfq[i] = hfrag(i);
#pragma unroll
                for (int i = 0; i < 4 * TM; ++i) {
                    const int c = i / TM, tm = i % TM;
                    const bf16x8 h = hfq[i % kHfAhead];
                    if (i + kHfAhead < 4 * TM) hfq[i % kHfAhead] = hfrag(i + kHfAhead);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        // wave-uniform: a panel slot the wave does not own costs no MFMA.  The chip is power-limited under
                        // random bf16 operands, so the skipped work raises the clock for everything else (M = 160: 279
                        // against 295 us); with one wave per SIMD the branches cost more than they save (339 us).
                        if (NW == 4 || tn == 0 || tn < wave_np)
                            acc[tn][tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wreg[tn][par * 4 + c]), h,
                                                                              acc[tn][tm], 0, 0, 0);
                    if (tm == TM - 1) {
                        if (c & 1) {                  // the chunk pair just consumed is requested again, RS slabs further
                            fetch_w(par * 4 + c - 1, sw);
                            fetch_w(par * 4 + c, sw);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                stash_h((s & 1) ^ 1, nxt);            // slab s+1, requested one slab ago
                __syncthreads();
            }
        }
        const int st_p0 = wave_p0, st_np = wave_np;
        ++pass;
        const bool more = pass < npass;
        if (more) {
            open_pass(pass);
            open_loads();
            __builtin_amdgcn_sched_barrier(0);
        }
        // acc[tn][tm][i] = C[row 16 tm + l16][entry 16 (st_p0 + tn) + 4 kg + i]
        if (STATS) {
            int cslot = l16 * NW + wave;                  // a running slot: ten addresses kept across the pass would spill
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                float best = -INFINITY;
                int bi = 0x7FFFFFFF;
                bool nan = false;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int e = (st_p0 + tn) * 16 + kg * 4 + i;
                        const float v = acc[tn][tm][i];
                        if (tn < st_np && e < V) {       // ascending e: the first maximum is the lowest index
                            nan |= (v != v);
                            if (v > best) { best = v; bi = e; }
                        }
                    }
#pragma unroll
                for (int sh = 16; sh <= 32; sh <<= 1) {   // the four lanes of a row
                    const float ov = __shfl_xor(best, sh, 64);
                    const int oi = __shfl_xor(bi, sh, 64);
                    nan |= (bool)__shfl_xor((int)nan, sh, 64);
                    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
                }
                if (kg == 0) {
                    cand_v[cslot] = nan ? __builtin_nanf("") : best;
                    cand_i[cslot] = bi;
                }
                cslot += 16 * NW;
                asm volatile("" : "+v"(cslot));
            }
        }
        if (vec_store) {
            // V % 4 == 0.  The tile is turned through the wave's own LDS patch so that one store instruction writes
            // all the wave's entries of a row (whole cache lines), 4 or 8 rows at a time, instead of 64 bytes of each of 16 rows.
            // LDS operations of one wave execute in order, so the patch needs no barrier and no second copy.
            constexpr int kLanesPerRow = TN * 4, kRowsPerStore = 64 / kLanesPerRow;
            const int srow = lane / kLanesPerRow, scol = (lane % kLanesPerRow) * 4;     // this lane's row and entry when storing
            const int col0 = st_p0 * 16 + scol;
            const bool col_ok = scol < st_np * 16 && col0 < V;
            uint32_t off = ((uint32_t)srow * (uint32_t)V + (uint32_t)col0) * 4u;
            const uint32_t row_step = (uint32_t)kRowsPerStore * 4u * (uint32_t)V;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    *reinterpret_cast<f32x4*>(patch + l16 * kPatchPitch + (tn * 16 + kg * 4) * 4) = acc[tn][tm];
                    acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int q = 0; q < 16 / kRowsPerStore; ++q) {
                    const int prow = q * kRowsPerStore + srow, row = tm * 16 + prow;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(patch + prow * kPatchPitch + scol * 4);
                    if (row < M && col_ok) {
                        f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<unsigned char*>(C) + off);
                        if constexpr (NT) __builtin_nontemporal_store(v, dst); else *dst = v;
                    }
                    off += row_step;                  // one running byte offset (M * V * 4 < 2^32 per launch) instead of
                    asm volatile("" : "+v"(off));     // one row address per store kept alive across the whole pass
                }
            }
        } else {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int row = tm * 16 + l16, e = (st_p0 + tn) * 16 + kg * 4;
                    if (row < M && tn < st_np) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (e + i < V) C[(size_t)row * V + e + i] = acc[tn][tm][i];
                    }
                    acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
        }
        if (!more) break;
    }
    if (STATS) {
        __syncthreads();
        merge_candidates(npass - 1);
        fill_empty_blocks(npass);
    }
}

Tunable g_lm_packed_wide{0};      // benchmark hook: 512-entry passes for M <= 160 (0 = automatic, 1 = always, 2 = never)
Tunable g_lm_packed_waves{8};     // benchmark hook: waves per workgroup of the packed kernel (4 or 8)

// panel ranges and panels per range of a launch: ranges is a multiple of 8 (one per XCD and step of the dealing), as many
// as there are CUs per row group; trailing ranges without panels are dropped 8 at a time
static void packed_geometry(int V, int groups, int* ranges, int* per_range)
{
    const int cus = device_cu_count();
    const int n_panels = (V + 15) / 16;
    const int r0 = max(8, cus / groups / 8 * 8);
    *per_range = (n_panels + r0 - 1) / r0;
    *ranges = ((n_panels + *per_range - 1) / *per_range + 7) / 8 * 8;
}

template <int TM, int RS, int NW, bool NT, int TN, bool STATS = false>
static int launch_packed(const uint16_t* a, const uint16_t* wp, float* c, int M, int H, int V, int groups, hipStream_t s,
                         float* blk_max = nullptr, int32_t* blk_arg = nullptr)
{
    constexpr int BM = TM * 16;
    const size_t smem = 2 * (size_t)BM * kPkHPitch + NW * 16 * (TN * 64 + 16) + (STATS ? (size_t)BM * NW * 8 : 0);
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&lm_head_packed_kernel<TM, RS, NW, NT, TN, STATS>), smem, granted, "spec_lm_head_packed")) return rc;
    int ranges, per_range;
    packed_geometry(V, groups, &ranges, &per_range);
    const int ppr = (per_range + NW * TN - 1) / (NW * TN);
    const bool vec_store = (V % 4 == 0);
    hipLaunchKernelGGL((lm_head_packed_kernel<TM, RS, NW, NT, TN, STATS>), dim3(ranges * groups), dim3(64 * NW), smem, s, a, wp, c, M, H, V,
                       (V + 15) / 16, per_range, vec_store, groups, BM, blk_max, blk_arg, ranges * ppr, ppr);
    return SPEC_OK;
}

template <int TM>
static int launch_packed_auto(const uint16_t* a, const uint16_t* wp, float* c, int M, int H, int V, int groups, hipStream_t s,
                              float* blk_max, int32_t* blk_arg)
{
    if (blk_max) {
        if (groups > 2) return launch_packed<TM, 1, 8, false, 2, true>(a, wp, c, M, H, V, groups, s, blk_max, blk_arg);
        return launch_packed<TM, 1, 8, true, 2, true>(a, wp, c, M, H, V, groups, s, blk_max, blk_arg);
    }
    // measured on MI355X at M = 160, V = 151936 inside the whole verify step: 8 waves 287 us, 4 waves 297 us (a 2-slab
    // W ring is 5 us slower with either); at M = 40 both take 218 us; at M = 576 and 1152 8 waves are 5 % ahead
    if (g_lm_packed_waves == 4) return launch_packed<TM, 1, 4, true, 4>(a, wp, c, M, H, V, groups, s);
    if (groups > 2) return launch_packed<TM, 1, 8, false, 2>(a, wp, c, M, H, V, groups, s);
    return launch_packed<TM, 1, 8, true, 2>(a, wp, c, M, H, V, groups, s);
}

}  // namespace specv

extern "C" size_t spec_lm_head_packed_bytes(int V, int H)
{
    if (V <= 0 || H <= 0) return 0;
    return (size_t)((V + 15) / 16) * 16 * (size_t)H * 2;
}

extern "C" int spec_lm_head_pack(const void* W, void* Wp, int V, int H, void* stream)
{
    using namespace specv;
    if (V < 0 || H <= 0) return fail(SPEC_EINVAL, "spec_lm_head_pack: negative size (V=%d H=%d)", V, H);
    if (V == 0) return SPEC_OK;
    if (!W || !Wp) return fail(SPEC_EINVAL, "spec_lm_head_pack: NULL pointer argument");
    if (H % 32 != 0) return fail(SPEC_ESHAPE, "spec_lm_head_pack: H=%d must be a multiple of 32", H);
    if (!aligned(W, 16) || !aligned(Wp, 16)) return fail(SPEC_EINVAL, "spec_lm_head_pack: operands must be 16-byte aligned");
    const size_t n_chunks = spec_lm_head_packed_bytes(V, H) / 16;
    const size_t want = (n_chunks + 255) / 256;
    const unsigned grid = (unsigned)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(lm_head_pack_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t*)W, (uint16_t*)Wp, V, H, n_chunks);
    return check_launch("spec_lm_head_pack");
}

namespace specv {

extern Tunable g_lm_packed_tile;
int lm_head_mfma_dispatch(const uint16_t* a, const uint16_t* wp, float* c, int M, int H, int V, const LmSummary* summary, hipStream_t s);
int lm_head_mfma_blocks(int M, int H, int V);

static int packed_groups(int M) { return (M + kPkMaxRows - 1) / kPkMaxRows; }

// shared by spec_lm_head_packed (blk_max == nullptr) and spec_lm_head_packed_stats
static int lm_head_packed_any(const char* who, const void* hidden, const void* Wp, float* logits, int M, int H, int V,
                              float* blk_max, int32_t* blk_arg, void* stream, const LmSummary* summary = nullptr)
{
    if (M < 0 || H <= 0 || V < 0) return fail(SPEC_EINVAL, "%s: negative size (M=%d H=%d V=%d)", who, M, H, V);
    if (M == 0 || V == 0) return SPEC_OK;
    if (!hidden || !Wp || !logits) return fail(SPEC_EINVAL, "%s: NULL pointer argument", who);
    if (H % (2 * kPkSlab) != 0) return fail(SPEC_ESHAPE, "%s: H=%d must be a multiple of %d", who, H, 2 * kPkSlab);
    if (!aligned(hidden, 16) || !aligned(Wp, 16) || !aligned(logits, 16))
        return fail(SPEC_EINVAL, "%s: operands must be 16-byte aligned", who);
    if ((size_t)V > ((size_t)1 << 32) / (4 * (size_t)(kPkMaxRows + 16)))
        return fail(SPEC_ESHAPE, "%s: V=%d is beyond the 32-bit row offsets of the kernel", who, V);
    hipStream_t s = (hipStream_t)stream;
    const uint16_t* wp = (const uint16_t*)Wp;
    // More than 160 rows: the contraction is bound by the matrix cores, and the large-tile kernel serves it
    const bool large_tile_fits = M > kPkMaxRows && (size_t)V <= ((size_t)1 << 32) / (4 * (size_t)(304 + 16));
    if (summary && !large_tile_fits) return fail(SPEC_ESHAPE, "%s: block summaries need more than %d rows (M=%d, V=%d)", who, kPkMaxRows, M, V);
    if (!blk_max && large_tile_fits && (summary || g_lm_packed_tile != 1)) {
        const int rc = lm_head_mfma_dispatch((const uint16_t*)hidden, wp, logits, M, H, V, summary, s);
        if (rc != SPEC_OK) return rc;
        return check_launch(who);
    }
    // More rows than a workgroup holds: the rows are cut into equal groups of at most 160 (a multiple of 16 each), and
    // the grid is groups x panel ranges.  HBM still sees W once; the other groups read it from the L2.
    int groups = packed_groups(M);
    int tm = ((M + groups - 1) / groups + 15) / 16;                     // 16-row tiles per group, 1 .. 10
    const uint16_t* a = (const uint16_t*)hidden;
    int rc;
    // Groups of at most 80 rows leave registers for 4 panels per wave: a pass is 512 entries wide, which halves the LDS
    // reads per MFMA and quarters the re-reads of hidden, at the price of W crossing L2 -> CU twice as often.
    if (!blk_max && g_lm_packed_wide == 1 && g_lm_packed_waves == 8) {
        groups = (M + kPkMaxRows / 2 - 1) / (kPkMaxRows / 2);
        tm = ((M + groups - 1) / groups + 15) / 16;                     // 1 .. 5
        if (groups > 2) rc = launch_packed<5, 1, 8, false, 4>(a, wp, logits, M, H, V, groups, s);
        else if (tm <= 2) rc = launch_packed<2, 1, 8, true, 4>(a, wp, logits, M, H, V, groups, s);
        else if (tm <= 4) rc = launch_packed<4, 1, 8, true, 4>(a, wp, logits, M, H, V, groups, s);
        else rc = launch_packed<5, 1, 8, true, 4>(a, wp, logits, M, H, V, groups, s);
        if (rc != SPEC_OK) return rc;
        return check_launch(who);
    }
    switch (tm) {
        case 1: case 2: rc = launch_packed_auto<2>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
        case 3: case 4: rc = launch_packed_auto<4>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
        case 5: case 6: rc = launch_packed_auto<6>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
        case 7: rc = launch_packed_auto<7>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
        case 8: rc = launch_packed_auto<8>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
        case 9: rc = launch_packed_auto<9>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
        default: rc = launch_packed_auto<10>(a, wp, logits, M, H, V, groups, s, blk_max, blk_arg); break;
    }
    if (rc != SPEC_OK) return rc;
    return check_launch(who);
}

}  // namespace specv

extern "C" int spec_lm_head_packed(const void* hidden, const void* Wp, float* logits, int M, int H, int V, void* stream)
{
    return specv::lm_head_packed_any("spec_lm_head_packed", hidden, Wp, logits, M, H, V, nullptr, nullptr, stream);
}

/* blocks per row of the statistics spec_lm_head_packed_stats writes; 0 = the packed kernel does not take this shape */
extern "C" int spec_lm_head_packed_stats_blocks(int M, int H, int V)
{
    using namespace specv;
    if (M <= 0 || H <= 0 || V <= 0 || H % (2 * kPkSlab) != 0) return 0;
    int ranges, per_range;
    packed_geometry(V, packed_groups(M), &ranges, &per_range);
    return ranges * ((per_range + 15) / 16);
}

/* blocks per row of the summaries spec_lm_head_packed_summary writes; 0 = that call does not take this shape */
extern "C" int spec_lm_head_packed_summary_blocks(int M, int H, int V)
{
    using namespace specv;
    if (M <= kPkMaxRows || (size_t)V > ((size_t)1 << 32) / (4 * (size_t)(304 + 16))) return 0;
    return lm_head_mfma_blocks(M, H, V);
}

extern "C" int spec_lm_head_packed_summary(const void* hidden, const void* Wp, float* logits, int M, int H, int V,
                                           const float* temperature, const int32_t* qo_indptr, int B,
                                           float* blk_max, float* blk_sum, int32_t* blk_span, void* stream)
{
    using namespace specv;
    if (M > 0 && V > 0 && (!temperature || !qo_indptr || B <= 0 || !blk_max || !blk_sum || !blk_span))
        return fail(SPEC_EINVAL, "spec_lm_head_packed_summary: NULL pointer argument or B=%d", B);
    LmSummary sm{};
    sm.temperature = temperature; sm.qo_indptr = qo_indptr; sm.B = B;
    sm.blk_max = blk_max; sm.blk_sum = blk_sum; sm.blk_span = blk_span;
    return lm_head_packed_any("spec_lm_head_packed_summary", hidden, Wp, logits, M, H, V, nullptr, nullptr, stream, &sm);
}

extern "C" int spec_lm_head_packed_stats(const void* hidden, const void* Wp, float* logits, int M, int H, int V,
                                         float* blk_max, int32_t* blk_arg, void* stream)
{
    using namespace specv;
    if (M > 0 && V > 0 && (!blk_max || !blk_arg)) return fail(SPEC_EINVAL, "spec_lm_head_packed_stats: NULL pointer argument");
    return lm_head_packed_any("spec_lm_head_packed_stats", hidden, Wp, logits, M, H, V, blk_max, blk_arg, stream);
}
