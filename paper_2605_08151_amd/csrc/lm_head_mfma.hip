// spec_lm_head_packed for batches of more than 160 rows: the MFMA-bound kernel (paper, Appendix "Target side": every
// position of every verification candidate is scored; the hybrid ordinary-parallel batch has ~1200 positions).
//
// With hundreds of rows the LM head is a dense contraction bound by the matrix cores, and what starves them is operand
// traffic: L2 -> CU bytes per flop fall with the workgroup's tile area, LDS bytes per flop with the vocabulary width a wave
// covers.  So: ONE wave per SIMD with the whole register file (512 registers), each wave holding a tile of
// 16 TM rows x 64 vocabulary entries in the accumulation registers (TM <= 16: the workgroup tile is up to 256 x 256),
//   * W goes from L2/HBM straight into MFMA operand registers (the packed layout is the A operand of
//     v_mfma_f32_16x16x32_bf16 lane by lane), through a ring of 4 slabs of 64 k, each chunk requested again right
//     after the MFMAs that consumed it: no W byte touches LDS;
//   * hidden goes from L2 into LDS by direct global->LDS loads (no staging registers), 4 slabs of 64 k deep, and
//     a fragment read from LDS feeds 4 MFMAs (one per panel of the wave);
//   * a wave is its own latency hiding: everything it needs is requested 2.5 to 4 slabs (2-4 us) ahead.
// The batch is cut into row groups of whole 16-row tiles, nearly equal and at most 256 rows each; the grid is groups x panel ranges, the groups of a
// range run on the same XCD at the same time and share that range's panels through the XCD's L2, so HBM sees W once.
// Per output element the products are added in the same order as in the other LM-head kernels (k ascending, one
// fp32 accumulator), so the logits are bit-identical to theirs.
#include "common.h"

#include <type_traits>

namespace specv {

constexpr int kMfSlab = 64;                    // k per slab
constexpr int kMfPitch = kMfSlab * 2;          // bytes per hidden row in LDS; 16-byte chunk c of row r sits at c ^ ((r >> 1) & 7)
constexpr int kMfWaves = 4;
constexpr int kMfTN = 4;                       // panels (16 vocabulary entries each) per wave
constexpr int kMfPassPanels = kMfWaves * kMfTN;
constexpr int kMfRing = 4;                     // slabs in flight: hidden slabs in LDS = W slabs in registers
constexpr int kMfPatchPitch = kMfTN * 64 + 16; // bytes per row of a wave's store patch

// (SUMMARY instantiations also leave the block summaries described at LmSummary)
template <int TM, bool NT, bool SUMMARY>
__global__ __launch_bounds__(64 * kMfWaves, 1) void lm_head_mfma_kernel(
    const uint16_t* __restrict__ A_all, const uint16_t* __restrict__ Wp, float* __restrict__ C_all,
    int M_all, int H, int V, int n_panels, int panels_per_wg, bool vec_store, int groups, int tiles_lo, int groups_hi,
    LmSummary sm)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int RW = kMfRing;
    constexpr int SR = (TM * 16 + 31) / 32 * 32;      // rows staged per slab: 8 per direct load, the same count for every wave
    constexpr int QN = SR / 32;                       // direct loads per wave and slab
    constexpr int kSlabBytes = SR * kMfPitch;
    constexpr int kHfAhead = 4;                       // hidden fragments read from LDS ahead of their MFMAs
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    // Workgroup -> (row group, panel range): workgroups are dealt round-robin to the 8 XCDs, so the groups of one range
    // are given consecutive slots of the same XCD.
    const int xcd = blockIdx.x & 7, dealt = blockIdx.x >> 3;
    const int group = dealt % groups, range = (dealt / groups) * 8 + xcd;
    // Row groups are whole 16-row tiles: the first groups_hi groups have tiles_lo + 1 = TM of them, the others tiles_lo.
    // A group with TM - 1 tiles issues no MFMA for the missing one: on this chip an MFMA that computes nothing still costs
    // the power that sets the clock for all the others.
    const int row0 = 16 * (group * tiles_lo + min(group, groups_hi));
    const bool full_tm = group < groups_hi || tiles_lo == TM;
    const int M = min(16 * (tiles_lo + (group < groups_hi ? 1 : 0)), M_all - row0);    // >= 1 by the host's choice of groups
    const unsigned char* __restrict__ A = reinterpret_cast<const unsigned char*>(A_all + (size_t)row0 * H);
    float* __restrict__ C = C_all + (size_t)row0 * V;
    const int p_begin = range * panels_per_wg;
    const int p_end = min(n_panels, p_begin + panels_per_wg);
    if (p_begin >= p_end) {
        if constexpr (SUMMARY) {                      // a range past the matrix: its block slots hold nothing
            if (group == 0)
                for (int b = tid; b < sm.passes_per_range * kMfWaves; b += 64 * kMfWaves) {
                    sm.blk_span[2 * (range * sm.passes_per_range * kMfWaves + b)] = 0;
                    sm.blk_span[2 * (range * sm.passes_per_range * kMfWaves + b) + 1] = 0;
                }
        }
        return;
    }
    const int n_own = p_end - p_begin;
    const int npass = (n_own + kMfPassPanels - 1) / kMfPassPanels;
    const int nslab = H / kMfSlab;                    // a multiple of 4 (host check)

    unsigned char* hbuf = smem;                                        // kMfRing slabs
    unsigned char* patch = smem + kMfRing * kSlabBytes + wave * (16 * kMfPatchPitch);
    float* row_scale = reinterpret_cast<float*>(smem + kMfRing * kSlabBytes + kMfWaves * (16 * kMfPatchPitch));   // [TM * 16], SUMMARY only
    if constexpr (SUMMARY) {
        // log2(e) / T of each row's request (0: greedy, or no such row); read again only after many barriers
        for (int r = tid; r < TM * 16; r += 64 * kMfWaves) {
            float sc = 0.0f;
            if (r < M) {
                int lo = 0, hi = sm.B - 1;                // largest i with qo_indptr[i] <= row
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (sm.qo_indptr[mid] <= row0 + r) lo = mid; else hi = mid - 1;
                }
                const float T = sm.temperature[lo];
                sc = T > 0.0f ? (float)(1.4426950408889634 / (double)T) : 0.0f;
            }
            row_scale[r] = sc;
        }
    }

    // ---- hidden: byte offset (from A) of the 16 bytes this lane moves in direct load q of a slab, k0 = 0.
    // Load q of wave w fills LDS rows 8 (QN w + q) .. +7: lane l writes position l % 8 of row 8 (QN w + q) + l / 8,
    // which must hold chunk (l % 8) ^ ((row >> 1) & 7) of that row.  Rows past the group repeat its last row.
    uint32_t hoff[QN];
#pragma unroll
    for (int q = 0; q < QN; ++q) {
        const int row = 8 * (QN * wave + q) + (lane >> 3);
        const int ch = (lane & 7) ^ ((row >> 1) & 7);
        hoff[q] = (uint32_t)min(row, M - 1) * (uint32_t)H * 2u + (uint32_t)ch * 16u;
    }
    auto stage_h = [&](int slab, int slot) {          // slab index in [0, nslab), ring slot
        const unsigned char* src = A + (size_t)slab * (kMfSlab * 2);
        unsigned char* dst = hbuf + slot * kSlabBytes + (QN * wave) * 1024;
#pragma unroll
        for (int q = 0; q < QN; ++q) lds_dma16(src + hoff[q], dst + q * 1024);
    };

    // ---- W: the wave's panels of a pass and their stream pointers
    const uint16_t* wcur[kMfTN];
    const uint16_t* wnext[kMfTN];
    int wave_p0 = 0, wave_np = 0;
    auto pass_panels = [&](int pass, int& p0, int& np) {
        const int lo = p_begin + pass * n_own / npass;                // 32-bit: passes x panels of a range is small
        const int hi = p_begin + (pass + 1) * n_own / npass;          // 1 <= hi - lo <= 16
        const int m = hi - lo;
        p0 = lo + wave * m / kMfWaves;
        np = lo + (wave + 1) * m / kMfWaves - p0;      // 0 .. 4; p0 < hi is a panel of the matrix either way
    };
    auto panel_ptrs = [&](int p0, int np, const uint16_t* (&ptr)[kMfTN]) {
#pragma unroll
        for (int tn = 0; tn < kMfTN; ++tn) {
            // slots past the wave's share re-read its last panel (branch-free loop); their results are never stored
            const int p = p0 + max(0, min(tn, np - 1));
            ptr[tn] = Wp + (size_t)p * 16 * H + lane * 8;
        }
    };
    u32x4 wreg[RW][2][kMfTN];
    // panel tn of chunk (k-tile t of slab `slab`) of ring slot `slot`; slabs past the end of the pass come from the next
    // pass's panels
    auto fetch_w1 = [&](int slot, int t, int tn, int slab) {
        const bool nxt = slab >= nslab;
        const int sl = nxt ? slab - nslab : slab;
        const uint16_t* base = nxt ? wnext[tn] : wcur[tn];
        wreg[slot][t][tn] = *reinterpret_cast<const u32x4*>(base + (size_t)(sl * 2 + t) * 512);
    };
    auto stage_h1 = [&](int slab, int slot, int q) {  // direct load q of this wave's share of a hidden slab
        lds_dma16(A + (size_t)slab * (kMfSlab * 2) + hoff[q], hbuf + slot * kSlabBytes + (QN * wave + q) * 1024);
    };

    f32x4 acc[kMfTN][TM];
#pragma unroll
    for (int tn = 0; tn < kMfTN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};

    // LDS offset of this lane's fragment of row tile 0, k-tile t inside a slab: row l16, chunk (4 t + kg) ^ ((l16 >> 1) & 7)
    // (row 16 tm + l16 has the same swizzle term: 8 tm vanishes under & 7)
    uint32_t hf_off[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) hf_off[t] = (uint32_t)(l16 * kMfPitch + (((t * 4 + kg) ^ ((l16 >> 1) & 7)) << 4));

    int pass = 0;
    pass_panels(0, wave_p0, wave_np);
    panel_ptrs(wave_p0, wave_np, wcur);
    {
        int p0n, npn;
        pass_panels(npass > 1 ? 1 : 0, p0n, npn);
        panel_ptrs(p0n, npn, wnext);
    }
    // prologue: hidden slabs 0..2 and W slabs 0..3 except the last chunk (the first step requests it); everything has landed
    // before the first step (once per workgroup)
    stage_h(0, 0);
    stage_h(1, 1);
    stage_h(2, 2);
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int tn = 0; tn < kMfTN; ++tn)
                if (r < RW - 1 || t == 0) fetch_w1(r, t, tn, r);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();

    // One step = one slab of 64 k for the whole tile; slab s lives in ring slot s % 4 (hidden in LDS, W in registers), and
    // because H is a multiple of 256 that slot is the same in every pass, so all ring indices are compile-time constants.
    // The steps of all passes form one stream: the requests for the slabs after the end of a pass are the first slabs of
    // the next pass, so the pipeline never drains between tiles.
    // A step is 2 TM groups of 4 MFMAs (one hidden fragment against the wave's 4 panels); after each group at most ONE
    // memory request is issued, so that the four waves of the CU, which run in step, never queue up behind each other at the
    // memory pipeline with nothing left for the matrix cores.  Requests of step s, in program order (fenced: the in-order
    // completion of a wave's requests is what every wait counts on):
    //   groups 0..3            W chunk k-tile 1 of slab s+3 (its ring slot was consumed at the end of the previous step)
    //   groups 4..4+QN-1       direct loads of hidden slab s+3 into the LDS slot that was read in the previous step
    //   groups TM..TM+3        W chunk k-tile 0 of slab s+4 (this step's slot, consumed by groups 0..TM-1)
    // The accumulators are pinned to the accumulation registers by writing the MFMA as an asm statement; its operands are
    // ordinary values, so the compiler still inserts the waits for the W loads and the LDS reads.  Those waits count W
    // loads only (the direct loads are invisible to the compiler): a wait for a chunk requested 3.5 steps ago allows ~28
    // younger requests in flight, i.e. it covers requests at least 1.75 steps old, and a direct load is needed 2.5 steps
    // after it was issued: it is never what the math waits for.
    static_assert(4 + QN <= TM, "the requests of k-tile 0 fit its groups");
    auto do_step = [&](auto rc, int s) {
        constexpr int r = decltype(rc)::value;        // ring slot of slab s
        constexpr int rp = (r + 3) % RW;              // ring slot of slab s-1 = of slab s+3
        const unsigned char* cur = hbuf + r * kSlabBytes;
        int s3 = s + 3;                               // hidden wraps into the next pass (same rows); W takes the next panels
        const int s3h = s3 >= nslab ? s3 - nslab : s3;
        const bool four_panels = wave_np == kMfTN;
        bf16x8 hfq[kHfAhead];
        auto hfrag = [&](int i) {                     // i = t * TM + tm
            return *reinterpret_cast<const bf16x8*>(cur + hf_off[i / TM] + (i % TM) * (16 * kMfPitch));
        };
#pragma unroll
        for (int i = 0; i < kHfAhead; ++i) hfq[i] = hfrag(i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * TM; ++i) {
            const int t = i / TM, tm = i % TM;
            const bf16x8 h = hfq[i % kHfAhead];
            if (tm < TM - 1 || full_tm) {             // wave-uniform
#pragma unroll
                for (int tn = 0; tn < kMfTN; ++tn)
                    if (tn < kMfTN - 1 || four_panels)    // wave-uniform: a panel slot the wave does not own costs no MFMA
                        asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[tn][tm]) : "v"(wreg[r][t][tn]), "v"(h));
            }
            if (i + kHfAhead < 2 * TM) hfq[i % kHfAhead] = hfrag(i + kHfAhead);
            if (i < 4) fetch_w1(rp, 1, i, s3);
            else if (i < 4 + QN) stage_h1(s3h, rp, i - 4);
            else if (i >= TM && i < TM + 4) fetch_w1(r, 0, i - TM, s + RW);
            __builtin_amdgcn_sched_barrier(0);
        }
        // Slab s+1 must be complete in LDS before anybody reads it.  This wave's share was requested in groups 4.. of
        // step s-2; younger than it are 4 W loads of that step and the 8 + QN requests of each of the two steps since (and,
        // after a tile was stored, that tile's stores, which then complete here too).
        constexpr int kYounger = 2 * QN + 20;
        static_assert(kYounger < 64, "s_waitcnt vmcnt has 6 bits");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (kYounger & 15) | ((kYounger >> 4) << 14));
        __syncthreads();
    };
    for (;;) {
        for (int sR = 0; sR < nslab; sR += RW) {
            do_step(std::integral_constant<int, 0>{}, sR);
            do_step(std::integral_constant<int, 1>{}, sR + 1);
            do_step(std::integral_constant<int, 2>{}, sR + 2);
            do_step(std::integral_constant<int, 3>{}, sR + 3);
        }
        // ---- the tile is complete; the next pass's first slabs are already in flight ----
        const int st_p0 = wave_p0, st_np = wave_np;
        ++pass;
        const bool more = pass < npass;
        if (more) {
            pass_panels(pass, wave_p0, wave_np);
#pragma unroll
            for (int tn = 0; tn < kMfTN; ++tn) wcur[tn] = wnext[tn];
            int p0n, npn;
            pass_panels(pass + 1 < npass ? pass + 1 : pass, p0n, npn);
            panel_ptrs(p0n, npn, wnext);
        }
        // acc[tn][tm][i] = C[row 16 tm + l16][entry 16 (st_p0 + tn) + 4 kg + i]
        // (SUMMARY) block of this wave and pass; its span is written once, by the first row group
        int blk = 0, count = 0;
        if constexpr (SUMMARY) {
            blk = (range * sm.passes_per_range + (pass - 1)) * kMfWaves + wave;
            const int first = st_p0 * 16;
            count = max(0, min(st_np * 16, V - first));
            if (group == 0 && lane == 0) { sm.blk_span[2 * blk] = first; sm.blk_span[2 * blk + 1] = count; }
        }
        if (vec_store || SUMMARY) {                   // (the summary instantiations are only launched for V % 4 == 0)
            // V % 4 == 0.  The tile is turned through the wave's own LDS patch so that one store instruction writes all
            // the wave's entries of a row (256 bytes), 4 rows at a time.  LDS operations of one wave execute in order, so
            // the patch needs no barrier and no second copy.
            constexpr int kLanesPerRow = kMfTN * 4, kRowsPerStore = 64 / kLanesPerRow;
            const int srow = lane / kLanesPerRow, scol = (lane % kLanesPerRow) * 4;     // this lane's row and entry when storing
            const int col0 = st_p0 * 16 + scol;
            const bool col_ok = scol < st_np * 16 && col0 < V;
            uint32_t off = ((uint32_t)srow * (uint32_t)V + (uint32_t)col0) * 4u;
            const uint32_t row_step = (uint32_t)kRowsPerStore * 4u * (uint32_t)V;
            // (SUMMARY) running element index of this lane's row in blk_max / blk_sum, stepped like `off`: computed afresh
            // per row it is invariant from pass to pass, and the compiler would keep all 4 TM of them in registers
            uint32_t sat = (uint32_t)(row0 + srow) * (uint32_t)sm.blocks + (uint32_t)blk;
            const uint32_t sat_step = (uint32_t)kRowsPerStore * (uint32_t)sm.blocks;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                f32x4 t[kMfTN];
#pragma unroll
                for (int tn = 0; tn < kMfTN; ++tn) {
                    t[tn] = acc[tn][tm];
                    *reinterpret_cast<f32x4*>(patch + l16 * kMfPatchPitch + (tn * 16 + kg * 4) * 4) = t[tn];
                    if constexpr (!SUMMARY) acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int q = 0; q < 16 / kRowsPerStore; ++q) {
                    const int prow = q * kRowsPerStore + srow, row = tm * 16 + prow;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(patch + prow * kMfPatchPitch + scol * 4);
                    if constexpr (SUMMARY) {
                        // In this layout a row's 64 entries lie in the 16 lanes of one 16-lane row, 4 consecutive entries
                        // each (the values are in registers for the store anyway; taking them from the accumulators instead
                        // needs 16 more registers per tile, which this kernel does not have).  Entries past the block do not
                        // count.  Rotations within the 16-lane row leave the full maximum / sums in every lane.
                        // scale = log2(e)/T of a sampled row; a greedy row gets 1 so that its sum, which nobody reads as a
                        // sum, still turns NaN when the block holds a NaN (fmaxf drops NaNs, the exponential does not)
                        const float rs = row_scale[row];
                        const float scale = rs > 0.0f ? rs : 1.0f;
                        const int lim = count - scol;
                        float x[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = e < lim ? v[e] : -INFINITY;
                        const float m = row16_max(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])));
                        const float base = m > -INFINITY ? m : 0.0f;
                        float z = 0.0f;
#pragma unroll
                        for (int e = 0; e < 4; ++e) z += __builtin_amdgcn_exp2f((x[e] - base) * scale);
                        z = row16_sum(z);
                        if ((lane & 15) == 0 && row < M) {
                            sm.blk_max[sat] = z != z ? z : m;
                            sm.blk_sum[sat] = rs > 0.0f ? z : 0.0f;
                        }
                        sat += sat_step;
                        asm volatile("" : "+v"(sat));
                    }
                    if (row < M && col_ok) {
                        f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<unsigned char*>(C) + off);
                        if constexpr (NT) __builtin_nontemporal_store(v, dst); else *dst = v;
                    }
                    off += row_step;                  // one running byte offset (rows x V x 4 < 2^32 per group)
                    asm volatile("" : "+v"(off));
                }
                // one row tile at a time: left to itself the scheduler interleaves the summaries of all tiles, and their
                // temporaries (16 values each) no longer fit beside the W ring
                if constexpr (SUMMARY) __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (SUMMARY) {
                // the accumulators are cleared only now, behind a fence: cleared tile by tile above, the clears were
                // moved to the front and every old value had to be copied out (and spilled) first
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < kMfTN; ++tn) acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        } else {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
                for (int tn = 0; tn < kMfTN; ++tn) {
                    const int row = tm * 16 + l16, e = (st_p0 + tn) * 16 + kg * 4;
                    if (row < M && tn < st_np) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (e + i < V) C[(size_t)row * V + e + i] = acc[tn][tm][i];
                    }
                    acc[tn][tm] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
        if (!more) break;
    }
    if constexpr (SUMMARY) {                          // block slots of passes this range does not have
        if (group == 0)
            for (int b = npass * kMfWaves + tid; b < sm.passes_per_range * kMfWaves; b += 64 * kMfWaves) {
                sm.blk_span[2 * (range * sm.passes_per_range * kMfWaves + b)] = 0;
                sm.blk_span[2 * (range * sm.passes_per_range * kMfWaves + b) + 1] = 0;
            }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);               // no direct load of this wave is still landing when the LDS is given up
}

Tunable g_lm_packed_tile{0};   // benchmark hook: 0 = automatic (this kernel for M > 160), 1 = the weight-streaming kernel over row groups
Tunable g_lm_mfma_nt{0};       // benchmark hook: nontemporal logits stores, 0 = automatic (one or two row groups), 1 = always, 2 = never
Tunable g_lm_mfma_rows{0};     // benchmark hook: rows per group of this kernel at most (144..256), 0 = automatic (208, or the whole batch up to 256)

// Row groups, panel ranges and the instantiation that serves them (host arithmetic, shared by the launch and by the
// callers that size the block summaries).
struct MfmaLayout { int groups, tiles_lo, groups_hi, tm, ranges, per_range, passes_per_range, blocks; bool nt; };

static MfmaLayout mfma_layout(int M, int V)
{
    constexpr int kMaxTM = 16;
    MfmaLayout L{};
    // Measured on MI355X (V = 151936, H = 4096): M = 1206 as 6 groups of 12-13 tiles 1314 us, as 5 groups of 15-16 tiles
    // 1346 us (the library GEMM of the image with fp32 output: 1342 us); a batch of at most 16 tiles stays one group.
    const int forced = g_lm_mfma_rows;
    const int tiles = (M + 15) / 16;                                     // 16-row tiles of the batch
    const int cap_tiles = forced >= 16 * 9 && forced <= 16 * kMaxTM ? forced / 16 : (tiles <= kMaxTM ? kMaxTM : 13);
    int groups = (tiles + cap_tiles - 1) / cap_tiles;
    while (groups > 1 && (tiles + groups - 1) / groups < 9) --groups;    // the kernel is built for 9..16 tiles per group
    L.groups = groups;
    L.tiles_lo = tiles / groups; L.groups_hi = tiles % groups;           // groups of tiles_lo + 1 first, then of tiles_lo
    L.tm = L.tiles_lo + (L.groups_hi ? 1 : 0);
    const int nt_forced = g_lm_mfma_nt;
    L.nt = nt_forced == 1 || (nt_forced == 0 && groups <= 2);
    // panel ranges: as many as there are CUs per row group, a multiple of 8 (one per XCD and step of the dealing)
    const int cus = device_cu_count();
    const int n_panels = (V + 15) / 16;
    const int r0 = max(8, cus / groups / 8 * 8);
    L.per_range = (n_panels + r0 - 1) / r0;
    L.ranges = ((n_panels + L.per_range - 1) / L.per_range + 7) / 8 * 8;
    L.passes_per_range = (L.per_range + kMfPassPanels - 1) / kMfPassPanels;
    L.blocks = L.ranges * L.passes_per_range * kMfWaves;
    return L;
}

template <int TM, bool NT, bool SUMMARY>
static int launch_mfma(const uint16_t* a, const uint16_t* wp, float* c, int M, int H, int V, const MfmaLayout& L, LmSummary sm, hipStream_t s)
{
    constexpr int SR = (TM * 16 + 31) / 32 * 32;
    const size_t smem = (size_t)kMfRing * SR * kMfPitch + (size_t)kMfWaves * 16 * kMfPatchPitch + (SUMMARY ? TM * 16 * 4 : 0);
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&lm_head_mfma_kernel<TM, NT, SUMMARY>), smem, granted, "spec_lm_head_packed")) return rc;
    hipLaunchKernelGGL((lm_head_mfma_kernel<TM, NT, SUMMARY>), dim3(L.ranges * L.groups), dim3(64 * kMfWaves), smem, s, a, wp, c, M, H, V,
                       (V + 15) / 16, L.per_range, V % 4 == 0, L.groups, L.tiles_lo, L.groups_hi, sm);
    return SPEC_OK;
}

// blocks per row of the summaries for this shape; 0 if the large-tile kernel does not take it
int lm_head_mfma_blocks(int M, int H, int V)
{
    // (V % 4 == 0: the summaries are taken while whole rows of the tile are stored; 32-bit element indices)
    if (M <= 0 || V <= 0 || V % 4 != 0 || H <= 0 || H % (kMfRing * kMfSlab) != 0) return 0;
    const MfmaLayout L = mfma_layout(M, V);
    if ((size_t)M * (size_t)L.blocks >= ((size_t)1 << 32)) return 0;
    return (L.tm >= 9 && L.tm <= 16) ? L.blocks : 0;
}

// Returns SPEC_OK after enqueueing, or a negative status.  summary == nullptr: logits only.
int lm_head_mfma_dispatch(const uint16_t* a, const uint16_t* wp, float* c, int M, int H, int V, const LmSummary* summary, hipStream_t s)
{
    const MfmaLayout L = mfma_layout(M, V);
    if (H % (kMfRing * kMfSlab) != 0)
        return fail(SPEC_ESHAPE, "spec_lm_head_packed: H=%d must be a multiple of %d", H, kMfRing * kMfSlab);
    LmSummary sm{};
    if (summary) {
        if (lm_head_mfma_blocks(M, H, V) == 0)
            return fail(SPEC_ESHAPE, "spec_lm_head_packed_summary: no block summaries for M=%d H=%d V=%d (V must be a multiple of 4)", M, H, V);
        sm = *summary; sm.blocks = L.blocks; sm.passes_per_range = L.passes_per_range;
    }
    switch (L.tm) {
#define SPECV_MF(TMv)                                                                                             \
        case TMv:                                                                                                 \
            if (summary) return L.nt ? launch_mfma<TMv, true, true>(a, wp, c, M, H, V, L, sm, s)                  \
                                     : launch_mfma<TMv, false, true>(a, wp, c, M, H, V, L, sm, s);                \
            return L.nt ? launch_mfma<TMv, true, false>(a, wp, c, M, H, V, L, sm, s)                              \
                        : launch_mfma<TMv, false, false>(a, wp, c, M, H, V, L, sm, s);
        SPECV_MF(9) SPECV_MF(10) SPECV_MF(11) SPECV_MF(12) SPECV_MF(13) SPECV_MF(14) SPECV_MF(15) SPECV_MF(16)
#undef SPECV_MF
        default: break;
    }
    return fail(SPEC_ESHAPE, "spec_lm_head_packed: no large-tile instantiation for %d row tiles per group", L.tm);
}

}  // namespace specv
