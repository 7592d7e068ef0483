// spec_verify_attn: ragged multi-query paged attention of the verification candidates (paper, Method:
// the target performs the verification pass on the merged batch Y_n; gamma_i = 0 rows are the padded
// parallel-mode candidates, i.e. ordinary decode).
//
// Work decomposition (HBM-bound: 512 bytes of K+V per key per kv head, 8..72 flop per byte):
//   grid = (kv split, kv head, request).  A workgroup of NW waves (8 when the query block is at most 32
//   rows, else 4) streams one contiguous chunk of one request's keys for one kv head; wave w owns keys
//   32w..32w+31 of every 32*NW-key step and all G * n_i query rows (query heads of the group x
//   candidate positions).  A wave copies ITS two pages
//   (K and V, 4 KB each, contiguous in HBM) straight into its private 16 KB of LDS with direct
//   global->LDS loads (no staging registers), so the waves of a workgroup never wait for each other
//   inside the loop; latency is hidden by the other waves resident on the SIMD.
//   Scores are computed transposed, S^T = K Q^T (v_mfma_f32_16x16x32_bf16, keys on the MFMA row
//   axis): a lane then holds 4 keys of ONE query row, the row maximum is an in-lane max plus two
//   cross-lane shuffles, and exp(S^T) is already the B operand of O^T += V^T P^T.  K and V stay
//   row-major in LDS (XOR-swizzled 16 B / 32 B chunks instead of padding); the V^T operand comes from
//   the transposing LDS read (ds_read_b64_tr_b16), Q fragments are re-read from a shared LDS copy.
//   Every chunk writes an unnormalised fp32 partial (O, running max, sum); a second kernel merges the
//   partials of a row in split order (deterministic) and writes bf16.
#include "common.h"

#include <cmath>
#include <type_traits>

namespace specv {

constexpr int kD = 128;                      // head dimension
constexpr int kP = 16;                       // tokens per page
constexpr int kRowBytes = kD * 2;            // one K or V row in LDS (unpadded, swizzled)
constexpr int kWaveLds = 2 * 32 * kRowBytes; // per wave: 32 K rows + 32 V rows = 16 KB
constexpr int kRedPitch = 36;                // floats per row of the epilogue reduction buffer (32 + 4)
constexpr float kNegBig = -1.0e30f;          // "nothing seen yet" running maximum (log2 domain)
constexpr float kMaxSlack = 6.0f;            // how far a step's maximum may exceed the reference before a rescale

typedef short s16x4 __attribute__((ext_vector_type(4)));

// Transposing LDS read.  In every group of 16 lanes, lane r supplies the address of 4 consecutive
// 16-bit elements M[r][0..3]; lane j receives M[j/4][j%4], M[4 + j/4][j%4], M[8 + j/4][j%4], M[12 + j/4][j%4].
__device__ inline s16x4 lds_read_tr(const void* lds)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)lds);
}

struct AttnParams {
    const uint16_t* q;
    const uint16_t* k_cache;
    const uint16_t* v_cache;
    const int32_t* page_table;
    const int32_t* seq_lens;
    const int32_t* qo_indptr;
    uint16_t* out;      // [M, Hq, 128] bf16
    float* lse;         // [M, Hq] or null
    float* part_o;      // [M*Hq, splits, 128]
    float* part_m;      // [M*Hq, splits]   running max, log2 domain
    float* part_l;      // [M*Hq, splits]
    int32_t* status_flags;
    // balanced work list written by verify_attn_plan_kernel (all null when requests are split by the fixed
    // chunk_target instead): hdr = {items, keys per chunk}; req[i] = {splits of request i, first partial slot};
    // items[k] = {request, split, splits of the request, first partial slot}
    const int32_t* parent;     // tree verification: row-local parent of every candidate row ([M], -1 for a root), or null = chains
    const int32_t* plan_hdr;
    const int32_t* plan_req;
    const int32_t* plan_items;
    int max_pages, num_pages, Hq, Hkv, G, M, max_kv_len, max_q_len, chunk_target, splits;
    float scale_log2e;
};

__device__ inline bool request_ok(int r0, int n, int c, const AttnParams& p)
{
    return n >= 1 && n <= p.max_q_len && r0 >= 0 && r0 + n <= p.M && c >= 0 && c + n <= p.max_kv_len;
}

// NR: 16-row query tiles per (request, kv head); NW: waves per workgroup (each owns 32 keys of a step);
// FINAL: no request is split, so the workgroup normalises and writes bf16 itself (no partials, no merge kernel).
// NBUF: K/V buffers per wave (2 = the next step's pages are in flight while this step is computed).
template <int NR, int NW, int NBUF, bool FINAL>
__global__ __launch_bounds__(NW * 64) void verify_attn_kernel(AttnParams p)
{
    constexpr int kThreads = NW * 64;
    constexpr int kTile = NW * 32;                    // keys per workgroup step
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int kvh = blockIdx.y;
    int split, i, ns_plan = 0, pb_plan = 0;
    if (p.plan_items) {
        // one workgroup per item of the balanced list; the grid is sized from a host bound
        if ((int)blockIdx.x >= p.plan_hdr[0]) return;
        const int* it = p.plan_items + 4 * (size_t)blockIdx.x;
        i = __builtin_amdgcn_readfirstlane(it[0]);
        split = __builtin_amdgcn_readfirstlane(it[1]);
        ns_plan = __builtin_amdgcn_readfirstlane(it[2]);
        pb_plan = __builtin_amdgcn_readfirstlane(it[3]);
    } else {
        split = blockIdx.x;
        i = blockIdx.z;
    }
    unsigned char* sKV = smem + wave * (NBUF * kWaveLds); // this wave's NBUF x (32 K rows, 32 V rows)
    unsigned char* sQ = smem + NW * NBUF * kWaveLds;      // shared: NR*16 query rows
    int32_t* sPT = reinterpret_cast<int32_t*>(sQ + NR * 16 * kRowBytes);   // shared: page ids of this chunk

    const int r0 = p.qo_indptr[i], n = p.qo_indptr[i + 1] - r0, c = p.seq_lens[i];
    if (!request_ok(r0, n, c, p)) {
        if (!p.plan_items && split == 0 && kvh == 0 && tid == 0 && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_LENGTH);
        return;
    }
    const int len = c + n;
    const int ns = p.plan_items ? ns_plan : (len + p.chunk_target - 1) / p.chunk_target;
    if (split >= ns) return;
    const int chunk = (((len + ns - 1) / ns) + kP - 1) & ~(kP - 1);
    const int kbeg = split * chunk;
    const int kend = min(len, kbeg + chunk);
    // partial slot of (candidate row j, head h, split): part_base + (j*Hq + h)*part_ns + split
    const size_t part_base = p.plan_items ? (size_t)pb_plan : (size_t)r0 * p.Hq * p.splits;
    const size_t part_ns = p.plan_items ? (size_t)ns : (size_t)p.splits;
    const int G = p.G, R = G * n;
    const int nrt = (R + 15) >> 4;                        // row tiles this request really has (wave-uniform, <= NR)
    const int32_t* pt = p.page_table + (size_t)i * p.max_pages;

    // ---- page ids of the chunk -> LDS, validated once (page 0 stands in for a bad id, which is flagged).
    // Inside the loop they are read back from LDS: a global load there would sit in the same in-order
    // queue as the direct K/V loads and force them to drain. ----
    int bad_page = 0;
    const int npages = (kend - kbeg + kP - 1) / kP;
    for (int pg = tid; pg < npages; pg += kThreads) {
        int page = pt[kbeg / kP + pg];
        if (page < 0 || page >= p.num_pages) { page = 0; bad_page = 1; }
        sPT[pg] = page;
    }
    __syncthreads();

    // ---- this wave's two pages of a step, K and V, HBM -> LDS (always 16 direct loads: positions past the
    // range read page 0 instead, so the wait counts below are constants) ----
    const int drow = lane >> 4, dpos = lane & 15;        // direct-load role: row within a group of 4, 16-byte position
    auto issue_step = [&](int wbase, unsigned char* buf) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            const int t0 = wbase + pg * kP;
            const int page = (t0 < kend) ? __builtin_amdgcn_readfirstlane(sPT[(t0 - kbeg) / kP]) : 0;
            const size_t base = ((size_t)page * p.Hkv + kvh) * (kP * kD);
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int row = q4 * 4 + drow;             // slot in the page = key & 15
                // K: chunk ch of a row is stored at position ch ^ (row & 15)
                lds_dma16(p.k_cache + base + row * kD + ((dpos ^ row) << 3), buf + (pg * 16 + q4 * 4) * kRowBytes);
                // V: 32-byte chunk c of a row is stored at position c ^ (row & 7)
                const int src16 = ((((dpos >> 1) ^ (row & 7)) << 1) | (dpos & 1));
                lds_dma16(p.v_cache + base + row * kD + (src16 << 3), buf + (32 + pg * 16 + q4 * 4) * kRowBytes);
            }
        }
    };
    const int wfirst = kbeg + wave * 32;
    if (wfirst < kend) issue_step(wfirst, sKV);           // in flight while Q is staged

    // ---- query rows -> LDS (row r = j*G + gq; 16-byte chunk ch of row r sits at position ch ^ (r & 15)) ----
    for (int idx = tid; idx < NR * 16 * 16; idx += kThreads) {
        const int row = idx >> 4, ch = idx & 15;
        u32x4 val = u32x4{0, 0, 0, 0};
        if (row < R) {
            const int j = row / G, gq = row - j * G;
            val = *reinterpret_cast<const u32x4*>(p.q + ((size_t)(r0 + j) * p.Hq + kvh * G + gq) * kD + ch * 8);
        }
        *reinterpret_cast<u32x4*>(sQ + row * kRowBytes + ((ch ^ (row & 15)) << 4)) = val;
    }
    int limit[NR];                    // row sees key positions t < limit
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) {
        const int r = rt * 16 + l16;
        limit[rt] = (r < R) ? min(c + r / G + 1, kend) : 0;
    }
    // Tree verification: candidate row j sees the committed prefix and the rows on its own path to the root.
    // anc[rt] has bit a set iff candidate a is such a row for this lane's query row (n <= 64 in this mode).
    const bool tree = p.parent != nullptr;
    // (the masks live in LDS and are read in the few steps that reach the candidates: in registers they would
    // cost every step of the loop two registers per row tile)
    int32_t* sPar = sPT + (min(p.chunk_target, p.max_kv_len) / kP + 1);
    unsigned long long* sAnc = reinterpret_cast<unsigned long long*>(sPar + 64);   // [NR * 16], 8-byte aligned
    if (tree) {
        int bad_tree = 0;
        if (tid < n) {
            const int par = p.parent[r0 + tid];
            sPar[tid] = par;
            bad_tree = tid == 0 ? par != -1 : (par < 0 || par >= tid);
        }
        if (__syncthreads_or(bad_tree)) {                 // uniform: the whole workgroup leaves the request alone
            if (tid == 0 && split == 0 && kvh == 0 && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_TREE);
            __builtin_amdgcn_s_waitcnt(0x0F70);           // the first step's direct loads have landed before the LDS is given up
            return;
        }
#pragma unroll
        for (int rt = 0; rt < NR; ++rt) limit[rt] = (rt * 16 + l16 < R) ? kend : 0;
    }
    // chains: every candidate below the causal limit is on the path (all bits set), so one masking loop serves both
    for (int r = tid; r < NR * 16; r += kThreads) {
        unsigned long long m = ~0ull;
        if (tree) {
            m = 0ull;
            if (r < R)
                for (int a = r / G; a >= 0; a = sPar[a]) m |= 1ull << a;
        }
        sAnc[r] = m;
    }
    __syncthreads();

    f32x4 o[NR][8];
    float m_run[NR], l_run[NR];
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) {
        m_run[rt] = kNegBig;
        l_run[rt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[rt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // The loop is instantiated for every number of row tiles A <= NR a request can have, so that a decode
    // row in a batch sized for 9-row candidates pays for one tile of math, not five.
    auto run_chunk = [&](auto active) {
    constexpr int A = decltype(active)::value;
    int it = 0;
    for (int wbase = wfirst; wbase < kend; wbase += kTile, ++it) {
        unsigned char* sK = sKV + (NBUF == 2 ? (it & 1) * kWaveLds : 0);
        unsigned char* sV = sK + 32 * kRowBytes;
        if (NBUF == 2) {
            // the other buffer was last read in the previous step; its reads have returned
            __builtin_amdgcn_s_waitcnt(0xC07F);           // lgkmcnt(0)
            if (wbase + kTile < kend) {
                issue_step(wbase + kTile, sKV + ((it + 1) & 1) * kWaveLds);
                __builtin_amdgcn_s_waitcnt(0x4F70);       // vmcnt(16): this step's pages have landed, the next 16 loads fly on
            } else {
                __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
            }
        } else {
            if (it > 0) {
                __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): the previous step's LDS reads have returned
                issue_step(wbase, sKV);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0): this step's pages have landed
        }
        if (wbase + 32 > kend) {
            // slots past the range may hold anything (even NaN patterns): P is 0 there, so V must be too
            for (int idx = lane; idx < 32 * 16; idx += 64) {
                const int row = idx >> 4;
                if (wbase + row >= kend) *reinterpret_cast<u32x4*>(sV + row * kRowBytes + (idx & 15) * 16) = u32x4{0, 0, 0, 0};
            }
        }

        // ---- S^T = K Q^T for the wave's two 16-key blocks ----
        bf16x8 kf[2][4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                kf[kb][s] = *reinterpret_cast<const bf16x8*>(sK + (kb * 16 + l16) * kRowBytes + (((s * 4 + g) ^ l16) << 4));
        const bool need_mask = wbase + 32 > min(c + 1, kend);
        // The row tiles go through every phase together (scores, maxima, exponentials) so that the
        // dependent chains of different tiles (MFMA -> max -> cross-lane max -> exp) overlap in the one wave.
        float sc[A][8];
#pragma unroll
        for (int rt = 0; rt < A; ++rt) {
            bf16x8 qf[4];
#pragma unroll
            for (int s = 0; s < 4; ++s)
                qf[s] = *reinterpret_cast<const bf16x8*>(sQ + (rt * 16 + l16) * kRowBytes + (((s * 4 + g) ^ l16) << 4));
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][s], qf[s], acc, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) sc[rt][kb * 4 + e] = acc[e] * p.scale_log2e;
            }
        }
        if (need_mask) {
#pragma unroll
            for (int rt = 0; rt < A; ++rt) {
                const unsigned long long anc = sAnc[rt * 16 + l16];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int t = wbase + kb * 16 + g * 4 + e, rel = t - c;
                        // a tree has at most 64 candidates (rel < 64 below the limit); a chain's mask is all ones
                        const bool seen = t < limit[rt] && (rel < 0 || ((anc >> (rel & 63)) & 1ull));
                        if (!seen) sc[rt][kb * 4 + e] = kNegBig;                       // exp2 of it is 0
                    }
            }
        }
        float tmax[A];
#pragma unroll
        for (int rt = 0; rt < A; ++rt) {
            float t = sc[rt][0];
#pragma unroll
            for (int e = 1; e < 8; ++e) t = fmaxf(t, sc[rt][e]);
            tmax[rt] = t;
        }
#pragma unroll
        for (int rt = 0; rt < A; ++rt) tmax[rt] = fmaxf(tmax[rt], __shfl_xor(tmax[rt], 16, 64));
#pragma unroll
        for (int rt = 0; rt < A; ++rt) tmax[rt] = fmaxf(tmax[rt], __shfl_xor(tmax[rt], 32, 64));
        // Lazy reference maximum: m_run only moves when a step's maximum exceeds it by more than kMaxSlack
        // (log2 units), so exp2(s - m_run) <= 2^kMaxSlack stays well inside fp32/bf16 range and the 32
        // accumulator registers of a row tile are rescaled a handful of times per chunk instead of almost
        // every step.  The result is the same softmax: O and l carry the same factor.
        bool grow = false;
#pragma unroll
        for (int rt = 0; rt < A; ++rt) grow |= tmax[rt] > m_run[rt] + kMaxSlack;
        if (__any(grow)) {
#pragma unroll
            for (int rt = 0; rt < A; ++rt) {
                if (__any(tmax[rt] > m_run[rt] + kMaxSlack)) {
                    const float m_new = fmaxf(m_run[rt], tmax[rt]);
                    const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
                    m_run[rt] = m_new;
                    l_run[rt] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) o[rt][dt] *= alpha;
                }
            }
        }
        bf16x8 pf[A];
#pragma unroll
        for (int rt = 0; rt < A; ++rt) {
            const float m_ref = m_run[rt];
            float pr[8], psum = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // a masked score is kNegBig: exp2(kNegBig - m_ref) is 0 unless the row has seen nothing at all
                // (m_ref == kNegBig), and such a row is masked by the comparison
                pr[e] = __builtin_amdgcn_exp2f(sc[rt][e] - m_ref);
                if (need_mask) pr[e] = (sc[rt][e] > 0.5f * kNegBig) ? pr[e] : 0.0f;
                psum += pr[e];
            }
            l_run[rt] += psum;
            const u32x4 pw = u32x4{pack_bf16x2(pr[0], pr[1]), pack_bf16x2(pr[2], pr[3]),
                                   pack_bf16x2(pr[4], pr[5]), pack_bf16x2(pr[6], pr[7])};
            pf[rt] = __builtin_bit_cast(bf16x8, pw);
        }
        // ---- O^T += V^T P^T: lane (d = 16dt + l16, k-group g) needs keys 4g..4g+3 of both blocks at one d.
        // For the transposing read, lane r of a group supplies key 4g + r/4, d = 16dt + 4*(r%4) .. +3. ----
        {
            const int vrow = 4 * g + (l16 >> 2);
            const unsigned char* v0 = sV + vrow * kRowBytes + 8 * (l16 & 3);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                const int off = (dt ^ (vrow & 7)) << 5;
                const s16x4 lo = lds_read_tr(v0 + off);
                const s16x4 hi = lds_read_tr(v0 + 16 * kRowBytes + off);
                struct { s16x4 a, b; } pair = {lo, hi};
                const bf16x8 vf = __builtin_bit_cast(bf16x8, pair);
#pragma unroll
                for (int rt = 0; rt < A; ++rt) o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[rt], o[rt][dt], 0, 0, 0);
            }
        }
    }
    };
    switch (nrt) {
        case 1: run_chunk(std::integral_constant<int, 1>{}); break;
        case 2: if constexpr (NR >= 2) run_chunk(std::integral_constant<int, 2>{}); break;
        case 3: if constexpr (NR >= 3) run_chunk(std::integral_constant<int, 3>{}); break;
        case 4: if constexpr (NR >= 4) run_chunk(std::integral_constant<int, 4>{}); break;
        case 5: if constexpr (NR >= 5) run_chunk(std::integral_constant<int, 5>{}); break;
        case 6: if constexpr (NR >= 6) run_chunk(std::integral_constant<int, 6>{}); break;
        case 7: if constexpr (NR >= 7) run_chunk(std::integral_constant<int, 7>{}); break;
        default: if constexpr (NR >= 8) run_chunk(std::integral_constant<int, 8>{}); break;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // nothing of this wave is still landing in LDS
    if (bad_page && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_PAGE);

    // ---- merge the waves: common maximum, then O in 4 slices of 32 d through LDS ----
    __syncthreads();                                      // every wave is done with its K/V rows and with Q
    float* s_m = reinterpret_cast<float*>(smem);          // [NW][NR*16]
    float* s_l = s_m + NW * NR * 16;                      // [NW][NR*16]
    float* s_mx = s_l + NW * NR * 16;                     // [NR*16] merged maximum
    float* s_lt = s_mx + NR * 16;                         // [NR*16] merged sum
    float* s_red = s_lt + NR * 16;                        // [NW][NR*16][kRedPitch]
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) {
        float l = l_run[rt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (g == 0) {
            s_m[wave * NR * 16 + rt * 16 + l16] = m_run[rt];
            s_l[wave * NR * 16 + rt * 16 + l16] = l;
        }
    }
    __syncthreads();
    for (int r = tid; r < NR * 16; r += kThreads) {
        float mx = kNegBig;
#pragma unroll
        for (int w = 0; w < NW; ++w) mx = fmaxf(mx, s_m[w * NR * 16 + r]);
        float l = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += s_l[w * NR * 16 + r] * exp2f(s_m[w * NR * 16 + r] - mx);
        s_mx[r] = mx;
        s_lt[r] = l;
    }
    __syncthreads();
    float fscale[NR];
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) fscale[rt] = exp2f(m_run[rt] - s_mx[rt * 16 + l16]);
    // rows of this unit: r = j*G + gq  ->  global (row r0+j, head kvh*G+gq)
#pragma unroll
    for (int ds = 0; ds < 4; ++ds) {
#pragma unroll
        for (int rt = 0; rt < NR; ++rt)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const f32x4 v = o[rt][ds * 2 + half] * fscale[rt];
                *reinterpret_cast<f32x4*>(s_red + ((size_t)(wave * NR * 16 + rt * 16 + l16)) * kRedPitch + half * 16 + g * 4) = v;
            }
        __syncthreads();
        for (int e = tid; e < R * 32; e += kThreads) {
            const int r = e >> 5, dl = e & 31;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += s_red[(size_t)(w * NR * 16 + r) * kRedPitch + dl];
            const int j = r / G, gq = r - j * G;
            const size_t rowhead = (size_t)(r0 + j) * p.Hq + kvh * G + gq;
            if (FINAL) p.out[rowhead * kD + ds * 32 + dl] = (uint16_t)f32_to_bf16_bits(sum / s_lt[r]);
            else p.part_o[(part_base + ((size_t)j * p.Hq + kvh * G + gq) * part_ns + split) * kD + ds * 32 + dl] = sum;
        }
        __syncthreads();
    }
    for (int r = tid; r < R; r += kThreads) {
        const int j = r / G, gq = r - j * G;
        const size_t rowhead = (size_t)(r0 + j) * p.Hq + kvh * G + gq;
        if (FINAL) {
            if (p.lse) p.lse[rowhead] = (s_mx[r] + log2f(s_lt[r])) * 0.6931471805599453f;
        } else {
            const size_t slot = part_base + ((size_t)j * p.Hq + kvh * G + gq) * part_ns + split;
            p.part_m[slot] = s_mx[r];
            p.part_l[slot] = s_lt[r];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Large query blocks (4..8 row tiles: 49..128 query rows per kv head, e.g. 8 query heads x 9 candidate rows).
// With that many rows the decomposition above keeps 32 accumulator registers per row tile in EVERY wave, which leaves
// one 4-wave workgroup per CU, one K/V step in flight per wave, a cross-wave merge of all those accumulators at the end
// of every chunk, and a prologue nobody overlaps: on chunks of ~1000 keys that overhead is as long as the streaming.
// Here the ROWS are divided instead: wave w owns row tile w (its Q fragments in registers, its softmax state and its
// 32 accumulator registers) and sees every key of the chunk; the K/V stages (32 keys = two pages of K and of V, 16 KB)
// are shared by the waves through a ring of two LDS buffers (four is an option) filled by direct global->LDS loads.
// A row belongs to one wave, so there is no merge: a wave normalises and stores its own 16 rows.  32 KB of LDS and ~100
// registers per wave let three to four workgroups share a CU, so that one's waits hide under the others' streams.
// ------------------------------------------------------------------------------------------------
constexpr int kRowsStageBytes = kWaveLds;      // 32 K rows + 32 V rows

// RING: K/V stages per workgroup in LDS (RING - 1 of them in flight while one is computed)
template <int NW, bool FINAL, int RING>
__global__ __launch_bounds__(NW * 64, (NW <= 5 ? 4 : (NW == 6 ? 3 : 2))) void verify_attn_rows_kernel(AttnParams p)
{
    constexpr int kRowsStages = RING;
    constexpr int kThreads = NW * 64;
    constexpr int kIssue = (16 + NW - 1) / NW;            // direct loads per wave and stage (16 in all; surplus slots repeat the last)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int kvh = blockIdx.y;
    int split, i, ns_plan = 0, pb_plan = 0;
    if (p.plan_items) {
        if ((int)blockIdx.x >= p.plan_hdr[0]) return;
        const int* it = p.plan_items + 4 * (size_t)blockIdx.x;
        i = __builtin_amdgcn_readfirstlane(it[0]);
        split = __builtin_amdgcn_readfirstlane(it[1]);
        ns_plan = __builtin_amdgcn_readfirstlane(it[2]);
        pb_plan = __builtin_amdgcn_readfirstlane(it[3]);
    } else {
        split = blockIdx.x;
        i = blockIdx.z;
    }
    unsigned char* sRing = smem;                                         // kRowsStages x (32 K rows, 32 V rows)
    int32_t* sPT = reinterpret_cast<int32_t*>(smem + kRowsStages * kRowsStageBytes);   // page ids of this chunk

    const int r0 = p.qo_indptr[i], n = p.qo_indptr[i + 1] - r0, c = p.seq_lens[i];
    if (!request_ok(r0, n, c, p)) {
        if (!p.plan_items && split == 0 && kvh == 0 && tid == 0 && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_LENGTH);
        return;
    }
    const int len = c + n;
    const int ns = p.plan_items ? ns_plan : (len + p.chunk_target - 1) / p.chunk_target;
    if (split >= ns) return;
    const int chunk = (((len + ns - 1) / ns) + kP - 1) & ~(kP - 1);
    const int kbeg = split * chunk;
    const int kend = min(len, kbeg + chunk);
    const size_t part_base = p.plan_items ? (size_t)pb_plan : (size_t)r0 * p.Hq * p.splits;
    const size_t part_ns = p.plan_items ? (size_t)ns : (size_t)p.splits;
    const int G = p.G, R = G * n;
    const int32_t* pt = p.page_table + (size_t)i * p.max_pages;

    // ---- page ids of the chunk -> LDS, validated once (page 0 stands in for a bad id, which is flagged) ----
    int bad_page = 0;
    const int npages = (kend - kbeg + kP - 1) / kP;
    for (int pg = tid; pg < npages; pg += kThreads) {
        int page = pt[kbeg / kP + pg];
        if (page < 0 || page >= p.num_pages) { page = 0; bad_page = 1; }
        sPT[pg] = page;
    }
    // ---- this wave's row tile: Q fragments straight into registers (row r = j*G + gq), and what the row may see ----
    const int row = wave * 16 + l16;
    const bool row_ok = row < R;
    const int qj = row_ok ? row / G : 0, qg = row_ok ? row - qj * G : 0;
    const size_t rowhead = (size_t)(r0 + qj) * p.Hq + kvh * G + qg;
    bf16x8 qf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        u32x4 v = u32x4{0, 0, 0, 0};
        if (row_ok) v = *reinterpret_cast<const u32x4*>(p.q + rowhead * kD + (s * 4 + g) * 8);
        qf[s] = __builtin_bit_cast(bf16x8, v);
    }
    const bool tree = p.parent != nullptr;
    int limit = row_ok ? (tree ? kend : min(c + qj + 1, kend)) : 0;      // the row sees key positions t < limit
    // tree verification: bit a of anc is set iff candidate a is on this row's path to the root (a chain: all ones)
    int32_t* sPar = sPT + (min(p.chunk_target, p.max_kv_len) / kP + 1);
    // (the masks live in LDS and are read in the few stages that reach the candidates, as in the kernel above)
    unsigned long long* sAnc = reinterpret_cast<unsigned long long*>(sPar + 64);   // [NW * 16]
    if (tree) {
        int bad_tree = 0;
        if (tid < n) {
            const int par = p.parent[r0 + tid];
            sPar[tid] = par;
            bad_tree = tid == 0 ? par != -1 : (par < 0 || par >= tid);
        }
        if (__syncthreads_or(bad_tree)) {                 // uniform: the whole workgroup leaves the request alone
            if (tid == 0 && split == 0 && kvh == 0 && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_TREE);
            return;
        }
    }
    // chains: every candidate below the causal limit is on the path (all bits set), so one masking loop serves both
    for (int r = tid; r < NW * 16; r += kThreads) {
        unsigned long long m = ~0ull;
        if (tree) {
            m = 0ull;
            if (r < R)
                for (int a = r / G; a >= 0; a = sPar[a]) m |= 1ull << a;
        }
        sAnc[r] = m;
    }
    __syncthreads();                                      // page ids and masks visible
    // The Q fragments came by ordinary loads.  The compiler cannot see the direct loads below (inline assembly), and with
    // some of them always in flight (rings deeper than two) it would make the loop wait for "all loads" at the first use
    // of a fragment in every stage, which serialises the ring (measured 230 against 187 us).  Waiting once here and handing
    // the registers through an empty statement tells it that nothing is pending on them.
    __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
    for (int s = 0; s < 4; ++s) asm volatile("" : "+v"(qf[s]));

    // ---- stage st of the chunk (keys kbeg + 32 st ..): its 16 direct loads are dealt to the waves, kIssue each; slots past the
    // range read page 0 (never used), so that the wait counts are constants ----
    const int drow = lane >> 4, dpos = lane & 15;        // direct-load role: row within a group of 4, 16-byte position
    auto issue_stage = [&](int st) {
        unsigned char* buf = sRing + (st & (kRowsStages - 1)) * kRowsStageBytes;
        const int t0s = kbeg + st * 32;
#pragma unroll
        for (int k = 0; k < kIssue; ++k) {
            // with a ring of two the wait in front of a stage is "all of this wave's loads", so a surplus slot may
            // simply stay empty; deeper rings count loads per stage, there the surplus slots repeat the last load
            if (kRowsStages == 2 && wave * kIssue + k > 15) break;
            const int q = min(wave * kIssue + k, 15);     // load q of the stage: which of K/V, which page, which 4 rows
            const int isv = q >> 3, pg = (q >> 2) & 1, q4 = q & 3;
            const int t0 = t0s + pg * kP;
            const int page = (t0 < kend) ? __builtin_amdgcn_readfirstlane(sPT[(t0 - kbeg) / kP]) : 0;
            const size_t base = ((size_t)page * p.Hkv + kvh) * (kP * kD);
            const int row4 = q4 * 4 + drow;               // slot in the page = key & 15
            // K: 16-byte chunk ch of a row is stored at position ch ^ (row & 15); V: 32-byte chunk c at c ^ (row & 7)
            const int src16 = isv ? ((((dpos >> 1) ^ (row4 & 7)) << 1) | (dpos & 1)) : (dpos ^ row4);
            const uint16_t* src = (isv ? p.v_cache : p.k_cache) + base + row4 * kD + (src16 << 3);
            lds_dma16(src, buf + (isv * 32 + pg * 16 + q4 * 4) * kRowBytes);
        }
    };
    const int nst = (kend - kbeg + 31) >> 5;
    const bool wave_has_rows = wave * 16 < R;
    // a masked raw score: scaled it is kNegBig.  A caller's scale <= 0 makes no sense for a softmax; it is clamped to a tiny
    // positive value so that the arithmetic stays finite
    const float scale = fmaxf(p.scale_log2e, 1e-30f);
    const float kMaskedRaw = kNegBig / scale < -3.0e38f ? -3.0e38f : kNegBig / scale;
#pragma unroll
    for (int st = 0; st < kRowsStages - 1; ++st) issue_stage(st);

    f32x4 o[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.0f;

    // the stage loop is unrolled over the ring, so that a stage's buffer is a compile-time offset of every LDS read
    auto do_stage = [&](auto slot, int st) {
        // this wave's loads of stage st have landed (RING - 2 younger stages may still fly); the barrier then says that every
        // wave's have, and that every wave is done reading the buffer that stage st + RING - 1 is about to overwrite
        constexpr int kYounger = (kRowsStages - 2) * kIssue;
        __builtin_amdgcn_s_waitcnt(0x0F70 | (kYounger & 15) | ((kYounger >> 4) << 14));
        __syncthreads();
        issue_stage(st + kRowsStages - 1);
        const int wbase = kbeg + st * 32;
        unsigned char* sK = sRing + decltype(slot)::value * kRowsStageBytes;
        unsigned char* sV = sK + 32 * kRowBytes;
        if (wbase + 32 > kend) {
            // slots past the range may hold anything (even NaN patterns): P is 0 there, so V must be too
            for (int idx = tid; idx < 32 * 16; idx += kThreads) {
                const int vr = idx >> 4;
                if (wbase + vr >= kend) *reinterpret_cast<u32x4*>(sV + vr * kRowBytes + (idx & 15) * 16) = u32x4{0, 0, 0, 0};
            }
            __syncthreads();
        }
        if (!wave_has_rows) return;                       // wave-uniform: a request with fewer row tiles than the launch was built for
        // ---- S^T = K Q^T for the two 16-key blocks; sc holds the RAW dot products, the softmax scale (log2 domain) is
        // folded into the one multiply-add in front of every exponential ----
        float sc[8];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + (kb * 16 + l16) * kRowBytes + (((s * 4 + g) ^ l16) << 4));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[s], acc, 0, 0, 0);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) sc[kb * 4 + e] = acc[e];
        }
        const bool need_mask = wbase + 32 > min(c + 1, kend);
        if (need_mask) {
            const unsigned long long anc = sAnc[row];
            const uint32_t anc_lo = (uint32_t)anc, anc_hi = (uint32_t)(anc >> 32);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int t = wbase + kb * 16 + g * 4 + e, rel = t - c;
                    // a tree has at most 64 candidates (rel < 64 below the limit); a chain's mask is all ones.  Written without
                    // short-circuit branches (plain selects on every lane): the branchy form of this test was miscompiled here
                    const uint32_t word = (rel & 32) ? anc_hi : anc_lo;
                    const uint32_t on_path = (word >> (rel & 31)) & 1u;
                    const bool seen = (t < limit) & ((rel < 0) | (on_path != 0u));
                    sc[kb * 4 + e] = seen ? sc[kb * 4 + e] : kMaskedRaw;
                }
        }
        float tmax = sc[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, sc[e]);
        tmax = four_rows_max(tmax) * scale;       // scale > 0: the maximum of the scaled scores
        if (__any(tmax > m_run + kMaxSlack)) {            // lazy reference maximum, as in the kernel above
            const float m_new = fmaxf(m_run, tmax);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) o[dt] *= alpha;
        }
        float pr[8], psum = 0.0f;
        const float neg_m = -m_run;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // a masked score is hugely negative: its exponential is 0 unless the row has seen nothing at all
            // (m_run == kNegBig), and such a row is masked by the comparison
            pr[e] = __builtin_amdgcn_exp2f(fmaf(sc[e], scale, neg_m));
            if (need_mask) pr[e] = (sc[e] > 0.5f * kMaskedRaw) ? pr[e] : 0.0f;
            psum += pr[e];
        }
        l_run += psum;
        const u32x4 pw = u32x4{pack_bf16x2(pr[0], pr[1]), pack_bf16x2(pr[2], pr[3]), pack_bf16x2(pr[4], pr[5]), pack_bf16x2(pr[6], pr[7])};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
        // ---- O^T += V^T P^T (transposing LDS read, as above) ----
        {
            const int vrow = 4 * g + (l16 >> 2);
            const unsigned char* v0 = sV + vrow * kRowBytes + 8 * (l16 & 3);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                const int off = (dt ^ (vrow & 7)) << 5;
                const s16x4 lo = lds_read_tr(v0 + off);
                const s16x4 hi = lds_read_tr(v0 + 16 * kRowBytes + off);
                struct { s16x4 a, b; } pair = {lo, hi};
                o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pair), pf, o[dt], 0, 0, 0);
            }
        }
    };
    for (int st0 = 0; st0 < nst; st0 += kRowsStages) {
        do_stage(std::integral_constant<int, 0>{}, st0);
        if (st0 + 1 < nst) do_stage(std::integral_constant<int, 1>{}, st0 + 1);
        if constexpr (kRowsStages > 2) {
            if (st0 + 2 < nst) do_stage(std::integral_constant<int, 2>{}, st0 + 2);
            if (st0 + 3 < nst) do_stage(std::integral_constant<int, 3>{}, st0 + 3);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // nothing of this wave is still landing in LDS
    if (bad_page && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_PAGE);

    // ---- the wave's own 16 rows: lane (l16, g) holds row l16, d = 16 dt + 4 g + e ----
    float l = l_run;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (!row_ok) return;
    if (FINAL) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            u32x2 packed;
            packed.x = pack_bf16x2(o[dt][0] * inv, o[dt][1] * inv);
            packed.y = pack_bf16x2(o[dt][2] * inv, o[dt][3] * inv);
            *reinterpret_cast<u32x2*>(p.out + rowhead * kD + dt * 16 + g * 4) = packed;
        }
        if (p.lse && g == 0) p.lse[rowhead] = (m_run + log2f(l)) * 0.6931471805599453f;
    } else {
        const size_t slot = part_base + ((size_t)qj * p.Hq + kvh * G + qg) * part_ns + split;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<f32x4*>(p.part_o + slot * kD + dt * 16 + g * 4) = o[dt];
        if (g == 0) { p.part_m[slot] = m_run; p.part_l[slot] = l; }
    }
}

// Balanced work list for ragged batches (one workgroup, B <= 1024 requests).  The fixed chunk_target of the
// host is sized for "every request as long as the bound"; when the real lengths are shorter or spread out,
// the chip is under-filled or unbalanced.  Here the chunk length is derived from the real total instead:
// the smallest c (a multiple of the workgroup step, min_chunk <= c <= max_chunk) with
// sum_i ceil(len_i / c) <= target_items, request i is cut into ceil(len_i / c) equal chunks, and the items are
// listed longest chunk first, so that workgroups dispatched in list order finish together.
// Launched with B rounded up to whole waves as the workgroup size.
__global__ __launch_bounds__(1024) void verify_attn_plan_kernel(AttnParams p, int B, int target_items, int step_keys,
                                                                int min_chunk, int max_chunk, int max_items,
                                                                int32_t* hdr, int32_t* req, int32_t* items)
{
    __shared__ __attribute__((aligned(16))) int s_key[1024];
    __shared__ int s_ns[1024], s_rows[1024], s_req[1024];
    __shared__ float s_redf[16];
    __shared__ int s_redi[2][16];
    __shared__ int s_scan_a[16], s_scan_b[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    int len = 0, n = 0, bad = 0;
    if (tid < B) {
        const int r0 = p.qo_indptr[tid];
        n = p.qo_indptr[tid + 1] - r0;
        const int c = p.seq_lens[tid];
        if (request_ok(r0, n, c, p)) len = c + n; else { bad = 1; n = 0; }
    }
    const int any_bad = __syncthreads_or(bad);
    // Total keys, as an fp32 estimate: it only seeds the chunk length, the loop below counts items exactly.
    float tf = (float)len;
    for (int d = 32; d >= 1; d >>= 1) tf += __shfl_xor(tf, d, 64);
    if (lane == 0) s_redf[wave] = tf;
    __syncthreads();
    float T = 0.0f;
    for (int w = 0; w < nw; ++w) T += s_redf[w];
    // chunk lengths are whole steps; the arithmetic is done in step units and in 32 bits / fp32 estimates
    // (64-bit integer division is a long software routine on this hardware)
    const int lo_steps = (min_chunk + step_keys - 1) / step_keys, hi_steps = max_chunk / step_keys;
    auto clamp_steps = [&](float x) -> int {
        int v = (int)ceilf(x);
        return v < lo_steps ? lo_steps : (v > hi_steps ? hi_steps : v);
    };
    int cs = clamp_steps(T / ((float)target_items * (float)step_keys));
    int c = cs * step_keys;
#pragma unroll 1
    for (int it = 0; it < 8; ++it) {
        int cnt = len ? (len + c - 1) / c : 0;
        for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
        if (lane == 0) s_redi[it & 1][wave] = cnt;        // two buffers: the next iteration writes the other one
        __syncthreads();
        int N = 0;
        for (int w = 0; w < nw; ++w) N += s_redi[it & 1][w];
        if (N <= target_items || cs >= hi_steps) break;
        const int cs2 = clamp_steps((float)cs * (float)N / (float)target_items);
        cs = cs2 > cs ? cs2 : cs + 1;
        c = cs * step_keys;
    }
    const int ns = len ? (len + c - 1) / c : 0;
    const int key = ns ? (len + ns - 1) / ns : 0;          // keys per chunk of this request
    // position in the list: requests ordered by chunk length, longest first (ties: request order).  Chunk
    // length (<= max_chunk < 2^21) and reversed request index are packed into one word, so that a position
    // costs one comparison per other request; 64 words are fetched per round before any is used.
    const uint32_t mine = ((uint32_t)key << 10) | (uint32_t)(1023 - tid);
    s_key[tid] = tid < B ? (int)mine : 0;
    __syncthreads();
    int rank = 0;
    if (tid < B) {
        const int kmax = (int)blockDim.x;
        for (int k0 = 0; k0 < kmax; k0 += 64) {
            u32x4 v[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = *reinterpret_cast<const u32x4*>(&s_key[k0 + 4 * j]);
#pragma unroll
            for (int j = 0; j < 16; ++j)
                rank += (int)(v[j].x > mine) + (int)(v[j].y > mine) + (int)(v[j].z > mine) + (int)(v[j].w > mine);
        }
    }
    __syncthreads();
    if (tid < B) { s_ns[rank] = ns; s_rows[rank] = ns * n; s_req[rank] = tid; }
    __syncthreads();
    // exclusive prefix sums over the ordered requests: items before, partial rows before
    int a = tid < B ? s_ns[tid] : 0, b = tid < B ? s_rows[tid] : 0;
    int ia = a, ib = b;
    for (int d = 1; d < 64; d <<= 1) {
        const int ua = __shfl_up(ia, d, 64), ub = __shfl_up(ib, d, 64);
        if (lane >= d) { ia += ua; ib += ub; }
    }
    if (lane == 63) { s_scan_a[wave] = ia; s_scan_b[wave] = ib; }
    __syncthreads();
    int base_a = 0, base_b = 0;
    for (int w = 0; w < wave; ++w) { base_a += s_scan_a[w]; base_b += s_scan_b[w]; }
    const int item0 = base_a + ia - a, row0 = base_b + ib - b;
    if (tid < B) {
        const int rq = s_req[tid];
        const int pb = row0 * p.Hq;                      // first partial slot of the request
        reinterpret_cast<u32x2*>(req)[rq] = u32x2{(uint32_t)a, (uint32_t)pb};
        for (int sp = 0; sp < a; ++sp)
            if (item0 + sp < max_items)
                reinterpret_cast<u32x4*>(items)[item0 + sp] = u32x4{(uint32_t)rq, (uint32_t)sp, (uint32_t)a, (uint32_t)pb};
    }
    if (tid == (int)blockDim.x - 1) {
        const int total = item0 + a;
        hdr[0] = total < max_items ? total : max_items;
        hdr[1] = c;
    }
    if (tid == 0 && any_bad && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_LENGTH);
}

// Merge the split partials of one (row, head) and write bf16 (and lse).  256 threads: lane group q = tid/32
// takes splits q, q+8, ..., thread t%32 four consecutive d; the 8 groups are then summed in group order, so
// the result does not depend on timing.
__global__ __launch_bounds__(256) void verify_attn_combine_kernel(AttnParams p, int B)
{
    __shared__ float s_num[8][kD];
    __shared__ float s_den[8];
    const int row = blockIdx.x, hq = blockIdx.y, tid = threadIdx.x, grp = tid >> 5, d4 = (tid & 31) * 4;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (p.qo_indptr[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int i = lo;
    const int n = p.qo_indptr[i + 1] - p.qo_indptr[i], c = p.seq_lens[i];
    if (!request_ok(p.qo_indptr[i], n, c, p) || row >= p.qo_indptr[i + 1]) return;
    const int len = c + n;
    const int ns = p.plan_req ? p.plan_req[2 * i] : (len + p.chunk_target - 1) / p.chunk_target;
    const size_t unit = p.plan_req ? (size_t)p.plan_req[2 * i + 1] + ((size_t)(row - p.qo_indptr[i]) * p.Hq + hq) * ns
                                   : ((size_t)row * p.Hq + hq) * p.splits;
    float mx = kNegBig;
    for (int s = 0; s < ns; ++s) mx = fmaxf(mx, p.part_m[unit + s]);
    f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
    float den = 0.0f;
    for (int s = grp; s < ns; s += 8) {
        const float w = exp2f(p.part_m[unit + s] - mx);
        num += w * *reinterpret_cast<const f32x4*>(p.part_o + (unit + s) * kD + d4);
        den += w * p.part_l[unit + s];
    }
    *reinterpret_cast<f32x4*>(&s_num[grp][d4]) = num;
    if ((tid & 31) == 0) s_den[grp] = den;
    __syncthreads();
    if (tid < kD) {
        float a = 0.0f, dsum = 0.0f;
#pragma unroll
        for (int q = 0; q < 8; ++q) { a += s_num[q][tid]; dsum += s_den[q]; }
        p.out[((size_t)row * p.Hq + hq) * kD + tid] = (uint16_t)f32_to_bf16_bits(a / dsum);
        if (p.lse && tid == 0) p.lse[(size_t)row * p.Hq + hq] = (mx + log2f(dsum)) * 0.6931471805599453f;
    }
}

// The same merge for requests cut into few pieces: one workgroup per candidate row, lane group q = tid/32 takes
// heads q, q+8, ... and walks the splits of its (row, head) in order; 8x fewer, fuller workgroups than above.
__global__ __launch_bounds__(256) void verify_attn_combine_rows_kernel(AttnParams p, int B)
{
    const int row = blockIdx.x, tid = threadIdx.x, grp = tid >> 5, d4 = (tid & 31) * 4;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (p.qo_indptr[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int i = lo;
    const int n = p.qo_indptr[i + 1] - p.qo_indptr[i], c = p.seq_lens[i];
    if (!request_ok(p.qo_indptr[i], n, c, p) || row >= p.qo_indptr[i + 1]) return;
    const int len = c + n;
    const int ns = p.plan_req ? p.plan_req[2 * i] : (len + p.chunk_target - 1) / p.chunk_target;
    for (int hq = grp; hq < p.Hq; hq += 8) {
        const size_t unit = p.plan_req ? (size_t)p.plan_req[2 * i + 1] + ((size_t)(row - p.qo_indptr[i]) * p.Hq + hq) * ns
                                       : ((size_t)row * p.Hq + hq) * p.splits;
        float mx = kNegBig;
        for (int s = 0; s < ns; ++s) mx = fmaxf(mx, p.part_m[unit + s]);
        f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
        float den = 0.0f;
        for (int s = 0; s < ns; ++s) {
            const float w = exp2f(p.part_m[unit + s] - mx);
            num += w * *reinterpret_cast<const f32x4*>(p.part_o + (unit + s) * kD + d4);
            den += w * p.part_l[unit + s];
        }
        const float inv = 1.0f / den;
        u32x2 packed;
        packed.x = pack_bf16x2(num.x * inv, num.y * inv);
        packed.y = pack_bf16x2(num.z * inv, num.w * inv);
        *reinterpret_cast<u32x2*>(p.out + ((size_t)row * p.Hq + hq) * kD + d4) = packed;
        if (p.lse && (tid & 31) == 0) p.lse[(size_t)row * p.Hq + hq] = (mx + log2f(den)) * 0.6931471805599453f;
    }
}

Tunable g_attn_chunk_override{0};

// Keys per kv split.  A split costs a prologue (Q to LDS), an epilogue (cross-wave merge) and a partial
// that the merge kernel re-reads, so requests are only split when there are too few (request, kv head)
// units to fill the chip or when they are long enough for the length spread to unbalance it.
static int attn_chunk_target(int B, int Hkv, int max_kv_len, int step_keys, int wgs_per_cu)
{
    long target;
    const int forced = g_attn_chunk_override;
    if (forced > 0) {
        target = forced;
    } else {
        // about one workgroup per CU when every request is as long as the bound (measured best on MI355X for
        // B=8 x 64k, B=64 x 4k and B=256 x 32k lognormal alike); shorter requests simply get fewer splits
        const long units = (long)B * Hkv, cus = device_cu_count();
        target = units * (long)max_kv_len / (cus * wgs_per_cu);
        if (target < 512) target = 512;
        if (target > 4096) target = 4096;
        if (target >= max_kv_len) target = max_kv_len;             // nobody is split: no partials, no merge kernel
    }
    if (target > 8192) target = 8192;                             // page ids of a chunk live in LDS (2 KB)
    return (int)((target + step_keys - 1) / step_keys * step_keys);
}

Tunable g_attn_nr3_waves{8};  // benchmark hook: waves per workgroup when a request has 3 row tiles (8, or 4 with two K/V buffers each)
static int attn_waves(int NR) { return NR <= 2 || (NR == 3 && g_attn_nr3_waves == 8) ? 8 : 4; }      // 8 waves need <= 256 registers per lane

Tunable g_attn_rows{0};       // benchmark hook: row-split kernel: 0 = automatic (4..8 row tiles), 1 = off, 2 = also for 2..3 row tiles
static int attn_rows_min_tiles() { const int v = g_attn_rows; return v == 1 ? 9 : (v == 2 ? 2 : 4); }
// workgroups of one CU the fixed chunk is sized for: the row-split kernel keeps three resident, the others one
static int attn_wgs_per_cu(int NR) { return NR >= attn_rows_min_tiles() ? 3 : 1; }

// Balanced work list (verify_attn_plan_kernel): used when requests are long enough for a few microseconds of
// planning to pay, numerous enough for their length spread to matter, and the fixed chunk would split them anyway.
Tunable g_attn_plan{0};          // benchmark hook: 0 = automatic, 1 = always (B <= 1024), 2 = never
Tunable g_attn_plan_waves{0};    // benchmark hook: work items per CU the plan aims at, 0 = automatic
constexpr int kPlanMinChunk = 512, kPlanMaxChunk = 8192;

struct AttnPlanCfg {
    bool on;
    int target_items, max_items, step_keys;
    size_t hdr_bytes, req_bytes, items_bytes, slots;
};

static AttnPlanCfg attn_plan_cfg(int B, int Hq, int Hkv, int max_kv_len, int max_q_len, int NR, int chunk_target)
{
    AttnPlanCfg c{};
    c.step_keys = attn_waves(NR) * 32;
    const bool splits_anyway = chunk_target < max_kv_len;
    const long cus = device_cu_count();
    // Pays when many requests of unknown, possibly very different lengths share the chip (measured on MI355X,
    // 256 requests of 256..32768 keys: 264 -> 213 us).  A few long requests are cut finely by the fixed chunk
    // anyway and run at the memory system's rate either way (8 x 32k..64k: 52 us without, 57 with the list).
    c.on = B <= 1024 && g_attn_plan != 2 &&
           (g_attn_plan == 1 || (splits_anyway && max_kv_len >= 8192 && (long)B * Hkv * 4 >= cus));
    // one workgroup is resident per CU (LDS): few requests are cut to exactly one round of equal items,
    // many requests to about two rounds, which the longest-first order packs
    const int plan_waves = g_attn_plan_waves;
    const int per_cu = plan_waves > 0 ? plan_waves : ((long)B * Hkv * 2 <= cus ? 1 : 2);
    long t = cus * per_cu / Hkv;
    if (t < 1) t = 1;
    c.target_items = (int)t;
    const long by_cap = (long)B * ((max_kv_len + kPlanMaxChunk - 1) / kPlanMaxChunk);
    const long mi = t + B > by_cap ? t + B : by_cap;
    c.max_items = (int)mi;
    c.hdr_bytes = 256;
    c.req_bytes = round_up((size_t)B * 8, 256);
    c.items_bytes = round_up((size_t)mi * 16, 256);
    c.slots = (size_t)mi * max_q_len * Hq;
    return c;
}

static size_t attn_smem_bytes(int NR, int NW, int NBUF, int chunk_keys)
{
    const size_t tiles = (size_t)NW * NBUF * kWaveLds + (size_t)NR * 16 * kRowBytes + (size_t)(chunk_keys / kP + 1) * 4 + 64 * 4 + 8 + (size_t)NR * 16 * 8;
    const size_t epi = (size_t)(2 * NW * NR * 16 + 2 * NR * 16 + NW * NR * 16 * kRedPitch) * sizeof(float);
    return tiles > epi ? tiles : epi;
}

template <int NR, int NW, int NBUF, bool FINAL>
static int launch_attn_one(const AttnParams& p, dim3 grid, hipStream_t s)
{
    const size_t smem = attn_smem_bytes(NR, NW, NBUF, p.chunk_target < p.max_kv_len ? p.chunk_target : p.max_kv_len);
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&verify_attn_kernel<NR, NW, NBUF, FINAL>), smem, granted,
                                    "spec_verify_attn")) return rc;
    hipLaunchKernelGGL((verify_attn_kernel<NR, NW, NBUF, FINAL>), grid, dim3(NW * 64), smem, s, p);
    return SPEC_OK;
}

Tunable g_attn_rows_ring{0};  // benchmark hook: K/V stages per workgroup of the row-split kernel, 2 or 4; 0 = automatic

static size_t attn_rows_smem_bytes(int chunk_keys, int ring)
{
    return (size_t)ring * kRowsStageBytes + (size_t)(chunk_keys / kP + 1) * 4 + 64 * 4 + 8 + 8 * 16 * 8;
}

template <int NW, bool FINAL, int RING>
static int launch_attn_rows_ring(const AttnParams& p, dim3 grid, hipStream_t s)
{
    const size_t smem = attn_rows_smem_bytes(p.chunk_target < p.max_kv_len ? p.chunk_target : p.max_kv_len, RING);
    static LdsGrantTable granted = {};
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(&verify_attn_rows_kernel<NW, FINAL, RING>), smem, granted,
                                    "spec_verify_attn")) return rc;
    hipLaunchKernelGGL((verify_attn_rows_kernel<NW, FINAL, RING>), grid, dim3(NW * 64), smem, s, p);
    return SPEC_OK;
}

template <int NW, bool FINAL>
static int launch_attn_rows(const AttnParams& p, dim3 grid, hipStream_t s)
{
    if (g_attn_rows_ring == 4) return launch_attn_rows_ring<NW, FINAL, 4>(p, grid, s);
    return launch_attn_rows_ring<NW, FINAL, 2>(p, grid, s);
}

// (the row-split kernel folds the scale into its exponentials, which needs a positive, finite scale)
static bool attn_uses_rows_kernel(int NR, float scale_log2e) { return NR >= attn_rows_min_tiles() && scale_log2e > 1e-30f && scale_log2e < 1e30f; }

template <int NR>
static int launch_attn(const AttnParams& p, dim3 grid, hipStream_t s)
{
    if constexpr (NR >= 2) {
        if (attn_uses_rows_kernel(NR, p.scale_log2e))
            return p.splits == 1 ? launch_attn_rows<NR, true>(p, grid, s) : launch_attn_rows<NR, false>(p, grid, s);
    }
    // up to 48 query rows: 8 waves (two per SIMD hide each other's loads, one K/V buffer per wave; with 3 row tiles
    // 238 registers, and 3-4 % faster than 4 waves on 32-64k contexts);
    // more rows need > 256 registers per lane: 4 waves, each double-buffering its own pages
    if constexpr (NR == 3) {
        if (g_attn_nr3_waves != 8)
            return p.splits == 1 ? launch_attn_one<NR, 4, 2, true>(p, grid, s) : launch_attn_one<NR, 4, 2, false>(p, grid, s);
    }
    constexpr int NW = NR <= 3 ? 8 : 4;
    constexpr int NBUF = (NR <= 3 || NR >= 7) ? 1 : 2;   // 7-8 row tiles leave no LDS for a second buffer
    return p.splits == 1 ? launch_attn_one<NR, NW, NBUF, true>(p, grid, s) : launch_attn_one<NR, NW, NBUF, false>(p, grid, s);
}

}  // namespace specv

extern "C" size_t spec_verify_attn_workspace_bytes(int B, int M, int Hq, int Hkv, int D, int max_kv_len, int max_q_len)
{
    using namespace specv;
    (void)D;
    if (B <= 0 || M <= 0 || Hq <= 0 || Hkv <= 0 || max_kv_len <= 0 || Hq % Hkv != 0) return 0;
    const int G = Hq / Hkv;
    const int NR = (G * (max_q_len > 0 ? max_q_len : 1) + 15) / 16;
    const int ct = attn_chunk_target(B, Hkv, max_kv_len, attn_waves(NR) * 32, attn_wgs_per_cu(NR));
    const size_t splits = (size_t)(max_kv_len + ct - 1) / ct;
    const size_t units = (size_t)M * Hq * splits;
    const size_t fixed = round_up(units * kD * 4, 256) + 2 * round_up(units * 4, 256);
    // the work-list mode has its own layout; the caller sizes the buffer before the mode is chosen
    const AttnPlanCfg pc = attn_plan_cfg(B, Hq, Hkv, max_kv_len, max_q_len > 0 ? max_q_len : 1, NR, ct);
    const size_t planned = pc.hdr_bytes + pc.req_bytes + pc.items_bytes + round_up(pc.slots * kD * 4, 256) + 2 * round_up(pc.slots * 4, 256);
    return (B <= 1024 && planned > fixed) ? planned : fixed;
}

extern "C" int spec_verify_attn(const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* page_table, int max_pages_per_seq, int num_pages,
                                const int32_t* seq_lens, const int32_t* qo_indptr, void* out, float* lse,
                                int B, int M, int Hq, int Hkv, int D, int page_size,
                                int max_kv_len, int max_q_len, float scale, int32_t* status_flags,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    return spec_verify_attn_tree(q, k_cache, v_cache, page_table, max_pages_per_seq, num_pages, seq_lens, qo_indptr,
                                 nullptr, out, lse, B, M, Hq, Hkv, D, page_size, max_kv_len, max_q_len, scale,
                                 status_flags, workspace, workspace_bytes, stream);
}

extern "C" int spec_verify_attn_tree(const void* q, const void* k_cache, const void* v_cache,
                                     const int32_t* page_table, int max_pages_per_seq, int num_pages,
                                     const int32_t* seq_lens, const int32_t* qo_indptr, const int32_t* parent,
                                     void* out, float* lse,
                                     int B, int M, int Hq, int Hkv, int D, int page_size,
                                     int max_kv_len, int max_q_len, float scale, int32_t* status_flags,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace specv;
    if (parent && max_q_len > 64)
        return fail(SPEC_ESHAPE, "spec_verify_attn_tree: max_q_len=%d, a tree has at most 64 rows", max_q_len);
    if (B == 0 || M == 0) return SPEC_OK;
    if (!q || !k_cache || !v_cache || !page_table || !seq_lens || !qo_indptr || !out)
        return fail(SPEC_EINVAL, "spec_verify_attn: NULL pointer argument");
    if (B < 0 || M < 0 || Hq <= 0 || Hkv <= 0 || max_pages_per_seq <= 0 || num_pages <= 0 || max_kv_len <= 0 || max_q_len <= 0)
        return fail(SPEC_EINVAL, "spec_verify_attn: non-positive size");
    if (D != kD || page_size != kP)
        return fail(SPEC_ESHAPE, "spec_verify_attn: built for D=128, page_size=16 (got D=%d page_size=%d)", D, page_size);
    if (Hq % Hkv != 0) return fail(SPEC_ESHAPE, "spec_verify_attn: Hq=%d is not a multiple of Hkv=%d", Hq, Hkv);
    const int G = Hq / Hkv;
    const int NR = (G * max_q_len + 15) / 16;
    if (NR > 8)
        return fail(SPEC_ESHAPE, "spec_verify_attn: (Hq/Hkv)*max_q_len = %d rows per kv head, at most 128", G * max_q_len);
    if ((long)max_pages_per_seq * kP < max_kv_len)
        return fail(SPEC_EINVAL, "spec_verify_attn: page table of %d pages cannot hold max_kv_len=%d", max_pages_per_seq, max_kv_len);
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16))
        return fail(SPEC_EINVAL, "spec_verify_attn: q and the caches must be 16-byte aligned");
    if (B > 65535 || Hkv > 65535 || M > 2147483647 / Hq) return fail(SPEC_ESHAPE, "spec_verify_attn: B, Hkv or M beyond the launch grid");
    const size_t need = spec_verify_attn_workspace_bytes(B, M, Hq, Hkv, D, max_kv_len, max_q_len);
    if (!workspace || !aligned(workspace, 256))
        return fail(SPEC_EINVAL, "spec_verify_attn: workspace is NULL or not 256-byte aligned");
    if (workspace_bytes < need)
        return fail(SPEC_EWORKSPACE, "spec_verify_attn: workspace %zu bytes, need %zu", workspace_bytes, need);

    AttnParams p;
    p.q = (const uint16_t*)q; p.k_cache = (const uint16_t*)k_cache; p.v_cache = (const uint16_t*)v_cache;
    p.page_table = page_table; p.seq_lens = seq_lens; p.qo_indptr = qo_indptr;
    p.status_flags = status_flags;
    p.max_pages = max_pages_per_seq; p.num_pages = num_pages; p.Hq = Hq; p.Hkv = Hkv; p.G = G;
    p.M = M; p.max_kv_len = max_kv_len; p.max_q_len = max_q_len;
    p.chunk_target = attn_chunk_target(B, Hkv, max_kv_len, attn_waves(NR) * 32, attn_wgs_per_cu(NR));
    p.out = (uint16_t*)out; p.lse = lse;
    p.splits = (max_kv_len + p.chunk_target - 1) / p.chunk_target;
    p.scale_log2e = scale * 1.4426950408889634f;
    p.plan_hdr = nullptr; p.plan_req = nullptr; p.plan_items = nullptr;
    p.parent = parent;
    hipStream_t s = (hipStream_t)stream;
    char* ws = (char*)workspace;
    const AttnPlanCfg pc = attn_plan_cfg(B, Hq, Hkv, max_kv_len, max_q_len, NR, p.chunk_target);
    dim3 grid(p.splits, Hkv, B);
    if (pc.on) {
        if (pc.slots * kD > 2147483647u || (size_t)pc.max_items > 2147483647u)
            return fail(SPEC_ESHAPE, "spec_verify_attn: work list beyond 32-bit slots");
        int32_t* hdr = (int32_t*)ws;
        int32_t* req = (int32_t*)(ws + pc.hdr_bytes);
        int32_t* items = (int32_t*)(ws + pc.hdr_bytes + pc.req_bytes);
        char* parts = ws + pc.hdr_bytes + pc.req_bytes + pc.items_bytes;
        p.part_o = (float*)parts;
        p.part_m = (float*)(parts + round_up(pc.slots * kD * 4, 256));
        p.part_l = (float*)(parts + round_up(pc.slots * kD * 4, 256) + round_up(pc.slots * 4, 256));
        hipLaunchKernelGGL(verify_attn_plan_kernel, dim3(1), dim3((B + 63) / 64 * 64), 0, s, p, B, pc.target_items, pc.step_keys,
                           kPlanMinChunk, kPlanMaxChunk, pc.max_items, hdr, req, items);
        int prc = check_launch("spec_verify_attn (plan)");
        if (prc != SPEC_OK) return prc;
        p.plan_hdr = hdr; p.plan_req = req; p.plan_items = items;
        p.chunk_target = kPlanMaxChunk;                   // sizes the page-id staging area in LDS
        p.splits = 2;                                     // "somebody is split": partials + merge kernel
        grid = dim3(pc.max_items, Hkv, 1);
    } else {
        const size_t units = (size_t)M * Hq * p.splits;
        p.part_o = (float*)ws;
        p.part_m = (float*)(ws + round_up(units * kD * 4, 256));
        p.part_l = (float*)(ws + round_up(units * kD * 4, 256) + round_up(units * 4, 256));
    }

    int rc = SPEC_OK;
    switch (NR) {
        case 1: rc = launch_attn<1>(p, grid, s); break;
        case 2: rc = launch_attn<2>(p, grid, s); break;
        case 3: rc = launch_attn<3>(p, grid, s); break;
        case 4: rc = launch_attn<4>(p, grid, s); break;
        case 5: rc = launch_attn<5>(p, grid, s); break;
        case 6: rc = launch_attn<6>(p, grid, s); break;
        case 7: rc = launch_attn<7>(p, grid, s); break;
        default: rc = launch_attn<8>(p, grid, s); break;
    }
    if (rc != SPEC_OK) return rc;
    rc = check_launch("spec_verify_attn");
    if (rc != SPEC_OK) return rc;
    if (p.splits == 1) return SPEC_OK;                    // the main kernel wrote the output itself
    // few pieces per request (typical count in work-list mode: items per request): one workgroup per row
    const bool few = pc.on ? (pc.target_items + B) / B <= 8 : p.splits <= 16;
    if (few) hipLaunchKernelGGL(verify_attn_combine_rows_kernel, dim3(M), dim3(256), 0, s, p, B);
    else hipLaunchKernelGGL(verify_attn_combine_kernel, dim3(M, Hq), dim3(256), 0, s, p, B);
    return check_launch("spec_verify_attn (combine)");
}
