// spec_verify_attn: ragged multi-query paged attention of the verification candidates (paper, Method:
// the target performs the verification pass on the merged batch Y_n; gamma_i = 0 rows are the padded
// parallel-mode candidates, i.e. ordinary decode).
//
// Work decomposition (HBM-bound: 512 bytes of K+V per key per kv head, 8..72 flop per byte):
//   grid = (kv split, kv head, request).  A workgroup of 4 waves streams one contiguous chunk of one
//   request's keys for one kv head; wave w owns keys 32w..32w+31 of every 128-key step and all
//   G * n_i query rows (query heads of the group x candidate positions).  A wave copies ITS two pages
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

namespace specv {

constexpr int kD = 128;                      // head dimension
constexpr int kP = 16;                       // tokens per page
constexpr int kTile = 128;                   // keys per workgroup step (4 waves x 32)
constexpr int kRowBytes = kD * 2;            // one K or V row in LDS (unpadded, swizzled)
constexpr int kWaveLds = 2 * 32 * kRowBytes; // per wave: 32 K rows + 32 V rows = 16 KB
constexpr int kRedPitch = 36;                // floats per row of the epilogue reduction buffer (32 + 4)
constexpr float kNegBig = -1.0e30f;          // "nothing seen yet" running maximum (log2 domain)

typedef short s16x4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform)
__device__ inline void lds_dma16(const void* g, void* lds_base)
{
    __builtin_amdgcn_global_load_lds(g, (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

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
    float* part_o;      // [M*Hq, splits, 128]
    float* part_m;      // [M*Hq, splits]   running max, log2 domain
    float* part_l;      // [M*Hq, splits]
    int32_t* status_flags;
    int max_pages, num_pages, Hq, Hkv, G, M, max_kv_len, max_q_len, chunk_target, splits;
    float scale_log2e;
};

__device__ inline bool request_ok(int r0, int n, int c, const AttnParams& p)
{
    return n >= 1 && n <= p.max_q_len && r0 >= 0 && r0 + n <= p.M && c >= 0 && c + n <= p.max_kv_len;
}

template <int NR>
__global__ __launch_bounds__(256) void verify_attn_kernel(AttnParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, i = blockIdx.z;
    unsigned char* sK = smem + wave * kWaveLds;          // this wave's 32 K rows
    unsigned char* sV = sK + 32 * kRowBytes;             // and 32 V rows
    unsigned char* sQ = smem + 4 * kWaveLds;             // shared: NR*16 query rows

    const int r0 = p.qo_indptr[i], n = p.qo_indptr[i + 1] - r0, c = p.seq_lens[i];
    if (!request_ok(r0, n, c, p)) {
        if (split == 0 && kvh == 0 && tid == 0 && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_LENGTH);
        return;
    }
    const int len = c + n;
    const int ns = (len + p.chunk_target - 1) / p.chunk_target;
    if (split >= ns) return;
    const int chunk = (((len + ns - 1) / ns) + kP - 1) & ~(kP - 1);
    const int kbeg = split * chunk;
    const int kend = min(len, kbeg + chunk);
    const int G = p.G, R = G * n;
    const int32_t* pt = p.page_table + (size_t)i * p.max_pages;

    // ---- query rows -> LDS (row r = j*G + gq; 16-byte chunk ch of row r sits at position ch ^ (r & 15)) ----
    for (int idx = tid; idx < NR * 16 * 16; idx += 256) {
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

    int bad_page = 0;
    const int drow = lane >> 4, dpos = lane & 15;        // direct-load role: row within a group of 4, 16-byte position
    for (int wbase = kbeg + wave * 32; wbase < kend; wbase += kTile) {
        // ---- this wave's two pages, K and V, HBM -> LDS ----
        __builtin_amdgcn_s_waitcnt(0xC07F);               // lgkmcnt(0): the previous step's LDS reads have returned
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            const int t0 = wbase + pg * kP;
            if (t0 < kend) {
                const int page = pt[t0 / kP];
                if (page >= 0 && page < p.num_pages) {
                    const size_t base = ((size_t)page * p.Hkv + kvh) * (kP * kD);
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const int row = q4 * 4 + drow;     // slot in the page = key & 15
                        // K: chunk ch of a row is stored at position ch ^ (row & 15)
                        lds_dma16(p.k_cache + base + row * kD + ((dpos ^ row) << 3), sK + (pg * 16 + q4 * 4) * kRowBytes);
                        // V: 32-byte chunk c of a row is stored at position c ^ (row & 7)
                        const int src16 = ((((dpos >> 1) ^ (row & 7)) << 1) | (dpos & 1));
                        lds_dma16(p.v_cache + base + row * kD + (src16 << 3), sV + (pg * 16 + q4 * 4) * kRowBytes);
                    }
                } else {
                    bad_page = 1;
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): the pages have landed
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
        bf16x8 pf[NR];
#pragma unroll
        for (int rt = 0; rt < NR; ++rt) {
            bf16x8 qf[4];
#pragma unroll
            for (int s = 0; s < 4; ++s)
                qf[s] = *reinterpret_cast<const bf16x8*>(sQ + (rt * 16 + l16) * kRowBytes + (((s * 4 + g) ^ l16) << 4));
            float sc[8];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][s], qf[s], acc, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) sc[kb * 4 + e] = acc[e] * p.scale_log2e;
            }
            bool vis[8];
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        vis[kb * 4 + e] = (wbase + kb * 16 + g * 4 + e) < limit[rt];
                        if (!vis[kb * 4 + e]) sc[kb * 4 + e] = kNegBig;
                    }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) vis[e] = true;
            }
            float tmax = sc[0];
#pragma unroll
            for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, sc[e]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float m_new = fmaxf(m_run[rt], tmax);
            const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
            m_run[rt] = m_new;
            float pr[8], psum = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pr[e] = vis[e] ? __builtin_amdgcn_exp2f(sc[e] - m_new) : 0.0f;
                psum += pr[e];
            }
            l_run[rt] = l_run[rt] * alpha + psum;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[rt][dt] *= alpha;
            }
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
                for (int rt = 0; rt < NR; ++rt) o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[rt], o[rt][dt], 0, 0, 0);
            }
        }
    }
    if (bad_page && p.status_flags) atomicOr(p.status_flags, SPEC_FLAG_BAD_PAGE);

    // ---- merge the 4 waves: common maximum, then O in 4 slices of 32 d through LDS ----
    __syncthreads();                                      // tile buffers are free
    float* s_m = reinterpret_cast<float*>(smem);          // [4][NR*16]
    float* s_l = s_m + 4 * NR * 16;                       // [4][NR*16]
    float* s_red = s_l + 4 * NR * 16;                     // [4][NR*16][kRedPitch]
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
    float fscale[NR];
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) {
        float mx = kNegBig;
#pragma unroll
        for (int w = 0; w < 4; ++w) mx = fmaxf(mx, s_m[w * NR * 16 + rt * 16 + l16]);
        fscale[rt] = exp2f(m_run[rt] - mx);
    }
    // rows of this unit: r = j*G + gq  ->  global (row r0+j, head kvh*G+gq)
    const size_t unit_stride = (size_t)p.splits;
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
        for (int e = tid; e < R * 32; e += 256) {
            const int r = e >> 5, dl = e & 31;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < 4; ++w) sum += s_red[(size_t)(w * NR * 16 + r) * kRedPitch + dl];
            const int j = r / G, gq = r - j * G;
            const size_t unit = ((size_t)(r0 + j) * p.Hq + kvh * G + gq) * unit_stride + split;
            p.part_o[unit * kD + ds * 32 + dl] = sum;
        }
        __syncthreads();
    }
    for (int r = tid; r < R; r += 256) {
        float mx = kNegBig;
#pragma unroll
        for (int w = 0; w < 4; ++w) mx = fmaxf(mx, s_m[w * NR * 16 + r]);
        float l = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) l += s_l[w * NR * 16 + r] * exp2f(s_m[w * NR * 16 + r] - mx);
        const int j = r / G, gq = r - j * G;
        const size_t unit = ((size_t)(r0 + j) * p.Hq + kvh * G + gq) * unit_stride + split;
        p.part_m[unit] = mx;
        p.part_l[unit] = l;
    }
}

// Merge the split partials of one (row, head) in split order and write bf16 (and lse).
__global__ __launch_bounds__(128) void verify_attn_combine_kernel(AttnParams p, uint16_t* __restrict__ out, float* __restrict__ lse, int B)
{
    const int row = blockIdx.x, hq = blockIdx.y, d = threadIdx.x;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (p.qo_indptr[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int i = lo;
    const int n = p.qo_indptr[i + 1] - p.qo_indptr[i], c = p.seq_lens[i];
    if (!request_ok(p.qo_indptr[i], n, c, p) || row >= p.qo_indptr[i + 1]) return;
    const int len = c + n;
    const int ns = (len + p.chunk_target - 1) / p.chunk_target;
    const size_t unit = ((size_t)row * p.Hq + hq) * p.splits;
    float mx = kNegBig;
    for (int s = 0; s < ns; ++s) mx = fmaxf(mx, p.part_m[unit + s]);
    float num = 0.0f, den = 0.0f;
    for (int s = 0; s < ns; ++s) {
        const float w = exp2f(p.part_m[unit + s] - mx);
        num += w * p.part_o[(unit + s) * kD + d];
        den += w * p.part_l[unit + s];
    }
    const float val = num / den;
    out[((size_t)row * p.Hq + hq) * kD + d] = (uint16_t)f32_to_bf16_bits(val);
    if (lse && d == 0) lse[(size_t)row * p.Hq + hq] = (mx + log2f(den)) * 0.6931471805599453f;
}

int g_attn_chunk_override = 0;

static int attn_chunk_target(int B, int Hkv, int max_kv_len)
{
    if (g_attn_chunk_override > 0) return (g_attn_chunk_override + kTile - 1) / kTile * kTile;
    // aim at ~1024 workgroups when every request is as long as the bound, chunks of 256..4096 keys
    long target = (long)B * Hkv * (long)max_kv_len / 1024;
    if (target < 256) target = 256;
    if (target > 4096) target = 4096;
    return (int)((target + kTile - 1) / kTile * kTile);
}

static size_t attn_smem_bytes(int NR)
{
    const size_t tiles = 4 * (size_t)kWaveLds + (size_t)NR * 16 * kRowBytes;
    const size_t epi = (size_t)(2 * 4 * NR * 16 + 4 * NR * 16 * kRedPitch) * sizeof(float);
    return tiles > epi ? tiles : epi;
}

template <int NR>
static int launch_attn(const AttnParams& p, dim3 grid, hipStream_t s)
{
    const size_t smem = attn_smem_bytes(NR);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&verify_attn_kernel<NR>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return fail(SPEC_EHIP, "spec_verify_attn: cannot reserve %zu bytes of LDS", smem);
        configured = true;
    }
    hipLaunchKernelGGL(verify_attn_kernel<NR>, grid, dim3(256), smem, s, p);
    return SPEC_OK;
}

}  // namespace specv

extern "C" size_t spec_verify_attn_workspace_bytes(int B, int M, int Hq, int Hkv, int D, int max_kv_len, int max_q_len)
{
    using namespace specv;
    (void)D; (void)max_q_len;
    if (B <= 0 || M <= 0 || Hq <= 0 || Hkv <= 0 || max_kv_len <= 0) return 0;
    const int ct = attn_chunk_target(B, Hkv, max_kv_len);
    const size_t splits = (size_t)(max_kv_len + ct - 1) / ct;
    const size_t units = (size_t)M * Hq * splits;
    return round_up(units * kD * 4, 256) + 2 * round_up(units * 4, 256);
}

extern "C" int spec_verify_attn(const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* page_table, int max_pages_per_seq, int num_pages,
                                const int32_t* seq_lens, const int32_t* qo_indptr, void* out, float* lse,
                                int B, int M, int Hq, int Hkv, int D, int page_size,
                                int max_kv_len, int max_q_len, float scale, int32_t* status_flags,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace specv;
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
    p.chunk_target = attn_chunk_target(B, Hkv, max_kv_len);
    p.splits = (max_kv_len + p.chunk_target - 1) / p.chunk_target;
    p.scale_log2e = scale * 1.4426950408889634f;
    const size_t units = (size_t)M * Hq * p.splits;
    char* ws = (char*)workspace;
    p.part_o = (float*)ws;
    p.part_m = (float*)(ws + round_up(units * kD * 4, 256));
    p.part_l = (float*)(ws + round_up(units * kD * 4, 256) + round_up(units * 4, 256));

    hipStream_t s = (hipStream_t)stream;
    const dim3 grid(p.splits, Hkv, B);
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
    hipLaunchKernelGGL(verify_attn_combine_kernel, dim3(M, Hq), dim3(128), 0, s, p, (uint16_t*)out, lse, B);
    return check_launch("spec_verify_attn (combine)");
}
