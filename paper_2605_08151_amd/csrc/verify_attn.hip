// spec_verify_attn: ragged multi-query paged attention of the verification candidates (paper, Method:
// the target performs the verification pass on the merged batch Y_n; gamma_i = 0 rows are the padded
// parallel-mode candidates, i.e. ordinary decode).
//
// Work decomposition (HBM-bound: 512 bytes of K+V per key per kv head, 8..72 flop per byte):
//   grid = (kv split, kv head, request).  A workgroup of 4 waves streams one contiguous chunk of one
//   request's keys for one kv head in tiles of 128 keys (8 pages); wave w owns keys 32w..32w+31 of
//   every tile and all G * n_i query rows (query heads of the group x candidate positions), so no
//   K/V byte is read from LDS twice and waves only meet at the tile barriers.
//   Scores are computed transposed, S^T = K Q^T (v_mfma_f32_16x16x32_bf16, keys on the MFMA row
//   axis): a lane then holds 4 keys of ONE query row, the row maximum is an in-lane max plus two
//   cross-lane shuffles, and exp(S^T) is already the B operand of O^T += V^T P^T.  V is transposed on
//   its way into LDS ([key quad][d][4 keys]) so that the V^T operand is two 8-byte LDS reads.
//   Every chunk writes an unnormalised fp32 partial (O, running max, sum); a second kernel merges the
//   partials of a row in split order (deterministic) and writes bf16.
#include "common.h"

#include <cmath>

namespace specv {

constexpr int kD = 128;                      // head dimension
constexpr int kP = 16;                       // tokens per page
constexpr int kTile = 128;                   // keys per LDS tile
constexpr int kKPitch = 272;                 // bytes per K row in LDS (256 + 16: 16 rows hit 16 distinct bank groups)
constexpr int kVPitch = 1152;                // bytes per key quad in LDS ([128 d][4 keys] bf16 = 1024, + 128)
constexpr int kKBytes = kTile * kKPitch;     // 34816
constexpr int kVBytes = (kTile / 4) * kVPitch;   // 36864
constexpr int kRedPitch = 36;                // floats per row of the epilogue reduction buffer (32 + 4)
constexpr float kNegBig = -1.0e30f;          // "nothing seen yet" running maximum (log2 domain)

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
    unsigned char* sK = smem;
    unsigned char* sV = smem + kKBytes;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, i = blockIdx.z;

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

    // ---- query fragments (B operand of S^T = K Q^T): lane (row l16, k-group g) holds d = 32s+8g..+7 ----
    bf16x8 qf[NR][4];
    int limit[NR];                    // row sees key positions t < limit
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) {
        const int r = rt * 16 + l16;
        const bool live = r < R;
        const int j = live ? r / G : 0, gq = live ? r - j * G : 0;
        limit[rt] = live ? min(c + j + 1, kend) : 0;
        const uint16_t* src = p.q + ((size_t)(r0 + j) * p.Hq + kvh * G + gq) * kD + g * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u32x4 t = live ? *reinterpret_cast<const u32x4*>(src + s * 32) : u32x4{0, 0, 0, 0};
            qf[rt][s] = __builtin_bit_cast(bf16x8, t);
        }
    }

    f32x4 o[NR][8];
    float m_run[NR], l_run[NR];
#pragma unroll
    for (int rt = 0; rt < NR; ++rt) {
        m_run[rt] = kNegBig;
        l_run[rt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[rt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- global -> register staging of one tile: 8 x 16 B of K and 8 x 16 B of V per thread ----
    u32x4 kreg[8], vreg[8];
    int bad_page = 0;
    const int v_page_sub = tid >> 6;              // V: which of 4 pages of a pass this wave loads
    const int v_quad = (tid & 63) >> 4, v_chunk = tid & 15;
    auto fetch = [&](int tile_base) {
        const int page0 = tile_base / kP;
#pragma unroll
        for (int pg = 0; pg < 8; ++pg) {
            const int t0 = tile_base + pg * kP;
            u32x4 val = u32x4{0, 0, 0, 0};
            if (t0 < kend) {
                const int page = pt[page0 + pg];
                if (page >= 0 && page < p.num_pages)
                    val = *reinterpret_cast<const u32x4*>(p.k_cache + ((size_t)page * p.Hkv + kvh) * (kP * kD) + tid * 8);
                else
                    bad_page = 1;
            }
            kreg[pg] = val;
        }
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int pg = ps * 4 + v_page_sub;
            const int t0 = tile_base + pg * kP;
            int page = -1;
            if (t0 < kend) {
                page = pt[page0 + pg];
                if (page < 0 || page >= p.num_pages) page = -1;      // flagged by the K path
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int key = v_quad * 4 + kk;
                u32x4 val = u32x4{0, 0, 0, 0};
                if (page >= 0 && t0 + key < kend)                      // slots past the range may hold anything
                    val = *reinterpret_cast<const u32x4*>(p.v_cache + ((size_t)page * p.Hkv + kvh) * (kP * kD) + key * kD + v_chunk * 8);
                vreg[ps * 4 + kk] = val;
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int pg = 0; pg < 8; ++pg) {
            const int row = pg * kP + (tid >> 4);
            *reinterpret_cast<u32x4*>(sK + row * kKPitch + (tid & 15) * 16) = kreg[pg];
        }
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int quad = (ps * 4 + v_page_sub) * 4 + v_quad;
            unsigned char* dst = sV + quad * kVPitch + v_chunk * 64;
            const u32x4 a = vreg[ps * 4 + 0], b = vreg[ps * 4 + 1], cc = vreg[ps * 4 + 2], d = vreg[ps * 4 + 3];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                // word w holds d = 2w (low half) and 2w+1 (high half) of each of the 4 keys
                u32x4 outv;
                outv.x = (a[w] & 0xFFFFu) | (b[w] << 16);
                outv.y = (cc[w] & 0xFFFFu) | (d[w] << 16);
                outv.z = (a[w] >> 16) | (b[w] & 0xFFFF0000u);
                outv.w = (cc[w] >> 16) | (d[w] & 0xFFFF0000u);
                *reinterpret_cast<u32x4*>(dst + w * 16) = outv;
            }
        }
    };

    const int ntiles = (kend - kbeg + kTile - 1) / kTile;
    if (ntiles > 0) fetch(kbeg);
    for (int it = 0; it < ntiles; ++it) {
        const int tile_base = kbeg + it * kTile;
        __syncthreads();
        stash();
        __syncthreads();
        if (it + 1 < ntiles) fetch(tile_base + kTile);

        const int wbase = tile_base + wave * 32;           // first key of this wave's 32
        if (wbase < kend) {
            // ---- S^T = K Q^T for two 16-key blocks ----
            f32x4 st[2][NR];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                bf16x8 kf[4];
                const unsigned char* krow = sK + (wave * 32 + kb * 16 + l16) * kKPitch + g * 16;
#pragma unroll
                for (int s = 0; s < 4; ++s) kf[s] = *reinterpret_cast<const bf16x8*>(krow + s * 64);
#pragma unroll
                for (int rt = 0; rt < NR; ++rt) {
                    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s], qf[rt][s], acc, 0, 0, 0);
                    st[kb][rt] = acc;
                }
            }
            // ---- V^T fragments: lane (d = 16dt + l16, k-group g) holds keys 4g..4g+3 of both blocks ----
            bf16x8 vf[8];
            {
                const unsigned char* v0 = sV + (wave * 8 + g) * kVPitch + l16 * 8;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    const u32x2 lo = *reinterpret_cast<const u32x2*>(v0 + dt * 128);
                    const u32x2 hi = *reinterpret_cast<const u32x2*>(v0 + 4 * kVPitch + dt * 128);
                    vf[dt] = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
                }
            }
            const bool need_mask = wbase + 32 > min(c + 1, kend);
#pragma unroll
            for (int rt = 0; rt < NR; ++rt) {
                float sc[8];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) sc[kb * 4 + e] = st[kb][rt][e] * p.scale_log2e;
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
                const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf, o[rt][dt], 0, 0, 0);
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
    const size_t tiles = kKBytes + kVBytes;
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
