// spec_accept: accepted length and bonus token per request (paper, Method, "Rollback-Based Mode
// Selection": after the verification pass the target performs rejection sampling and identifies the
// rollback set; Appendix "Target side": the target computes the accepted length L).
//
// Kernels, all HBM-bound scans or tiny per-request work:
//   1. row_stats      grid (segments, rows): per 4096-logit segment the max, the lowest argmax, a NaN
//                     flag and, for sampled requests, sum exp((l - max_seg)/T): in fp32 (an estimate good to
//                     2^-16, the default) or in fp64.
//   2. decide         one workgroup per request, one wave per row: merges the segments of each row; then every
//                     draft's test is evaluated at once (prefix match, or u*q < p with a Philox uniform) and the
//                     accepted length is the position of the first failure.  With fp32 sums the test is taken
//                     against both ends of the interval p must lie in; where they disagree the row is summed
//                     again in fp64 by the workgroup, so the outcome is always that of the fp64 definition.
//                     Greedy requests are finished here.
//   3a. bonus_z       (fp32 sums only) grid (segments, requests): fp64 segment sums of exp((l - m)/T) on the one
//                     row per sampled request that the bonus token is drawn from.
//   3. residual_sums  grid (segments, requests): for sampled requests, fp64 segment sums of the
//                     residual max(0, p - q) (and of p) on that row.
//   4. pick           one workgroup per request: inverse CDF over segment sums, then inside the segment.
// The fp64 exponential over all M rows made row_stats ALU-bound (103 us against 59 us for the same scan without it,
// B = 64, M = 576, V = 151936); only one row per request needs its normaliser to the last bit.
// Probabilities are formed in fp64 and rounded to fp32 before they are compared or subtracted, so the
// integer outputs do not depend on summation order beyond ~1e-16 relative.
#include "common.h"

namespace specv {

constexpr int kSeg = 4096;          // logits per segment
constexpr int kThreads = 256;
constexpr int kPerThread = kSeg / kThreads;   // 16
constexpr int kMaxRows = 64;        // gamma_max + 1 <= 64
constexpr int kPickLds = 512;       // segment sums staged in LDS by the pick kernel (V <= 2M entries)

// benchmark / test hook: 0 = automatic (on), 1 = on, 2 = off (fp64 sums over every row), 3 = on with an interval so wide
// that most tests are settled by the exact fallback
Tunable g_accept_filter{0};

struct AcceptWorkspace {
    float* seg_max;      // [M, nseg]
    int32_t* seg_arg;    // [M, nseg]
    int32_t* seg_bad;    // [M, nseg]
    double* seg_z;       // [M, nseg]
    double* res_sum;     // [B, nseg]
    double* p_sum;       // [B, nseg]
    double* job_m;       // [B]
    double* job_z;       // [B]
    float* job_u;        // [B]
    float* job_t;        // [B]
    int32_t* job_row;    // [B]  logits row the bonus is drawn from, -1 = nothing to draw
    int32_t* job_qrow;   // [B]  draft_probs row subtracted, -1 = none
    int32_t* job_onehot; // [B]  token of a one-hot drafter, -1 = none
    double* job_zseg;    // [B, nseg]  fp64 segment sums of exp((l - m)/T) on the bonus row (when the bulk sums are fp32)
};

static size_t carve(AcceptWorkspace* w, char* base, int B, int M, int nseg)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += round_up(bytes, 256); return p; };
    const size_t rs = (size_t)M * nseg, bs = (size_t)B * nseg;
    w->seg_z = (double*)take(rs * 8);
    w->res_sum = (double*)take(bs * 8);
    w->p_sum = (double*)take(bs * 8);
    w->job_zseg = (double*)take(bs * 8);
    w->job_m = (double*)take((size_t)B * 8);
    w->job_z = (double*)take((size_t)B * 8);
    w->seg_max = (float*)take(rs * 4);
    w->seg_arg = (int32_t*)take(rs * 4);
    w->seg_bad = (int32_t*)take(rs * 4);
    w->job_u = (float*)take((size_t)B * 4);
    w->job_t = (float*)take((size_t)B * 4);
    w->job_row = (int32_t*)take((size_t)B * 4);
    w->job_qrow = (int32_t*)take((size_t)B * 4);
    w->job_onehot = (int32_t*)take((size_t)B * 4);
    return off;
}

// ---- Philox4x32-10 (Salmon et al., SC'11), written for the device ----------------------------
__device__ inline float philox_uniform(uint64_t seed, uint32_t round, uint32_t j, uint32_t tag)
{
    uint32_t x0 = 0u, x1 = j, x2 = tag, x3 = round;
    uint32_t ka = (uint32_t)seed, kb = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, x0), lo0 = 0xD2511F53u * x0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, x2), lo1 = 0xCD9E8D57u * x2;
        const uint32_t y0 = hi1 ^ x1 ^ ka, y2 = hi0 ^ x3 ^ kb;
        x0 = y0; x1 = lo1; x2 = y2; x3 = lo0;
        ka += 0x9E3779B9u;
        kb += 0xBB67AE85u;
    }
    return (float)(x0 >> 8) * (1.0f / 16777216.0f);
}

// ---- reductions --------------------------------------------------------------------------------
__device__ inline void wave_max_arg(float& m, int& a)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float om = __shfl_xor(m, d, 64);
        const int oa = __shfl_xor(a, d, 64);
        if (om > m || (om == m && oa < a)) { m = om; a = oa; }
    }
}

__device__ inline double wave_sum(double x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

__device__ inline int find_request(const int32_t* __restrict__ qo_indptr, int B, int row)
{
    int lo = 0, hi = B - 1;            // largest i with qo_indptr[i] <= row
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (qo_indptr[mid] <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// loads the 16 logits this thread owns in its segment; out-of-range slots read as -inf
__device__ inline void load_strided(const float* __restrict__ row, int v0, int vend, bool vec, int tid, float (&x)[kPerThread])
{
#pragma unroll
    for (int it = 0; it < kPerThread / 4; ++it) {
        const int idx = v0 + (it * kThreads + tid) * 4;
        if (vec && idx + 3 < vend) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(row + idx);
            x[it * 4 + 0] = t.x; x[it * 4 + 1] = t.y; x[it * 4 + 2] = t.z; x[it * 4 + 3] = t.w;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) x[it * 4 + k] = (idx + k < vend) ? row[idx + k] : -INFINITY;
        }
    }
}

// ---- exp for the bulk sums ---------------------------------------------------------------------
// exp(x), x <= 0, for the ~V values per row that enter Z and the residual: x = (64 m + j) ln2/64 + r with
// |r| <= ln2/128, exp(x) = 2^m * 2^(j/64) * (1 + r + ... + r^5/120).  The 64 table values are correctly rounded;
// the reduction constant is split so that n * hi is exact.  Relative error <= 3.3e-16 (checked against 60-digit
// arithmetic on 2e5 arguments), about 20 issue slots instead of the ~46 of the library routine.  Single compared
// values (the accept test) still use the library exp.
__device__ const double kExp2Tbl[64] = {
    1.0, 1.0108892860517005, 1.0218971486541166, 1.0330248790212284,
    1.0442737824274138, 1.0556451783605572, 1.0671404006768237, 1.0787607977571199,
    1.0905077326652577, 1.102382583307841, 1.1143867425958924, 1.1265216186082418,
    1.1387886347566916, 1.1511892299529827, 1.1637248587775775, 1.1763969916502812,
    1.189207115002721, 1.202156731452703, 1.215247359980469, 1.22848053610687,
    1.241857812073484, 1.255380757024691, 1.2690509571917332, 1.2828700160787783,
    1.2968395546510096, 1.3109612115247644, 1.3252366431597413, 1.339667524053303,
    1.3542555469368927, 1.3690024229745905, 1.383909881963832, 1.3989796725383112,
    1.4142135623730951, 1.42961333839197, 1.4451808069770467, 1.460917794180647,
    1.4768261459394993, 1.4929077282912648, 1.5091644275934228, 1.5255981507445384,
    1.5422108254079407, 1.559004400237837, 1.5759808451078865, 1.593142151342267,
    1.6104903319492543, 1.6280274218573478, 1.645755478153965, 1.6636765803267364,
    1.681792830507429, 1.7001063537185235, 1.718619298122478, 1.7373338352737062,
    1.7562521603732995, 1.7753764925265212, 1.7947090750031072, 1.8142521755003989,
    1.8340080864093424, 1.8539791250833855, 1.8741676341103, 1.8945759815869656,
    1.9152065613971474, 1.9360617934922943, 1.9571441241754002, 1.978456026387951
};

__device__ inline void load_exp_table(double* s_tbl, int tid)
{
    if (tid < 64) s_tbl[tid] = kExp2Tbl[tid];
}

__device__ inline double exp_bulk(double x, const double* s_tbl)
{
    // Below -700 the true value (< 1e-304) cannot change a sum that holds a term >= 1 nor survive the
    // rounding of a probability to fp32, so the argument is clamped there: the result then stays a normal
    // number and 2^m can be applied by adding m to the exponent field.  -inf (a masked entry) ends here too.
    x = fmax(x, -700.0);
    const double kMagic = 6755399441055744.0;             // 1.5 * 2^52: the sum's low mantissa bits are rint(.)
    const double t = fma(x, 92.33248261689366, kMagic);   // 64 / ln 2
    const int n = __double2loint(t);
    const double nd = t - kMagic;
    double r = fma(nd, -0.01083042469326756, x);          // ln2/64, high part (21 trailing zero bits)
    r = fma(nd, -2.9815858269852933e-12, r);              // ln2/64, low part
    double q = fma(r, 1.0 / 120.0, 1.0 / 24.0);
    q = fma(r, q, 1.0 / 6.0);
    q = fma(r, q, 0.5);
    q = fma(r, q, 1.0);
    q = fma(r, q, 1.0);
    const double v = s_tbl[n & 63] * q;                   // in (0.99, 2.02)
    return __hiloint2double(__double2hiint(v) + ((n >> 6) << 20), __double2loint(v));
}

// ---- 1. per-segment statistics ---------------------------------------------------------------
constexpr int kSegPerWg = 1;        // consecutive segments one workgroup handles (all loads issued up front)

__global__ __launch_bounds__(kThreads) void accept_row_stats_kernel(
    const float* __restrict__ logits, const float* __restrict__ temperature,
    const int32_t* __restrict__ qo_indptr, int B, int V, int nseg, bool vec,
    AcceptWorkspace w, int32_t* __restrict__ stats, bool greedy_rows_covered, bool fp32_sums)
{
    __shared__ float s_m[kSegPerWg][kThreads / 64];
    __shared__ int s_a[kSegPerWg][kThreads / 64];
    __shared__ int s_bad[kSegPerWg][kThreads / 64];
    __shared__ double s_z[kSegPerWg][kThreads / 64];
    __shared__ double s_tbl[64];
    const int seg0 = blockIdx.x * kSegPerWg, row = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    load_exp_table(s_tbl, tid);                           // visible after the barrier below
    if (stats && blockIdx.x == 0 && row == 0 && tid < 4) stats[tid] = (tid == 2) ? B : 0;
    const float* lrow = logits + (size_t)row * V;
    float x[kSegPerWg][kPerThread];
#pragma unroll
    for (int q = 0; q < kSegPerWg; ++q) {
        const int v0 = (seg0 + q) * kSeg;
        load_strided(lrow, min(v0, V), min(V, v0 + kSeg), vec, tid, x[q]);      // past the row: all -inf
    }
    const float T = temperature ? temperature[find_request(qo_indptr, B, row)] : 0.0f;   // null: every request greedy
    if (greedy_rows_covered && T == 0.0f) return;         // the decision reads the LM head's block statistics instead
#pragma unroll
    for (int q = 0; q < kSegPerWg; ++q) {
        const int v0 = (seg0 + q) * kSeg;
        float m = -INFINITY;
        int arg = 0x7FFFFFFF, bad = 0;
#pragma unroll
        for (int it = 0; it < kPerThread / 4; ++it)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float xv = x[q][it * 4 + k];
                bad |= (xv != xv);
                if (xv > m) { m = xv; arg = v0 + (it * kThreads + tid) * 4 + k; }
            }
        wave_max_arg(m, arg);
        bad = __any(bad);
        if (lane == 0) { s_m[q][wave] = m; s_a[q][wave] = arg; s_bad[q][wave] = bad; }
    }
    __syncthreads();
    float bm[kSegPerWg];
    int ba[kSegPerWg], bb[kSegPerWg];
#pragma unroll
    for (int q = 0; q < kSegPerWg; ++q) {
        bm[q] = s_m[q][0]; ba[q] = s_a[q][0]; bb[q] = s_bad[q][0];
#pragma unroll
        for (int k = 1; k < kThreads / 64; ++k) {
            if (s_m[q][k] > bm[q] || (s_m[q][k] == bm[q] && s_a[q][k] < ba[q])) { bm[q] = s_m[q][k]; ba[q] = s_a[q][k]; }
            bb[q] |= s_bad[q][k];
        }
    }
    if (T > 0.0f) {
        const double inv_t = 1.0 / (double)T;
#pragma unroll
        for (int q = 0; q < kSegPerWg; ++q) {
            double z = 0.0;
            if (!bb[q] && bm[q] > -INFINITY && bm[q] < INFINITY) {
                if (fp32_sums) {
                    // An estimate for the interval test of the decision kernel, which asks for it within 2^-14 of the
                    // fp64 sum.  Per term: the exponent (l - max) * log2(e)/T carries three fp32 roundings (<= 1.8e-7
                    // relative, i.e. <= 1.24e-7 |a| relative in 2^a) and the hardware exponential one ulp, together
                    // <= 8.1e-6 for |a| <= 64; terms beyond add < 4096 * 2^-64 to a sum >= 1; sixteen fp32 additions
                    // per lane add <= 1e-6.  The partial sums are then carried in fp64.  Total < 2^-16.
                    const float c = (float)(1.4426950408889634 * inv_t), fm = bm[q];
                    float zf = 0.0f;
#pragma unroll
                    for (int k = 0; k < kPerThread; ++k) zf += __builtin_amdgcn_exp2f((x[q][k] - fm) * c);
                    z = (double)zf;
                } else {
                    const double dm = (double)bm[q];
#pragma unroll
                    for (int k = 0; k < kPerThread; ++k) z += exp_bulk(((double)x[q][k] - dm) * inv_t, s_tbl);
                }
            }
            z = wave_sum(z);
            if (lane == 0) s_z[q][wave] = z;
        }
        __syncthreads();
    }
    if (tid < kSegPerWg && seg0 + tid < nseg) {
        double z = 0.0;
        if (T > 0.0f)
            for (int k = 0; k < kThreads / 64; ++k) z += s_z[tid][k];
        // pick this thread's segment out of the register arrays without dynamic indexing
        float fm = bm[0]; int fa = ba[0], fb = bb[0];
#pragma unroll
        for (int q = 1; q < kSegPerWg; ++q) if (tid == q) { fm = bm[q]; fa = ba[q]; fb = bb[q]; }
        const size_t o = (size_t)row * nseg + seg0 + tid;
        w.seg_max[o] = fm; w.seg_arg[o] = fa; w.seg_bad[o] = fb; w.seg_z[o] = z;
    }
}

// Counter reset for batches in which row_stats is not launched at all.
__global__ void accept_reset_stats_kernel(int32_t* __restrict__ stats, int B)
{
    if (threadIdx.x < 4) stats[threadIdx.x] = (threadIdx.x == 2) ? B : 0;
}

// ---- 2. per-request decision -----------------------------------------------------------------
// Block summaries of the large-tile LM head (LmSummary in common.h), when the caller has them: per row and block of
// at most 64 entries the maximum and, for sampled rows, the fp32 sum of 2^((l - max) log2(e)/T); blk_span = {first entry,
// entries} per block.  With them no row of logits is scanned: a greedy row looks its argmax up inside the one block that
// holds the row maximum, a sampled row gets its estimated normaliser from the block sums.
struct AcceptSummary {
    const float* blk_max;
    const float* blk_sum;
    const int32_t* blk_span;
    int blocks;
};

constexpr int kDecideThreads = 1024;   // 16 waves: the rows of a request (gamma + 1 <= 16 in practice) are merged side by side

__global__ __launch_bounds__(kDecideThreads) void accept_decide_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ tokens, const float* __restrict__ draft_probs,
    const float* __restrict__ temperature, const uint64_t* __restrict__ seeds, uint32_t round,
    const int32_t* __restrict__ qo_indptr, int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens,
    uint8_t* __restrict__ rollback, int32_t* __restrict__ stats, int M, int V, int nseg, int gamma_max,
    AcceptWorkspace w, int32_t* __restrict__ status_flags,
    const float* __restrict__ blk_max, const int32_t* __restrict__ blk_arg, int nblk, float band, AcceptSummary sum)
{
    __shared__ double s_m[kMaxRows], s_z[kMaxRows];
    __shared__ int s_arg[kMaxRows], s_bad[kMaxRows];
    const int i = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, tid = threadIdx.x;
    const int r0 = qo_indptr[i], gamma = qo_indptr[i + 1] - r0 - 1;
    int32_t* emit = out_tokens + (size_t)i * (gamma_max + 1);
    for (int j = tid; j <= gamma_max; j += kDecideThreads) emit[j] = -1;
    if (tid == 0) { w.job_row[i] = -1; accept_len[i] = 0; if (rollback) rollback[i] = 0; }
    if (gamma < 0 || gamma > gamma_max || r0 < 0 || r0 + gamma + 1 > M) {
        if (tid == 0 && status_flags) atomicOr(status_flags, SPEC_FLAG_BAD_LENGTH);
        return;
    }
    const float T = temperature[i];
    const double Td = (double)T;
    const bool from_blocks = nblk > 0 && T == 0.0f;        // greedy: maxima the LM head left per vocabulary block
    for (int j = wave; j <= gamma; j += kDecideThreads / 64) {   // one wave per row
        const size_t base = (size_t)(r0 + j) * nseg;
        float m = -INFINITY;
        int arg = 0x7FFFFFFF, bad = 0;
        if (sum.blocks > 0) {
            const size_t bb = (size_t)(r0 + j) * sum.blocks;
            int mb = 0x7FFFFFFF;                          // lowest block that holds the row maximum
            for (int s0 = lane; s0 < sum.blocks; s0 += 64 * 8) {
                float sm[8];
                int cnt[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int s = s0 + 64 * u;
                    cnt[u] = s < sum.blocks ? sum.blk_span[2 * s + 1] : 0;
                    sm[u] = s < sum.blocks ? sum.blk_max[bb + s] : -INFINITY;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (cnt[u] <= 0) continue;            // a slot without entries: its records were never written
                    bad |= (sm[u] != sm[u]);
                    if (sm[u] > m) { m = sm[u]; mb = s0 + 64 * u; }     // (ascending s: ties keep the lower block)
                }
            }
            wave_max_arg(m, mb);
            bad = __any(bad) || !(m > -INFINITY && m < INFINITY);
            double z = 0.0;
            if (!bad && T == 0.0f) {
                const int first = sum.blk_span[2 * mb], count = sum.blk_span[2 * mb + 1];
                const float x = lane < count ? logits[(size_t)(r0 + j) * V + first + lane] : -INFINITY;
                const unsigned long long hit = __ballot(x == m);
                arg = first + (hit ? __ffsll((long long)hit) - 1 : 0);
            } else if (!bad) {
                // the block sums are fp32 estimates: rescaling them with the hardware exponential (another ~1e-5 at
                // most for exponents down to -64, nothing below) keeps the total inside the band of the interval test
                const float c = (float)(1.4426950408889634 / Td);
                for (int s0 = lane; s0 < sum.blocks; s0 += 64 * 8) {
                    float sm[8], sz[8];
                    int cnt[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int s = s0 + 64 * u;
                        cnt[u] = s < sum.blocks ? sum.blk_span[2 * s + 1] : 0;
                        sm[u] = s < sum.blocks ? sum.blk_max[bb + s] : -INFINITY;
                        sz[u] = s < sum.blocks ? sum.blk_sum[bb + s] : 0.0f;
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (cnt[u] > 0 && sm[u] > -INFINITY) z += (double)(sz[u] * __builtin_amdgcn_exp2f((sm[u] - m) * c));
                }
                z = wave_sum(z);
            }
            if (lane == 0) { s_m[j] = (double)m; s_z[j] = z; s_arg[j] = arg; s_bad[j] = bad; }
            continue;
        }
        if (from_blocks) {
            // ~V/128 blocks per row: eight loads in flight per lane, or the walk is one memory latency per 64 blocks
            const size_t bb = (size_t)(r0 + j) * nblk;
            for (int s0 = lane; s0 < nblk; s0 += 64 * 8) {
                float sm[8];
                int sa[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int s = s0 + 64 * u;
                    sm[u] = s < nblk ? blk_max[bb + s] : -INFINITY;
                    sa[u] = s < nblk ? blk_arg[bb + s] : 0x7FFFFFFF;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    bad |= (sm[u] != sm[u]);
                    if (sm[u] > m || (sm[u] == m && sa[u] < arg)) { m = sm[u]; arg = sa[u]; }
                }
            }
        } else
        for (int s = lane; s < nseg; s += 64) {
            const float sm = w.seg_max[base + s];
            const int sa = w.seg_arg[base + s];
            bad |= w.seg_bad[base + s];
            if (sm > m || (sm == m && sa < arg)) { m = sm; arg = sa; }
        }
        // (the first 64 segment sums are requested together with the maxima: one memory round trip for V <= 262144)
        const double z_first = (T > 0.0f && lane < nseg) ? w.seg_z[base + lane] : 0.0;
        const float m_first = lane < nseg ? w.seg_max[base + lane] : -INFINITY;
        wave_max_arg(m, arg);
        bad = __any(bad) || !(m > -INFINITY && m < INFINITY);
        double z = 0.0;
        if (T > 0.0f && !bad) {
            if (m_first > -INFINITY) z = z_first * exp(((double)m_first - (double)m) / Td);
            for (int s = lane + 64; s < nseg; s += 64) {
                const float sm = w.seg_max[base + s];
                if (sm > -INFINITY) z += w.seg_z[base + s] * exp(((double)sm - (double)m) / Td);
            }
            z = wave_sum(z);
        }
        if (lane == 0) { s_m[j] = (double)m; s_z[j] = z; s_arg[j] = arg; s_bad[j] = bad; }
    }
    // what the walk below needs per draft (token, its logit on the previous row, its draft probability) is
    // fetched by gamma threads at once: one memory round trip instead of one per draft
    __shared__ int s_tok[kMaxRows];
    __shared__ float s_logit[kMaxRows], s_qd[kMaxRows];
    if (tid >= 1 && tid <= gamma) {
        const int d = tokens[r0 + tid];
        const bool ok = d >= 0 && d < V;
        s_tok[tid] = d;
        s_logit[tid] = (ok && T > 0.0f) ? logits[(size_t)(r0 + tid - 1) * V + d] : 0.0f;
        s_qd[tid] = (ok && T > 0.0f && draft_probs) ? draft_probs[(size_t)(r0 - i + tid - 1) * V + d] : 1.0f;
    }
    __syncthreads();

    // Every wave evaluates the same tests on the same LDS data (so that the branches below are uniform for the whole
    // workgroup); wave 0 alone writes.  Lane j looks at row j (its logits usable?) and at draft j (1 <= j <= gamma <= 63):
    // every draft's test is evaluated at once, and the accepted length is the number of drafts before the first that fails.
    const bool w0 = wave == 0;
    const bool has_draft = lane >= 1 && lane <= gamma;
    const int d = has_draft ? s_tok[lane] : 0;
    int flags = 0;
    bool valid = (T >= 0.0f);
    if (T > 0.0f && seeds == nullptr) { valid = false; flags |= SPEC_FLAG_NO_SEED; }
    if (__any(lane <= gamma && s_bad[lane])) { valid = false; flags |= SPEC_FLAG_BAD_LOGITS; }
    if (__any(has_draft && (d < 0 || d >= V))) { valid = false; flags |= SPEC_FLAG_BAD_TOKEN; }
    if (!(T >= 0.0f)) flags |= SPEC_FLAG_BAD_LOGITS;
    if (!valid) {
        if (tid == 0) {
            if (rollback) rollback[i] = (uint8_t)(gamma > 0);
            if (stats) { if (gamma > 0) atomicAdd(stats + 0, 1); }
            if (status_flags && flags) atomicOr(status_flags, flags);
        }
        return;
    }
    int a, bonus = -1;
    if (T == 0.0f) {
        const unsigned long long miss = __ballot(has_draft && d != s_arg[lane - 1]);
        a = miss ? __ffsll((long long)miss) - 2 : gamma;  // bit j is the first mismatch: drafts 1..j-1 stand
        bonus = s_arg[a];
    } else {
        // Draft j stands iff fl32(u q) < fl32(e / Z), e = exp((l - m)/T), Z the fp64 sum over the row.  s_z holds Z itself
        // (band == 0) or an fp32-summed estimate within a relative `band` of it: the test is then taken against both ends
        // of the interval that fl32(e / Z) must lie in, and only where the two disagree is the row summed again in fp64,
        // by the whole workgroup.  The outcome is that of the exact test in every case.
        enum { kPass = 0, kFail = 1, kOpen = 2 };
        const uint64_t seed = seeds[i];
        int state = kPass;
        double e = 0.0;
        float x = 0.0f;
        if (has_draft) {
            e = exp(((double)s_logit[lane] - s_m[lane - 1]) / Td);
            const double zj = s_z[lane - 1];
            const float u = philox_uniform(seed, round, (uint32_t)lane, 0u);
            x = (float)((double)u * (double)s_qd[lane]);
            const float p_lo = (float)(e / (zj * (1.0 + (double)band))), p_hi = (float)(e / (zj * (1.0 - (double)band)));
            state = x < p_lo ? kPass : (x < p_hi ? kOpen : kFail);
        }
        __shared__ int s_need;
        __shared__ double s_exact, s_part[kDecideThreads / 64], s_tbl[64];
        bool table_loaded = false;
        for (;;) {
            const unsigned long long fails = __ballot(state == kFail), opens = __ballot(state == kOpen);
            const unsigned long long before_fail = fails ? ((fails & (0ull - fails)) - 1ull) : ~0ull;
            const unsigned long long undecided = opens & before_fail;     // open tests that the outcome depends on
            const int need = undecided ? __ffsll((long long)undecided) - 2 : -1;   // bit j: draft j is tested on row j-1
            if (need < 0) break;                          // (the same in every wave: same data, same arithmetic)
            if (!table_loaded) { load_exp_table(s_tbl, tid); table_loaded = true; __syncthreads(); }
            const float* lrow = logits + (size_t)(r0 + need) * V;
            const double mrow = s_m[need], inv_t = 1.0 / Td;
            double z = 0.0;
            for (int v = tid; v < V; v += kDecideThreads) z += exp_bulk(((double)lrow[v] - mrow) * inv_t, s_tbl);
            z = wave_sum(z);
            if (lane == 0) s_part[wave] = z;
            __syncthreads();
            if (tid == 0) {
                double t = 0.0;
                for (int k = 0; k < kDecideThreads / 64; ++k) t += s_part[k];
                s_exact = t; s_z[need] = t;
            }
            __syncthreads();
            if (lane == need + 1) state = x < (float)(e / s_exact) ? kPass : kFail;
            __syncthreads();                              // s_part and s_exact are free again
        }
        const unsigned long long fail_mask = __ballot(state == kFail);
        const int rejected_at = fail_mask ? __ffsll((long long)fail_mask) - 1 : 0;
        a = rejected_at ? rejected_at - 1 : gamma;
        if (tid == 0) {
            // the bonus is drawn on the row that rejected (from the residual) or on the last row (from the target itself)
            const int jr = rejected_at ? rejected_at - 1 : gamma;
            w.job_row[i] = r0 + jr;
            w.job_qrow[i] = (rejected_at && draft_probs) ? (r0 - i + jr) : -1;
            w.job_onehot[i] = (rejected_at && !draft_probs) ? s_tok[rejected_at] : -1;
            w.job_u[i] = philox_uniform(seed, round, (uint32_t)(rejected_at ? rejected_at : gamma + 1), 1u);
            w.job_m[i] = s_m[jr];
            w.job_z[i] = s_z[jr];                         // (an estimate when band > 0: the draw then sums the row itself)
            w.job_t[i] = T;
        }
    }
    if (!w0) return;
    // lane j writes slot j: the accepted drafts, then (greedy) the bonus; sampled requests get theirs from the draw
    if (lane < a) emit[lane] = s_tok[lane + 1];
    else if (lane == a && bonus >= 0) emit[lane] = bonus;
    if (lane == 0) {
        accept_len[i] = a;
        if (rollback) rollback[i] = (uint8_t)(a < gamma);
        if (stats) {
            if (a < gamma) atomicAdd(stats + 0, 1);
            atomicAdd(stats + 1, a + 1);
        }
    }
}

// ---- 2b. greedy decision on a candidate tree ---------------------------------------------------
// Same merge of the per-segment maxima as above; then one thread walks from the root: at node u the target's
// token is the argmax of row u; the walk goes on to the child of u that carries it (the lowest row among equal
// children) and stops where there is none.  path = the visited rows, out_tokens = their tokens then the bonus.
__global__ __launch_bounds__(256) void accept_decide_tree_kernel(
    const int32_t* __restrict__ tokens, const int32_t* __restrict__ parent, const int32_t* __restrict__ qo_indptr,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens, int32_t* __restrict__ path,
    uint8_t* __restrict__ rollback, int32_t* __restrict__ stats, int M, int V, int nseg, int gamma_max,
    AcceptWorkspace w, int32_t* __restrict__ status_flags)
{
    __shared__ int s_arg[kMaxRows], s_bad[kMaxRows], s_tok[kMaxRows], s_par[kMaxRows];
    const int i = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, tid = threadIdx.x;
    const int r0 = qo_indptr[i], n = qo_indptr[i + 1] - r0;
    int32_t* emit = out_tokens + (size_t)i * (gamma_max + 1);
    int32_t* pth = path + (size_t)i * (gamma_max + 1);
    for (int j = tid; j <= gamma_max; j += 256) { emit[j] = -1; pth[j] = j == 0 ? 0 : -1; }
    if (tid == 0) { accept_len[i] = 0; if (rollback) rollback[i] = 0; }
    if (n < 1 || n - 1 > gamma_max || r0 < 0 || r0 + n > M) {
        if (tid == 0 && status_flags) atomicOr(status_flags, SPEC_FLAG_BAD_LENGTH);
        return;
    }
    for (int j = wave; j < n; j += 4) {
        const size_t base = (size_t)(r0 + j) * nseg;
        float m = -INFINITY;
        int arg = 0x7FFFFFFF, bad = 0;
        for (int s = lane; s < nseg; s += 64) {
            const float sm = w.seg_max[base + s];
            const int sa = w.seg_arg[base + s];
            bad |= w.seg_bad[base + s];
            if (sm > m || (sm == m && sa < arg)) { m = sm; arg = sa; }
        }
        wave_max_arg(m, arg);
        bad = __any(bad) || !(m > -INFINITY && m < INFINITY);
        if (lane == 0) { s_arg[j] = arg; s_bad[j] = bad; }
    }
    if (tid < n) { s_tok[tid] = tokens[r0 + tid]; s_par[tid] = parent[r0 + tid]; }
    __syncthreads();
    if (tid != 0) return;
    int flags = 0;
    for (int j = 0; j < n; ++j) {
        if (s_bad[j]) flags |= SPEC_FLAG_BAD_LOGITS;
        if (j > 0 && (s_tok[j] < 0 || s_tok[j] >= V)) flags |= SPEC_FLAG_BAD_TOKEN;
        if (j == 0 ? s_par[0] != -1 : (s_par[j] < 0 || s_par[j] >= j)) flags |= SPEC_FLAG_BAD_TREE;
    }
    if (flags) {
        if (rollback) rollback[i] = (uint8_t)(n > 1);
        if (stats && n > 1) atomicAdd(stats + 0, 1);
        if (status_flags) atomicOr(status_flags, flags);
        return;
    }
    int u = 0, a = 0;
    for (;;) {
        int next = -1;
        for (int v = u + 1; v < n; ++v)
            if (s_par[v] == u && s_tok[v] == s_arg[u]) { next = v; break; }
        if (next < 0) break;
        emit[a] = s_tok[next];
        ++a;
        pth[a] = next;
        u = next;
    }
    emit[a] = s_arg[u];
    accept_len[i] = a;
    int has_child = 0;
    for (int v = u + 1; v < n; ++v) has_child |= (s_par[v] == u);
    if (rollback) rollback[i] = (uint8_t)has_child;
    if (stats) {
        if (has_child) atomicAdd(stats + 0, 1);
        atomicAdd(stats + 1, a + 1);
    }
}

// residual weight of vocabulary entry v on the job's row: max(0, p(v) - q(v)) in fp32, and p(v)
// e / z with z >= 1 and 0 < e <= 2.03 (no scaling needed): rz is the correctly rounded 1 / z, the product is within an
// ulp of the quotient, and one exact remainder (a fused multiply-add) corrects it to the correctly rounded quotient
// (Markstein's theorem), i.e. to the value the division instruction sequence returns, in 3 instead of ~15 operations.
__device__ inline double quotient_by(double e, double z, double rz)
{
    const double q0 = e * rz;
    return fma(fma(-q0, z, e), rz, q0);
}

__device__ inline void residual_of(float l, float qv, double m, double inv_t, double z, double rz, const double* s_tbl, float& p, float& rho)
{
    p = (float)quotient_by(exp_bulk(((double)l - m) * inv_t, s_tbl), z, rz);
    const float diff = p - qv;
    rho = diff > 0.0f ? diff : 0.0f;
}

// What a workgroup needs to know about the row a request's bonus token is drawn from.  Every field is fetched before
// the first is looked at (one memory round trip); for a request that draws nothing (row < 0) the rest is stale, unused.
struct BonusJob {
    int row, qrow, onehot;
    double m, inv_t;
    float u;
};

__device__ inline BonusJob load_job(const AcceptWorkspace& w, int i)
{
    BonusJob j;
    j.row = w.job_row[i]; j.qrow = w.job_qrow[i]; j.onehot = w.job_onehot[i];
    j.m = w.job_m[i]; j.u = w.job_u[i];
    j.inv_t = 1.0 / (double)w.job_t[i];
    return j;
}

// Z of the bonus row: either what the decision kernel left (sums_exact: every row's Z was summed in fp64), or the sum
// of the per-segment fp64 sums of accept_bonus_z_kernel.  Lane s of wave 0 takes segments s, s + 64, ...; the butterfly
// that follows adds in a fixed order, so every workgroup of a request arrives at the same bits.  Returned through LDS
// (s_z), visible after the caller's next barrier.
__device__ inline void stage_bonus_z(const AcceptWorkspace& w, int i, int nseg, bool z_from_segments, double* s_z, int tid)
{
    if (tid >= 64) return;
    double z = 0.0;
    if (z_from_segments) {
        for (int s = tid; s < nseg; s += 64) z += w.job_zseg[(size_t)i * nseg + s];
        z = wave_sum(z);
    } else {
        z = w.job_z[i];
    }
    if (tid == 0) *s_z = z;
}

// ---- 3a. exact Z of the one row per request that the bonus is drawn from --------------------------
// (only when the bulk sums were taken in fp32, see accept_row_stats_kernel)
constexpr int kJobSegs = 1;         // consecutive segments per workgroup of the two bonus-row kernels (2 measured no faster:
                                    // their time is launch + two memory round trips + the fp64 exponentials, all in one round)

__global__ __launch_bounds__(kThreads) void accept_bonus_z_kernel(const float* __restrict__ logits, int V, int nseg, bool vec,
                                                                  AcceptWorkspace w)
{
    __shared__ double s_part[kJobSegs][kThreads / 64];
    __shared__ double s_tbl[64];
    const int seg0 = blockIdx.x * kJobSegs, i = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const BonusJob job = load_job(w, i);
    if (job.row < 0) return;
    load_exp_table(s_tbl, tid);
    float x[kJobSegs][kPerThread];
#pragma unroll
    for (int q = 0; q < kJobSegs; ++q) {
        const int v0 = (seg0 + q) * kSeg;
        load_strided(logits + (size_t)job.row * V, min(v0, V), min(V, v0 + kSeg), vec, tid, x[q]);   // past the row: all -inf
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kJobSegs; ++q) {
        double z = 0.0;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) z += exp_bulk(((double)x[q][k] - job.m) * job.inv_t, s_tbl);   // -inf slots add ~1e-304
        z = wave_sum(z);
        if (lane == 0) s_part[q][wave] = z;
    }
    __syncthreads();
    if (tid < kJobSegs && seg0 + tid < nseg) {
        double t = 0.0;
        for (int k = 0; k < kThreads / 64; ++k) t += s_part[tid][k];
        w.job_zseg[(size_t)i * nseg + seg0 + tid] = t;
    }
}

// ---- 3. segment sums of the residual ---------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_residual_sums_kernel(
    const float* __restrict__ logits, const float* __restrict__ draft_probs, int V, int nseg, bool vec,
    bool z_from_segments, AcceptWorkspace w)
{
    __shared__ double s_r[kJobSegs][kThreads / 64], s_p[kJobSegs][kThreads / 64];
    __shared__ double s_tbl[64];
    __shared__ double s_z;
    const int seg0 = blockIdx.x * kJobSegs, i = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const BonusJob job = load_job(w, i);
    stage_bonus_z(w, i, nseg, z_from_segments, &s_z, tid);
    if (job.row < 0) return;
    load_exp_table(s_tbl, tid);
    float x[kJobSegs][kPerThread], qv[kJobSegs][kPerThread];
#pragma unroll
    for (int q = 0; q < kJobSegs; ++q) {
        const int v0 = min((seg0 + q) * kSeg, V), vend = min(V, v0 + kSeg);
        load_strided(logits + (size_t)job.row * V, v0, vend, vec, tid, x[q]);
        if (job.qrow >= 0) load_strided(draft_probs + (size_t)job.qrow * V, v0, vend, vec, tid, qv[q]);
    }
    __syncthreads();
    const double z = s_z, rz = 1.0 / z;
#pragma unroll
    for (int q = 0; q < kJobSegs; ++q) {
        const int v0 = (seg0 + q) * kSeg, vend = min(V, v0 + kSeg);
        double rs = 0.0, ps = 0.0;
#pragma unroll
        for (int it = 0; it < kPerThread / 4; ++it)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int v = v0 + (it * kThreads + tid) * 4 + k;
                if (v < vend) {
                    const float qd = job.qrow >= 0 ? qv[q][it * 4 + k] : (v == job.onehot ? 1.0f : 0.0f);
                    float p, rho;
                    residual_of(x[q][it * 4 + k], qd, job.m, job.inv_t, z, rz, s_tbl, p, rho);
                    rs += (double)rho;
                    ps += (double)p;
                }
            }
        rs = wave_sum(rs);
        ps = wave_sum(ps);
        if (lane == 0) { s_r[q][wave] = rs; s_p[q][wave] = ps; }
    }
    __syncthreads();
    if (tid < kJobSegs && seg0 + tid < nseg) {
        double r = 0.0, p = 0.0;
        for (int k = 0; k < kThreads / 64; ++k) { r += s_r[tid][k]; p += s_p[tid][k]; }
        w.res_sum[(size_t)i * nseg + seg0 + tid] = r;
        w.p_sum[(size_t)i * nseg + seg0 + tid] = p;
    }
}

// ---- 4. inverse CDF ----------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_pick_kernel(
    const float* __restrict__ logits, const float* __restrict__ draft_probs, const int32_t* __restrict__ accept_len,
    int32_t* __restrict__ out_tokens, int V, int nseg, int gamma_max, bool vec, bool z_from_segments, AcceptWorkspace w)
{
    __shared__ int s_seg, s_use_p, s_best, s_last;
    __shared__ double s_before, s_target, s_wave[kThreads / 64], s_z;
    __shared__ double s_tbl[64];
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // everything that depends on the request alone is requested at once: one memory round trip, not five
    const BonusJob job = load_job(w, i);
    const int slot = accept_len[i];
    // the segment sums are walked by one thread: up to kPickLds of them come to LDS first
    __shared__ double s_rs[kPickLds], s_ps[kPickLds];
    const bool staged = nseg <= kPickLds;
    if (staged) {
        for (int s = tid; s < nseg; s += kThreads) {
            s_rs[s] = w.res_sum[(size_t)i * nseg + s];
            s_ps[s] = w.p_sum[(size_t)i * nseg + s];
        }
    }
    stage_bonus_z(w, i, nseg, z_from_segments, &s_z, tid);
    if (job.row < 0) return;
    load_exp_table(s_tbl, tid);
    __syncthreads();
    if (wave == 0) {
        // Wave 0 walks the segment sums 64 at a time: totals, then an inclusive scan against u * total.  (One thread
        // doing this serially spends a load latency per segment.)  The sums are non-negative, so the first lane whose
        // running sum exceeds the target marks the segment.
        auto seg_sum = [&](int s, int from_p) -> double {
            if (staged) return from_p ? s_ps[s] : s_rs[s];
            return from_p ? w.p_sum[(size_t)i * nseg + s] : w.res_sum[(size_t)i * nseg + s];
        };
        double tr = 0.0, tp = 0.0;
        for (int s = lane; s < nseg; s += 64) { tr += seg_sum(s, 0); tp += seg_sum(s, 1); }
        tr = wave_sum(tr);
        tp = wave_sum(tp);
        const int use_p = !(tr > 0.0);                    // p == q numerically: draw from p itself
        const double target = (double)job.u * (use_p ? tp : tr);
        double carry = 0.0, before = 0.0;
        int found = -1, last_pos = 0;
        for (int base = 0; base < nseg && found < 0; base += 64) {
            const int s = base + lane;
            const double v = s < nseg ? seg_sum(s, use_p) : 0.0;
            double incl = v;
#pragma unroll
            for (int dd = 1; dd < 64; dd <<= 1) {
                const double up = __shfl_up(incl, dd, 64);
                if (lane >= dd) incl += up;
            }
            const unsigned long long over = __ballot(s < nseg && carry + incl > target);
            const unsigned long long pos = __ballot(s < nseg && v > 0.0);
            if (over) {
                const int l = __ffsll((long long)over) - 1;
                found = base + l;
                before = carry + __shfl(incl - v, l, 64);
                const unsigned long long pos_upto = pos & ((2ull << l) - 1ull);
                if (pos_upto) last_pos = base + 63 - __clzll((long long)pos_upto);
            } else {
                if (pos) last_pos = base + 63 - __clzll((long long)pos);
                carry += __shfl(incl, 63, 64);
            }
        }
        if (found < 0) {                                  // rounding ran the CDF out: last segment with weight
            found = last_pos;
            double b = 0.0;
            for (int s = lane; s < found; s += 64) b += seg_sum(s, use_p);
            before = wave_sum(b);
        }
        if (lane == 0) {
            s_seg = found; s_use_p = use_p; s_before = before; s_target = target;
            s_best = 0x7FFFFFFF; s_last = -1;
        }
    }
    __syncthreads();
    const int seg = s_seg, use_p = s_use_p;
    const int qrow = use_p ? -1 : job.qrow, onehot = use_p ? -1 : job.onehot;
    const double z = s_z, rz = 1.0 / z;
    const int v0 = seg * kSeg + tid * kPerThread;          // this thread owns 16 consecutive entries
    const float* lrow = logits + (size_t)job.row * V;
    const float* qptr = qrow >= 0 ? draft_probs + (size_t)qrow * V : nullptr;
    float lv[kPerThread], qv[kPerThread];
    if (vec && v0 + kPerThread <= V) {                     // (V % 4 == 0 and 16-byte aligned rows)
#pragma unroll
        for (int k4 = 0; k4 < kPerThread / 4; ++k4) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(lrow + v0 + 4 * k4);
            lv[4 * k4] = t.x; lv[4 * k4 + 1] = t.y; lv[4 * k4 + 2] = t.z; lv[4 * k4 + 3] = t.w;
            f32x4 q4 = f32x4{0.f, 0.f, 0.f, 0.f};
            if (qptr) q4 = *reinterpret_cast<const f32x4*>(qptr + v0 + 4 * k4);
            qv[4 * k4] = q4.x; qv[4 * k4 + 1] = q4.y; qv[4 * k4 + 2] = q4.z; qv[4 * k4 + 3] = q4.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const int v = v0 + k;
            lv[k] = v < V ? lrow[v] : -INFINITY;
            qv[k] = (v < V && qptr) ? qptr[v] : 0.0f;
        }
    }
    float rho[kPerThread];
    double mine = 0.0;
    int my_last = -1;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        const int v = v0 + k;
        rho[k] = 0.0f;
        if (v < V) {
            const float q = qptr ? qv[k] : (v == onehot ? 1.0f : 0.0f);
            float p, r;
            residual_of(lv[k], q, job.m, job.inv_t, z, rz, s_tbl, p, r);
            rho[k] = use_p ? p : r;
            if (rho[k] > 0.0f) my_last = v;
        }
        mine += (double)rho[k];
    }
    // exclusive prefix of the per-thread sums, in thread order
    double incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const double up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    double before = s_before;
    for (int k = 0; k < wave; ++k) before += s_wave[k];
    double run = before + (incl - mine);
    const double target = s_target;
    int hit = 0x7FFFFFFF;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        run += (double)rho[k];
        if (hit == 0x7FFFFFFF && run > target && v0 + k < V) hit = v0 + k;
    }
    if (hit != 0x7FFFFFFF) atomicMin(&s_best, hit);
    if (my_last >= 0) atomicMax(&s_last, my_last);
    __syncthreads();
    if (tid == 0) {
        const int bonus = s_best != 0x7FFFFFFF ? s_best : s_last;
        out_tokens[(size_t)i * (gamma_max + 1) + slot] = bonus;
    }
}

}  // namespace specv

static int accept_nseg(int V) { return (V + specv::kSeg - 1) / specv::kSeg; }

extern "C" size_t spec_accept_workspace_bytes(int B, int M, int V, int gamma_max)
{
    (void)gamma_max;
    if (B < 0 || M < 0 || V <= 0) return 0;
    specv::AcceptWorkspace w;
    return specv::carve(&w, nullptr, B, M, accept_nseg(V));
}

static int accept_impl(const float* logits, const int32_t* tokens, const float* draft_probs,
                       const float* temperature, const uint64_t* seeds, uint32_t round,
                       const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens,
                       uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                       const float* blk_max, const int32_t* blk_arg, int blocks, specv::AcceptSummary sum,
                       int32_t* status_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace specv;
    if (B < 0 || M < 0 || V <= 0 || gamma_max < 0 || blocks < 0)
        return fail(SPEC_EINVAL, "spec_accept: negative size (B=%d M=%d V=%d gamma_max=%d blocks=%d)", B, M, V, gamma_max, blocks);
    if (B == 0) return SPEC_OK;
    if (!logits || !tokens || !temperature || !qo_indptr || !accept_len || !out_tokens)
        return fail(SPEC_EINVAL, "spec_accept: NULL pointer argument");
    if (blocks > 0 && (!blk_max || !blk_arg)) return fail(SPEC_EINVAL, "spec_accept_stats: blocks > 0 but no block statistics");
    if (gamma_max + 1 > kMaxRows)
        return fail(SPEC_ESHAPE, "spec_accept: gamma_max=%d, at most %d candidate rows per request", gamma_max, kMaxRows);
    if (M < B) return fail(SPEC_EINVAL, "spec_accept: M=%d < B=%d (every request has at least one row)", M, B);
    const int nseg = accept_nseg(V);
    if (nseg > 65535 || M > 65535 || B > 65535)
        return fail(SPEC_ESHAPE, "spec_accept: V=%d or M=%d beyond the launch grid", V, M);
    AcceptWorkspace w;
    const size_t need = carve(&w, nullptr, B, M, nseg);
    if (!workspace || !aligned(workspace, 256))
        return fail(SPEC_EINVAL, "spec_accept: workspace is NULL or not 256-byte aligned");
    if (workspace_bytes < need)
        return fail(SPEC_EWORKSPACE, "spec_accept: workspace %zu bytes, need %zu", workspace_bytes, need);
    carve(&w, (char*)workspace, B, M, nseg);
    const bool vec = (V % 4 == 0) && aligned(logits, 16) && (!draft_probs || aligned(draft_probs, 16));
    hipStream_t s = (hipStream_t)stream;
    // Sampled requests: the bulk sums over all candidate rows in fp32 and an interval test, fp64 sums only on the row
    // the bonus is drawn from (and on rows whose test the interval leaves open); or fp64 sums over every row.
    const int filter_mode = g_accept_filter;
    const bool filter = seeds != nullptr && (filter_mode != 2 || sum.blocks > 0);   // block sums are estimates: the interval test is needed
    const float band = !filter ? 0.0f : (filter_mode == 3 ? 0.25f : 6.103515625e-05f);   // 2^-14; 0.25 leaves most tests open
    if (sum.blocks > 0 || (blocks > 0 && !seeds)) {
        // every row's summary is at hand (or: all greedy, seeds == NULL promises it, and every row's maxima are):
        // no row of logits is scanned
        if (stats) hipLaunchKernelGGL(accept_reset_stats_kernel, dim3(1), dim3(64), 0, s, stats, B);
    } else {
        hipLaunchKernelGGL(accept_row_stats_kernel, dim3((nseg + kSegPerWg - 1) / kSegPerWg, M), dim3(kThreads), 0, s, logits, temperature,
                           qo_indptr, B, V, nseg, vec, w, stats, blocks > 0, filter);
    }
    hipLaunchKernelGGL(accept_decide_kernel, dim3(B), dim3(kDecideThreads), 0, s, logits, tokens, draft_probs, temperature, seeds,
                       round, qo_indptr, accept_len, out_tokens, rollback, stats, M, V, nseg, gamma_max, w, status_flags,
                       blk_max, blk_arg, blocks, band, sum);
    if (seeds) {   // seeds == NULL promises an all-greedy batch: nothing is ever drawn
        if (filter) hipLaunchKernelGGL(accept_bonus_z_kernel, dim3((nseg + kJobSegs - 1) / kJobSegs, B), dim3(kThreads), 0, s, logits, V, nseg, vec, w);
        hipLaunchKernelGGL(accept_residual_sums_kernel, dim3((nseg + kJobSegs - 1) / kJobSegs, B), dim3(kThreads), 0, s, logits, draft_probs, V,
                           nseg, vec, filter, w);
        hipLaunchKernelGGL(accept_pick_kernel, dim3(B), dim3(kThreads), 0, s, logits, draft_probs, accept_len,
                           out_tokens, V, nseg, gamma_max, vec, filter, w);
    }
    return check_launch("spec_accept");
}

extern "C" int spec_accept_stats(const float* logits, const int32_t* tokens, const float* draft_probs,
                                 const float* temperature, const uint64_t* seeds, uint32_t round,
                                 const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens,
                                 uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                                 const float* blk_max, const int32_t* blk_arg, int blocks,
                                 int32_t* status_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    return accept_impl(logits, tokens, draft_probs, temperature, seeds, round, qo_indptr, accept_len, out_tokens, rollback, stats,
                       B, M, V, gamma_max, blk_max, blk_arg, blocks, specv::AcceptSummary{}, status_flags, workspace,
                       workspace_bytes, stream);
}

extern "C" int spec_accept_summary(const float* logits, const int32_t* tokens, const float* draft_probs,
                                   const float* temperature, const uint64_t* seeds, uint32_t round,
                                   const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens,
                                   uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                                   const float* blk_max, const float* blk_sum, const int32_t* blk_span, int blocks,
                                   int32_t* status_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    if (blocks < 0 || (blocks > 0 && (!blk_max || !blk_sum || !blk_span)))
        return specv::fail(SPEC_EINVAL, "spec_accept_summary: blocks=%d without block summaries", blocks);
    specv::AcceptSummary sum{blk_max, blk_sum, blk_span, blocks};
    return accept_impl(logits, tokens, draft_probs, temperature, seeds, round, qo_indptr, accept_len, out_tokens, rollback, stats,
                       B, M, V, gamma_max, nullptr, nullptr, 0, sum, status_flags, workspace, workspace_bytes, stream);
}

extern "C" int spec_accept(const float* logits, const int32_t* tokens, const float* draft_probs,
                           const float* temperature, const uint64_t* seeds, uint32_t round,
                           const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens,
                           uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                           int32_t* status_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    return spec_accept_stats(logits, tokens, draft_probs, temperature, seeds, round, qo_indptr, accept_len, out_tokens,
                             rollback, stats, B, M, V, gamma_max, nullptr, nullptr, 0, status_flags, workspace,
                             workspace_bytes, stream);
}

// ---- spec_accept for callers that cannot allocate: the scratch lives in the library image -----------------------
// One array per GPU (every device that loads the code object holds its own copy at its own address) for as long as
// the process lives.  Nothing in it has to start at zero: every kernel of the call writes what a later one reads.
namespace specv {
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of this GPU's copy of `scratch`, resolved once per device with that device current.  The array's
// name is only a host-side handle: kernels must be given the address looked up here.
static int static_scratch(void** out)
{
    static std::atomic<void*> resolved[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(SPEC_EHIP, "spec_accept_static: no current device (or ordinal beyond %d)", kMaxDevices - 1);
    void* ptr = resolved[dev].load(std::memory_order_acquire);
    if (!ptr) {
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(SPEC_EHIP, "spec_accept_static: cannot resolve the scratch array on device %d: %s", dev, hipGetErrorString(e));
        resolved[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return SPEC_OK;
}
}  // namespace specv

extern "C" int spec_accept_static(const float* logits, const int32_t* tokens, const float* draft_probs,
                                  const float* temperature, const uint64_t* seeds, uint32_t round,
                                  const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens,
                                  uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                                  int32_t* status_flags, void* stream)
{
    using namespace specv;
    const size_t need = spec_accept_workspace_bytes(B, M, V, gamma_max);
    if (need > kStaticScratchBytes)
        return fail(SPEC_EWORKSPACE, "spec_accept_static: B=%d M=%d V=%d needs %zu bytes of scratch, the built-in array holds %zu; "
                    "use spec_accept with a workspace", B, M, V, need, kStaticScratchBytes);
    void* ptr = nullptr;
    if (int rc = static_scratch(&ptr)) return rc;
    return spec_accept_stats(logits, tokens, draft_probs, temperature, seeds, round, qo_indptr, accept_len, out_tokens,
                             rollback, stats, B, M, V, gamma_max, nullptr, nullptr, 0, status_flags, ptr,
                             kStaticScratchBytes, stream);
}

extern "C" int spec_accept_tree(const float* logits, const int32_t* tokens, const int32_t* parent,
                                const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens, int32_t* path,
                                uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                                int32_t* status_flags, void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace specv;
    if (B < 0 || M < 0 || V <= 0 || gamma_max < 0)
        return fail(SPEC_EINVAL, "spec_accept_tree: negative size (B=%d M=%d V=%d gamma_max=%d)", B, M, V, gamma_max);
    if (B == 0) return SPEC_OK;
    if (!logits || !tokens || !parent || !qo_indptr || !accept_len || !out_tokens || !path)
        return fail(SPEC_EINVAL, "spec_accept_tree: NULL pointer argument");
    if (gamma_max + 1 > kMaxRows)
        return fail(SPEC_ESHAPE, "spec_accept_tree: gamma_max=%d, at most %d candidate rows per request", gamma_max, kMaxRows);
    if (M < B) return fail(SPEC_EINVAL, "spec_accept_tree: M=%d < B=%d (every request has at least one row)", M, B);
    const int nseg = accept_nseg(V);
    if (nseg > 65535 || M > 65535 || B > 65535)
        return fail(SPEC_ESHAPE, "spec_accept_tree: V=%d or M=%d beyond the launch grid", V, M);
    AcceptWorkspace w;
    const size_t need = carve(&w, nullptr, B, M, nseg);
    if (!workspace || !aligned(workspace, 256))
        return fail(SPEC_EINVAL, "spec_accept_tree: workspace is NULL or not 256-byte aligned");
    if (workspace_bytes < need)
        return fail(SPEC_EWORKSPACE, "spec_accept_tree: workspace %zu bytes, need %zu", workspace_bytes, need);
    carve(&w, (char*)workspace, B, M, nseg);
    const bool vec = (V % 4 == 0) && aligned(logits, 16);
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(accept_row_stats_kernel, dim3((nseg + kSegPerWg - 1) / kSegPerWg, M), dim3(kThreads), 0, s, logits,
                       (const float*)nullptr, qo_indptr, B, V, nseg, vec, w, stats, false, false);
    hipLaunchKernelGGL(accept_decide_tree_kernel, dim3(B), dim3(256), 0, s, tokens, parent, qo_indptr, accept_len, out_tokens,
                       path, rollback, stats, M, V, nseg, gamma_max, w, status_flags);
    return check_launch("spec_accept_tree");
}

