// Draft-side primitives (paper, Appendix "Draft side": "Message handling and update", "State recovery";
// Method, "Draft-side context compression", eq. token_eviction).  Integer-only ragged work; none of it is on the
// target's critical path, so the kernels are plain: one workgroup per request, coalesced token reads.
#include "common.h"

namespace specv {

// delta_i = min{ t : p_i[t] != h_i[t] }, or the shorter length when one sequence is a prefix of the other.
__global__ __launch_bounds__(256) void divergence_kernel(
    const int32_t* __restrict__ p_tokens, const int32_t* __restrict__ p_indptr,
    const int32_t* __restrict__ h_tokens, const int32_t* __restrict__ h_indptr, int32_t* __restrict__ delta)
{
    __shared__ int s_first;
    const int i = blockIdx.x, tid = threadIdx.x;
    const int p0 = p_indptr[i], h0 = h_indptr[i];
    const int n = min(p_indptr[i + 1] - p0, h_indptr[i + 1] - h0);
    if (tid == 0) s_first = n > 0 ? n : 0;
    __syncthreads();
    // chunks of 256 positions in order: the first chunk with a difference ends the walk for the whole workgroup
    for (int base = 0; base < n; base += 256) {
        const int t = base + tid;
        const bool differs = t < n && p_tokens[p0 + t] != h_tokens[h0 + t];
        if (differs) atomicMin(&s_first, t);
        if (__syncthreads_or(differs)) break;
    }
    __syncthreads();
    if (tid == 0) delta[i] = s_first;
}

// Rollback(S, delta): keep min(len_i, max(keep_len[i], 0)) tokens, unmap and free the pages beyond.
// Same single-workgroup block scan as the commit kernel, so the free list order is request-ascending, then
// logical-page-ascending.
constexpr int kTruncThreads = 1024;

__global__ __launch_bounds__(kTruncThreads) void kv_truncate_kernel(
    int32_t* __restrict__ page_table, int max_pages, int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ keep_len, int32_t* __restrict__ free_list, int free_capacity,
    int32_t* __restrict__ free_count, int B, int P, int32_t* __restrict__ status_flags)
{
    __shared__ int wave_total[kTruncThreads / 64];
    __shared__ int block_total;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int base = *free_count;          // every thread reads it before the single write at the end
    __syncthreads();
    int flags = 0;
    for (int start = 0; start < B; start += kTruncThreads) {
        const int i = start + tid;
        int keep = 0, had = 0, new_len = 0, nfree = 0;
        bool live = false;
        if (i < B) {
            const int c = seq_lens[i];
            if (c >= 0) {
                live = true;
                const int k = keep_len[i];
                new_len = k < 0 ? 0 : (k > c ? c : k);
                had = (c + P - 1) / P;
                if (had > max_pages) had = max_pages;
                keep = (new_len + P - 1) / P;
                for (int pg = keep; pg < had; ++pg)
                    nfree += page_table[(size_t)i * max_pages + pg] >= 0;
            } else {
                flags |= SPEC_FLAG_BAD_LENGTH;
            }
        }
        int incl = nfree;
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        if (wave == 0) {
            const int t = lane < kTruncThreads / 64 ? wave_total[lane] : 0;
            int ti = t;
            for (int d = 1; d < 16; d <<= 1) {
                const int up = __shfl_up(ti, d, 64);
                if (lane >= d) ti += up;
            }
            if (lane < kTruncThreads / 64) wave_total[lane] = ti - t;
            if (lane == kTruncThreads / 64 - 1) block_total = ti;
        }
        __syncthreads();
        int slot = base + wave_total[wave] + incl - nfree;
        if (live) {
            for (int pg = keep; pg < had; ++pg) {
                int32_t* e = page_table + (size_t)i * max_pages + pg;
                const int v = *e;
                if (v >= 0) {
                    if (slot < free_capacity) free_list[slot] = v;
                    else flags |= SPEC_FLAG_FREE_OVERFLOW;
                    ++slot;
                    *e = -1;
                }
            }
            seq_lens[i] = new_len;
        }
        base += block_total;
        __syncthreads();
    }
    if (tid == 0) *free_count = base < free_capacity ? base : free_capacity;
    if (flags && status_flags) atomicOr(status_flags, flags);
}

// E(x_{1:S}) = [x_{:k}, x_{S-k+1:}], k = floor(p S / 2) with p = p_num / p_den; a prompt with 2k >= S is kept whole.
// One workgroup per prompt: its place in the ragged output is the sum of the kept counts of the prompts before it.
__device__ inline int kept_count(int S, int p_num, int p_den)
{
    const long long k = (long long)p_num * S / (2LL * p_den);
    return 2 * k >= S ? S : (int)(2 * k);
}

__global__ __launch_bounds__(256) void compress_prompts_kernel(
    const int32_t* __restrict__ tokens, const int32_t* __restrict__ indptr, int B, int p_num, int p_den,
    int32_t* __restrict__ out_tokens, int32_t* __restrict__ out_indptr, int32_t* __restrict__ kept_index)
{
    __shared__ int s_part[4];
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int before = 0;
    for (int j = tid; j < i; j += 256) before += kept_count(indptr[j + 1] - indptr[j], p_num, p_den);
    for (int d = 32; d >= 1; d >>= 1) before += __shfl_xor(before, d, 64);
    if (lane == 0) s_part[wave] = before;
    __syncthreads();
    const int off = s_part[0] + s_part[1] + s_part[2] + s_part[3];
    const int x0 = indptr[i], S = indptr[i + 1] - x0;
    const int kept = kept_count(S, p_num, p_den), k = kept / 2;
    for (int t = tid; t < kept; t += 256) {
        const int srcpos = (kept == S || t < k) ? t : S - kept + t;     // second half: the last k tokens
        out_tokens[off + t] = tokens[x0 + srcpos];
        if (kept_index) kept_index[off + t] = srcpos;
    }
    if (tid == 0) {
        out_indptr[i + 1] = off + kept;
        if (i == 0) out_indptr[0] = 0;
    }
}

__global__ void zero_first_kernel(int32_t* p) { if (threadIdx.x == 0) p[0] = 0; }

}  // namespace specv

extern "C" int spec_divergence(const int32_t* p_tokens, const int32_t* p_indptr, const int32_t* h_tokens,
                               const int32_t* h_indptr, int32_t* delta, int B, void* stream)
{
    using namespace specv;
    if (B < 0) return fail(SPEC_EINVAL, "spec_divergence: negative B=%d", B);
    if (B == 0) return SPEC_OK;
    if (!p_tokens || !p_indptr || !h_tokens || !h_indptr || !delta) return fail(SPEC_EINVAL, "spec_divergence: NULL pointer argument");
    hipLaunchKernelGGL(divergence_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, p_tokens, p_indptr, h_tokens, h_indptr, delta);
    return check_launch("spec_divergence");
}

extern "C" int spec_kv_truncate(int32_t* page_table, int max_pages_per_seq, int32_t* seq_lens, const int32_t* keep_len,
                                int32_t* free_list, int32_t free_capacity, int32_t* free_count, int B, int page_size,
                                int32_t* status_flags, void* stream)
{
    using namespace specv;
    if (B < 0 || page_size <= 0 || max_pages_per_seq < 0 || free_capacity < 0)
        return fail(SPEC_EINVAL, "spec_kv_truncate: negative size (B=%d page_size=%d max_pages=%d cap=%d)", B, page_size,
                    max_pages_per_seq, free_capacity);
    if (B == 0) return SPEC_OK;
    if (!page_table || !seq_lens || !keep_len || !free_list || !free_count)
        return fail(SPEC_EINVAL, "spec_kv_truncate: NULL pointer argument");
    hipLaunchKernelGGL(kv_truncate_kernel, dim3(1), dim3(kTruncThreads), 0, (hipStream_t)stream, page_table, max_pages_per_seq,
                       seq_lens, keep_len, free_list, free_capacity, free_count, B, page_size, status_flags);
    return check_launch("spec_kv_truncate");
}

extern "C" int spec_compress_prompts(const int32_t* tokens, const int32_t* indptr, int B, int p_num, int p_den,
                                     int32_t* out_tokens, int32_t* out_indptr, int32_t* kept_index, void* stream)
{
    using namespace specv;
    if (B < 0 || p_num < 0 || p_den <= 0)
        return fail(SPEC_EINVAL, "spec_compress_prompts: need B >= 0 and a ratio p_num / p_den >= 0 (got %d, %d / %d)", B, p_num, p_den);
    if (!out_indptr) return fail(SPEC_EINVAL, "spec_compress_prompts: NULL pointer argument");
    if (B == 0) {
        hipLaunchKernelGGL(zero_first_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, out_indptr);
        return check_launch("spec_compress_prompts");
    }
    if (!tokens || !indptr || !out_tokens) return fail(SPEC_EINVAL, "spec_compress_prompts: NULL pointer argument");
    hipLaunchKernelGGL(compress_prompts_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, tokens, indptr, B, p_num, p_den,
                       out_tokens, out_indptr, kept_index);
    return check_launch("spec_compress_prompts");
}
