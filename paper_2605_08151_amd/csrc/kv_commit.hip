// spec_kv_commit: Commit(p_n, y_n, L_n) on the paged KV cache (paper, Appendix "Target side";
// rollback frees the KV of the rejected suffix, Appendix "Draft side", State recovery).
//
// Integer-only and tiny: one workgroup walks the requests in blocks of 1024, an exclusive
// block scan of "pages this request frees" gives every request its slot range in the free list,
// so the list order is request-ascending then logical-page-ascending whatever the thread timing.
#include "common.h"

namespace specv {

constexpr int kCommitThreads = 1024;

__global__ __launch_bounds__(kCommitThreads) void kv_commit_kernel(
    int32_t* __restrict__ page_table, int max_pages, int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ qo_indptr, const int32_t* __restrict__ accept_len,
    int32_t* __restrict__ free_list, int free_capacity, int32_t* __restrict__ free_count,
    int B, int P, int32_t* __restrict__ status_flags)
{
    __shared__ int wave_total[kCommitThreads / 64];
    __shared__ int block_total;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int base = *free_count;          // every thread reads it before the single write at the end
    __syncthreads();
    int flags = 0;
    for (int start = 0; start < B; start += kCommitThreads) {
        const int i = start + tid;
        int keep = 0, had = 0, new_len = 0, nfree = 0;
        bool live = false;
        if (i < B) {
            const int n = qo_indptr[i + 1] - qo_indptr[i];
            const int c = seq_lens[i];
            if (n >= 1 && c >= 0) {
                live = true;
                int a = accept_len[i];
                a = a < 0 ? 0 : (a > n - 1 ? n - 1 : a);
                new_len = c + a + 1;
                had = (c + n + P - 1) / P;
                if (had > max_pages) had = max_pages;
                keep = (new_len + P - 1) / P;
                for (int pg = keep; pg < had; ++pg)
                    nfree += page_table[(size_t)i * max_pages + pg] >= 0;
            } else {
                flags |= SPEC_FLAG_BAD_LENGTH;
            }
        }
        // inclusive scan inside the wave, then across the 16 waves
        int incl = nfree;
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        if (wave == 0) {
            int t = lane < kCommitThreads / 64 ? wave_total[lane] : 0;
            int ti = t;
            for (int d = 1; d < 16; d <<= 1) {
                const int up = __shfl_up(ti, d, 64);
                if (lane >= d) ti += up;
            }
            if (lane < kCommitThreads / 64) wave_total[lane] = ti - t;     // exclusive wave offsets
            if (lane == kCommitThreads / 64 - 1) block_total = ti;
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
        __syncthreads();             // wave_total / block_total are rewritten next round
    }
    if (tid == 0) *free_count = base < free_capacity ? base : free_capacity;
    if (flags && status_flags) atomicOr(status_flags, flags);
}

// Commit of an accepted tree path (Appendix "Target side", "Unified verification interface": candidates form a
// verification tree; only target-verified tokens enter the committed prefix).  The K/V of the accepted nodes sit at
// cache positions c + path[k]; they are moved to c + k, k = 1 .. a, so that the prefix is contiguous again.
// One workgroup per request; the moves are done in increasing k with a barrier in between: path is increasing and
// path[k] >= k, so a destination is never a later move's source.
__global__ __launch_bounds__(256) void kv_gather_path_kernel(
    uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache, const int32_t* __restrict__ page_table, int max_pages,
    const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ qo_indptr, const int32_t* __restrict__ accept_len,
    const int32_t* __restrict__ path, int gamma_max, int num_pages, int Hkv, int D, int P, int32_t* __restrict__ status_flags)
{
    const int i = blockIdx.x, tid = threadIdx.x;
    const int n = qo_indptr[i + 1] - qo_indptr[i], c = seq_lens[i];
    if (n < 1 || c < 0) return;                           // the commit kernel flags it
    int a = accept_len[i];
    a = a < 0 ? 0 : (a > n - 1 ? n - 1 : a);
    const int chunks = Hkv * (D / 8);                     // 16-byte pieces of one position's K (and of its V)
    for (int k = 1; k <= a; ++k) {
        const int pk = path[(size_t)i * (gamma_max + 1) + k];
        const int src = c + pk, dst = c + k;
        if (pk < k || pk >= n) {                          // not a root path in topological order: leave the rest alone
            if (tid == 0 && status_flags) atomicOr(status_flags, SPEC_FLAG_BAD_TREE);
            return;
        }
        if (src != dst) {
            const int ps = page_table[(size_t)i * max_pages + src / P], pd = page_table[(size_t)i * max_pages + dst / P];
            if (ps < 0 || ps >= num_pages || pd < 0 || pd >= num_pages) {
                if (tid == 0 && status_flags) atomicOr(status_flags, SPEC_FLAG_BAD_PAGE);
                return;
            }
            for (int e = tid; e < 2 * chunks; e += 256) {
                uint16_t* cache = e < chunks ? k_cache : v_cache;
                const int q = e < chunks ? e : e - chunks, h = q / (D / 8), ch = q - h * (D / 8);
                const size_t so = (((size_t)ps * Hkv + h) * P + src % P) * D + ch * 8;
                const size_t dn = (((size_t)pd * Hkv + h) * P + dst % P) * D + ch * 8;
                *reinterpret_cast<u32x4*>(cache + dn) = *reinterpret_cast<const u32x4*>(cache + so);
            }
        }
        __syncthreads();                                  // the next move may overwrite what a thread is still reading here
    }
}

}  // namespace specv

extern "C" int spec_kv_commit(int32_t* page_table, int max_pages_per_seq, int32_t* seq_lens,
                              const int32_t* qo_indptr, const int32_t* accept_len,
                              int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                              int B, int page_size, int32_t* status_flags, void* stream)
{
    using namespace specv;
    if (B < 0 || page_size <= 0 || max_pages_per_seq < 0 || free_capacity < 0)
        return fail(SPEC_EINVAL, "spec_kv_commit: negative size (B=%d page_size=%d max_pages=%d cap=%d)", B,
                    page_size, max_pages_per_seq, free_capacity);
    if (B == 0) return SPEC_OK;
    if (!page_table || !seq_lens || !qo_indptr || !accept_len || !free_list || !free_count)
        return fail(SPEC_EINVAL, "spec_kv_commit: NULL pointer argument");
    hipLaunchKernelGGL(kv_commit_kernel, dim3(1), dim3(kCommitThreads), 0, (hipStream_t)stream, page_table,
                       max_pages_per_seq, seq_lens, qo_indptr, accept_len, free_list, free_capacity, free_count, B,
                       page_size, status_flags);
    return check_launch("spec_kv_commit");
}

extern "C" int spec_kv_commit_tree(void* k_cache, void* v_cache, int32_t* page_table, int max_pages_per_seq, int num_pages,
                                   int32_t* seq_lens, const int32_t* qo_indptr, const int32_t* accept_len,
                                   const int32_t* path, int gamma_max,
                                   int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                                   int B, int Hkv, int D, int page_size, int32_t* status_flags, void* stream)
{
    using namespace specv;
    if (B < 0 || page_size <= 0 || max_pages_per_seq < 0 || free_capacity < 0 || gamma_max < 0 || Hkv <= 0 || D <= 0 || num_pages <= 0)
        return fail(SPEC_EINVAL, "spec_kv_commit_tree: non-positive size");
    if (D % 8 != 0) return fail(SPEC_ESHAPE, "spec_kv_commit_tree: D=%d must be a multiple of 8", D);
    if (B == 0) return SPEC_OK;
    if (!k_cache || !v_cache || !page_table || !seq_lens || !qo_indptr || !accept_len || !path || !free_list || !free_count)
        return fail(SPEC_EINVAL, "spec_kv_commit_tree: NULL pointer argument");
    if (!aligned(k_cache, 16) || !aligned(v_cache, 16)) return fail(SPEC_EINVAL, "spec_kv_commit_tree: caches must be 16-byte aligned");
    hipLaunchKernelGGL(kv_gather_path_kernel, dim3(B), dim3(256), 0, (hipStream_t)stream, (uint16_t*)k_cache, (uint16_t*)v_cache,
                       page_table, max_pages_per_seq, seq_lens, qo_indptr, accept_len, path, gamma_max, num_pages, Hkv, D,
                       page_size, status_flags);
    hipLaunchKernelGGL(kv_commit_kernel, dim3(1), dim3(kCommitThreads), 0, (hipStream_t)stream, page_table,
                       max_pages_per_seq, seq_lens, qo_indptr, accept_len, free_list, free_capacity, free_count, B,
                       page_size, status_flags);
    return check_launch("spec_kv_commit_tree");
}

