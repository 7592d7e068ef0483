// spec_assemble_next: the candidates y_{n+1} of the next verification round, built on the device from what
// spec_accept left (paper, Method, "Execution in ordinary mode" / "Execution in parallel mode":
// eqs. ordinary_rollback_seq, ordinary_stable_seq, parallel_stable_seq, parallel_rollback_pad; Appendix
// "Target side", eq. target_suffix_reuse; "Rollback-Based Mode Selection": the rollback set holds the requests
// whose verified drafts were not all accepted or whose prepared continuation no longer fits the outcome).
//
// Integer-only and tiny: one workgroup walks the requests in blocks of 1024; a block scan of the row counts
// gives every request its place in the ragged output, so the layout does not depend on thread timing.
#include "common.h"

namespace specv {

constexpr int kAsmThreads = 1024;

__global__ __launch_bounds__(kAsmThreads) void assemble_next_kernel(
    const int32_t* __restrict__ accept_len, const int32_t* __restrict__ out_tokens, int gamma_max,
    const int32_t* __restrict__ qo_indptr, int B,
    const int32_t* __restrict__ cont, int cont_stride, const int32_t* __restrict__ cont_len,
    const int32_t* __restrict__ repair, int repair_stride, const int32_t* __restrict__ repair_len,
    int mode, int gamma_next,
    int32_t* __restrict__ next_tokens, int32_t* __restrict__ next_qo_indptr, uint8_t* __restrict__ rollback,
    int32_t* __restrict__ stats)
{
    __shared__ int wave_total[kAsmThreads / 64];
    __shared__ int block_total;
    __shared__ int s_rolled[kAsmThreads / 64], s_emitted[kAsmThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int base = 0, rolled_all = 0, emitted_all = 0;
    for (int start = 0; start < B; start += kAsmThreads) {
        const int i = start + tid;
        int rows = 0, g = 0, b = -1, is_rb = 0, emitted = 0;
        const int32_t* from = nullptr;
        if (i < B) {
            const int gamma = qo_indptr[i + 1] - qo_indptr[i] - 1;
            const int a = accept_len[i];
            const bool ok = gamma >= 0 && gamma <= gamma_max && a >= 0 && a <= gamma;
            b = ok ? out_tokens[(size_t)i * (gamma_max + 1) + a] : -1;
            is_rb = 1;
            if (b >= 0) {
                const int cl = (cont && cont_len) ? cont_len[i] : 0;
                if (a == gamma && cl >= 1 && cont[(size_t)i * cont_stride] == b) {
                    is_rb = 0;                            // stable: the prepared continuation goes on
                    g = min(cl - 1, gamma_next);
                    from = cont + (size_t)i * cont_stride + 1;
                } else if (mode == SPEC_MODE_ORDINARY && repair && repair_len) {
                    g = max(0, min(repair_len[i], gamma_next));
                    from = repair + (size_t)i * repair_stride;
                }
                emitted = a + 1;
            } else {
                is_rb = gamma > 0;
            }
            rows = 1 + g;
        }
        // inclusive scan of the row counts inside the wave, then across the 16 waves
        int incl = rows;
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        int rsum = is_rb, esum = emitted;
        for (int d = 32; d >= 1; d >>= 1) { rsum += __shfl_xor(rsum, d, 64); esum += __shfl_xor(esum, d, 64); }
        if (lane == 63) wave_total[wave] = incl;
        if (lane == 0) { s_rolled[wave] = rsum; s_emitted[wave] = esum; }
        __syncthreads();
        if (wave == 0) {
            const int t = lane < kAsmThreads / 64 ? wave_total[lane] : 0;
            int ti = t;
            for (int d = 1; d < 16; d <<= 1) {
                const int up = __shfl_up(ti, d, 64);
                if (lane >= d) ti += up;
            }
            if (lane < kAsmThreads / 64) wave_total[lane] = ti - t;    // exclusive wave offsets
            if (lane == kAsmThreads / 64 - 1) block_total = ti;
        }
        __syncthreads();
        if (i < B) {
            int pos = base + wave_total[wave] + incl - rows;
            next_tokens[pos++] = b;
            for (int j = 0; j < g; ++j) next_tokens[pos++] = from[j];
            next_qo_indptr[i + 1] = pos;
            if (rollback) rollback[i] = (uint8_t)is_rb;
        }
        for (int w = 0; w < kAsmThreads / 64; ++w) { rolled_all += s_rolled[w]; emitted_all += s_emitted[w]; }
        base += block_total;
        __syncthreads();                                  // the shared arrays are rewritten by the next block
    }
    if (tid == 0) {
        next_qo_indptr[0] = 0;
        if (stats) { stats[0] = rolled_all; stats[1] = emitted_all; stats[2] = B; stats[3] = base; }
    }
}

}  // namespace specv

extern "C" int spec_assemble_next(const int32_t* accept_len, const int32_t* out_tokens, int gamma_max,
                                  const int32_t* qo_indptr, int B,
                                  const int32_t* cont, int cont_stride, const int32_t* cont_len,
                                  const int32_t* repair, int repair_stride, const int32_t* repair_len,
                                  int mode, int gamma_next,
                                  int32_t* next_tokens, int32_t* next_qo_indptr, uint8_t* rollback,
                                  int32_t* stats, void* stream)
{
    using namespace specv;
    if (B < 0 || gamma_max < 0 || gamma_next < 0 || cont_stride < 0 || repair_stride < 0)
        return fail(SPEC_EINVAL, "spec_assemble_next: negative size (B=%d gamma_max=%d gamma_next=%d)", B, gamma_max, gamma_next);
    if (mode != SPEC_MODE_ORDINARY && mode != SPEC_MODE_PARALLEL)
        return fail(SPEC_EINVAL, "spec_assemble_next: mode %d is neither SPEC_MODE_ORDINARY nor SPEC_MODE_PARALLEL", mode);
    if (!next_qo_indptr) return fail(SPEC_EINVAL, "spec_assemble_next: NULL pointer argument");
    if (B > 0 && (!accept_len || !out_tokens || !qo_indptr || !next_tokens))
        return fail(SPEC_EINVAL, "spec_assemble_next: NULL pointer argument");
    if ((cont != nullptr) != (cont_len != nullptr) || (repair != nullptr) != (repair_len != nullptr))
        return fail(SPEC_EINVAL, "spec_assemble_next: a token buffer and its lengths come together");
    if ((cont && cont_stride < 1) || (repair && repair_stride < 1))
        return fail(SPEC_EINVAL, "spec_assemble_next: a token buffer needs a row stride >= 1");
    hipLaunchKernelGGL(assemble_next_kernel, dim3(1), dim3(kAsmThreads), 0, (hipStream_t)stream, accept_len, out_tokens,
                       gamma_max, qo_indptr, B, cont, cont_stride, cont_len, repair, repair_stride, repair_len, mode,
                       gamma_next, next_tokens, next_qo_indptr, rollback, stats);
    return check_launch("spec_assemble_next");
}
