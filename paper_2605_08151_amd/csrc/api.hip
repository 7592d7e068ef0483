// Library-wide pieces of the C ABI: error text, version, tuning hooks.
#include "common.h"

#include <cmath>
#include <cstring>

namespace specv {

char* error_buffer()
{
    static thread_local char buf[512] = "";
    return buf;
}

extern Tunable g_attn_chunk_override;
extern Tunable g_lm_kernel;
extern Tunable g_lm_kernel_waves;
extern Tunable g_attn_plan;
extern Tunable g_attn_plan_waves;
extern Tunable g_attn_nr3_waves;
extern Tunable g_attn_rows;
extern Tunable g_attn_rows_ring;
extern Tunable g_accept_filter;
extern Tunable g_lm_packed_waves;
extern Tunable g_lm_packed_wide;
extern Tunable g_lm_packed_tile;
extern Tunable g_lm_mfma_rows;
extern Tunable g_lm_mfma_nt;

}  // namespace specv

extern "C" const char* spec_last_error_string(void) { return specv::error_buffer(); }

extern "C" int spec_version(void) { return 1000; }

// Benchmark hook, not part of the numerical contract: overrides launch heuristics.
//   "attn_chunk"  keys per kv split of spec_verify_attn (0 = automatic)
//   "lm_kernel"   kernel used by spec_lm_head (0 = automatic)
//   "lm_big_waves"  waves per workgroup of its MFMA-bound kernels (4 or 8)
//   "attn_plan"   balanced work list of spec_verify_attn: 0 = automatic, 1 = always, 2 = never
//   "attn_plan_waves"  work items per CU the list aims at (0 = automatic)
//   "lm_packed_waves"  waves per workgroup of spec_lm_head_packed (4 or 8)
extern "C" int spec_set_tuning(const char* key, int value)
{
    if (key && std::strcmp(key, "attn_chunk") == 0) { specv::g_attn_chunk_override = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_kernel") == 0) { specv::g_lm_kernel = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_big_waves") == 0) { specv::g_lm_kernel_waves = value == 4 ? 4 : 8; return SPEC_OK; }
    if (key && std::strcmp(key, "attn_plan") == 0) { specv::g_attn_plan = value; return SPEC_OK; }
    if (key && std::strcmp(key, "attn_plan_waves") == 0) { specv::g_attn_plan_waves = value; return SPEC_OK; }
    if (key && std::strcmp(key, "attn_nr3_waves") == 0) { specv::g_attn_nr3_waves = value == 4 ? 4 : 8; return SPEC_OK; }
    if (key && std::strcmp(key, "attn_rows_ring") == 0) { specv::g_attn_rows_ring = value; return SPEC_OK; }
    if (key && std::strcmp(key, "accept_filter") == 0) { specv::g_accept_filter = value; return SPEC_OK; }
    if (key && std::strcmp(key, "attn_rows") == 0) { specv::g_attn_rows = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_packed_wide") == 0) { specv::g_lm_packed_wide = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_packed_tile") == 0) { specv::g_lm_packed_tile = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_mfma_nt") == 0) { specv::g_lm_mfma_nt = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_mfma_rows") == 0) { specv::g_lm_mfma_rows = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_packed_waves") == 0) { specv::g_lm_packed_waves = value == 4 ? 4 : 8; return SPEC_OK; }
    return specv::fail(SPEC_EINVAL, "spec_set_tuning: unknown key '%s'", key ? key : "(null)");
}

// Mode of the next round from the counters spec_accept left in stats[4] (paper, Method, "Rollback-Based Mode
// Selection", eq. mode_switch_batch; threshold: Section "Throughput-Guided Hybrid Coordination", eq. r_threshold).
// Host arithmetic on four integers; nothing is launched.
extern "C" int spec_next_mode(const int32_t* stats_host, double gamma, double t_draft, double t_target,
                              double* r_hat, double* r_star)
{
    using namespace specv;
    if (!stats_host) return fail(SPEC_EINVAL, "spec_next_mode: NULL stats");
    const int rollbacks = stats_host[0], emitted = stats_host[1], B = stats_host[2];
    if (B <= 0 || rollbacks < 0 || rollbacks > B || emitted < 0)
        return fail(SPEC_EINVAL, "spec_next_mode: inconsistent stats (rollbacks=%d emitted=%d B=%d)", rollbacks, emitted, B);
    if (!(gamma >= 1.0) || !(t_draft >= 0.0) || !(t_target > 0.0))
        return fail(SPEC_EINVAL, "spec_next_mode: need gamma >= 1, t_draft >= 0, t_target > 0");
    const double rh = (double)rollbacks / (double)B;
    const double L = (double)emitted / (double)B;
    // with L <= 1 a round yields one token per request in either mode and the ordinary round is the longer one
    const double rs = L > 1.0 ? (gamma - 1.0) * L * t_draft / ((t_target + (gamma - 1.0) * t_draft) * (L - 1.0))
                              : (double)INFINITY;
    if (r_hat) *r_hat = rh;
    if (r_star) *r_star = rs;
    return rh <= rs ? SPEC_MODE_PARALLEL : SPEC_MODE_ORDINARY;
}
