// Library-wide pieces of the C ABI: error text, version, tuning hooks.
#include "common.h"

#include <cstring>

namespace specv {

char* error_buffer()
{
    static thread_local char buf[512] = "";
    return buf;
}

extern int g_attn_chunk_override;
extern int g_lm_kernel;

}  // namespace specv

extern "C" const char* spec_last_error_string(void) { return specv::error_buffer(); }

extern "C" int spec_version(void) { return 1000; }

// Benchmark hook, not part of the numerical contract: overrides launch heuristics.
//   "attn_chunk"  keys per kv split of spec_verify_attn (0 = automatic)
//   "lm_kernel"   kernel used by spec_lm_head (0 = automatic)
extern "C" int spec_set_tuning(const char* key, int value)
{
    if (key && std::strcmp(key, "attn_chunk") == 0) { specv::g_attn_chunk_override = value; return SPEC_OK; }
    if (key && std::strcmp(key, "lm_kernel") == 0) { specv::g_lm_kernel = value; return SPEC_OK; }
    return specv::fail(SPEC_EINVAL, "spec_set_tuning: unknown key '%s'", key ? key : "(null)");
}
