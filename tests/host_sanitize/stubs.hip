// Stand-ins for the kernel launchers, so that the kernel-free host part of the library (argument
// checks, launch planning, the page map) links without any device code.  The driver only makes
// calls that return before a launch; reaching one of these is a test failure.
#include <cstdio>
#include <cstdlib>
#include "cs_common.h"

namespace cs {

[[noreturn]] static int reached(const char* what) {
    std::fprintf(stderr, "host-only test reached a kernel launcher: %s\n", what);
    std::abort();
}

int launch_append(const cs_kv_pool&, int32_t, const cs_batch&, const void*, const void*, hipStream_t) { reached("append"); }
int launch_page_copy(const cs_kv_pool&, int32_t, int32_t, const int32_t*, int32_t, void*, bool, hipStream_t, bool) { reached("page copy"); }
int launch_token_copy(const cs_kv_pool&, int32_t, int32_t, const int32_t*, int32_t, void*, bool, hipStream_t) { reached("token copy"); }
int launch_plain_copy(void*, const void*, size_t, hipStream_t) { reached("plain copy"); }
int launch_decode(const cs_kv_pool&, int32_t, const cs_batch&, const DecodePlan&, const void*, void*, int32_t, float, void*,
                  hipStream_t, bool, bool) { reached("decode"); }
int launch_prefill(const cs_kv_pool&, int32_t, const cs_batch&, const PrefillPlan&, const void*, void*, int32_t, float, void*,
                   hipStream_t, bool) { reached("prefill"); }
int launch_prefill_merge(const cs_kv_pool&, const cs_batch&, const PrefillPlan&, void*, int32_t, void*, hipStream_t, bool) { reached("prefill merge"); }
int launch_mixed(const cs_kv_pool&, int32_t, const cs_batch&, const DecodePlan&, const PrefillPlan&, const void*, void*, int32_t, float,
                 void*, void*, hipStream_t, bool, int32_t, int32_t) { reached("mixed"); }

}  // namespace cs
