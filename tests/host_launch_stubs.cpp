// Stand-ins for the kernel launchers, for a host-only build of the library's host code (argument
// checks, shape bookkeeping, the Eq. 3 schedule) under AddressSanitizer and UBSan on the CPU.
// Nothing here touches a GPU: a launch that the host code lets through is recorded as done.
#include "stem_common.h"

namespace stem {

int launch_pool(const Problem&, int, const void*, const void*, const void*, float*, float*, float*, hipStream_t) {
    return STEM_OK;
}
int launch_block_scores(const Problem&, int, const float*, const float*, const float*, float, float, bool, float*,
                        hipStream_t) {
    return STEM_OK;
}
int launch_group_scores(const Problem&, const float*, int, float*, hipStream_t) { return STEM_OK; }
int launch_select(const Problem&, int, const float*, const int32_t*, int32_t, int32_t, int32_t*, int32_t*, int32_t,
                  hipStream_t) {
    return STEM_OK;
}
int launch_score_select(const Problem&, int, const float*, const float*, const float*, float, float, const int32_t*,
                        int32_t, int32_t, int32_t*, int32_t*, int32_t, float*, hipStream_t) {
    return STEM_OK;
}
int launch_sparse_attn(const Problem&, const void*, const void*, const void*, const int32_t*, const int32_t*, int32_t,
                       bool, float, void*, float*, hipStream_t) {
    return STEM_OK;
}

}  // namespace stem

// lives in a file of its own with the device array it uses; the host-only build has no device
extern "C" int stem_estimate_static(const stem_shape*, const void*, const void*, const void*, float, float, int32_t,
                                    float*, void*) {
    return STEM_ERR_HIP;
}
