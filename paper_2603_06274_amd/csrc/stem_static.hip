// stem_estimate_static: stage 1 for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The pooled block
// representations, which stem_estimate keeps in a caller-provided workspace, live here in an array
// that is part of the library's code object: every GPU the library runs on holds its own copy from
// the moment the module is loaded until the process ends.
#include <mutex>

#include "stem_common.h"

namespace {

// The array's name is only a host-side handle: the device address is looked up once per device
// and kept in scratch_ptr; host code hands kernels that pointer, never the name.
static __device__ __align__(256) unsigned char scratch[STEM_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static void* scratch_ptr[kMaxDevices];
static std::mutex scratch_mutex;

// Device address of this device's copy of the array (nullptr on failure).
void* device_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

}  // namespace

extern "C" int stem_estimate_static(const stem_shape* shape, const void* q, const void* k, const void* v,
                                    float beta, float route_scale, int32_t ad_stride, float* scores,
                                    void* hip_stream) {
    size_t need = 0;
    int st = stem_workspace_bytes(shape, ad_stride, &need);
    if (st != STEM_OK) return st;
    // a chunk's scores read the pooled keys of earlier calls, which this shared array cannot promise
    if (shape->host_chunk_start != nullptr) return STEM_ERR_UNSUPPORTED;
    if (need > (size_t)STEM_STATIC_WORKSPACE_BYTES) return STEM_ERR_WORKSPACE;
    void* ws = device_scratch();
    if (ws == nullptr) return STEM_ERR_HIP;
    return stem_estimate(shape, q, k, v, beta, route_scale, ad_stride, 1, scores, ws,
                         (size_t)STEM_STATIC_WORKSPACE_BYTES, hip_stream);
}
