// sepattn_decode_noalloc: the decode call for callers that cannot allocate device memory and have no
// workspace to hand over (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  It runs the kernels of sepattn_decode; the partial results of the cache slices, which
// sepattn_decode keeps in the caller's workspace, live in a fixed array inside the library instead.
#include <mutex>

#include "common.h"

namespace {

// One copy per GPU the library runs on, held until the process ends.  In host code the array's name
// is only a handle for hipGetSymbolAddress: the kernels get the device address obtained from it.
static __device__ __align__(256) unsigned char scratch[SEPATTN_DECODE_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up once per device, with it current)
void *scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

size_t sepattn_decode_noalloc_scratch_bytes(const sepkv_params *p) { return sepattn_decode_workspace_bytes(p); }

int sepattn_decode_noalloc(const sepkv_params *p, const void *q, const void *Kc, const void *Vc,
                           const int32_t *sizes, void *out, float *lse, void *stream) {
    int rc = sepattn::check_kv_params(p);
    if (rc != SEPATTN_OK) return rc;
    if (!q || !Kc || !Vc || !sizes || !out) return SEPATTN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(Kc) % 16 ||
        reinterpret_cast<uintptr_t>(Vc) % 16 || reinterpret_cast<uintptr_t>(out) % 16)
        return SEPATTN_ERR_PARAM;
    // the slices' partial results must fit the fixed array
    if (sepattn::decode_workspace(*p) > (size_t)SEPATTN_DECODE_NOALLOC_SCRATCH_BYTES) return SEPATTN_ERR_WORKSPACE;
    void *ptr = scratch_of_current_device();
    if (!ptr) return SEPATTN_ERR_HIP;
    sepattn::discard_stale_hip_error();
    // every slot of the partials that the merge step reads is written by this call's first kernel, so
    // nothing has to be cleared between calls
    return sepattn::launch_decode(*p, q, Kc, Vc, sizes, nullptr, 0, out, lse, ptr, static_cast<hipStream_t>(stream));
}

}  // extern "C"
