// tman_mpgemv for callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc): the tickets and partial sums that tman_mpgemv takes as a caller
// workspace live in a fixed array in device memory that belongs to the library.
//
// The array's name is only a host-side stand-in for the symbol: its device address is looked up once per
// device with hipGetSymbolAddress (each GPU holds its own copy at its own address) and that pointer is what
// the kernels receive, exactly as they receive the caller's workspace in tman_mpgemv.
#include <mutex>

#include "tman_internal.h"

namespace tman {

static __device__ __align__(256) unsigned char scratch[TMAN_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[kMaxDevices];  // device address of `scratch` on device i, once resolved

// Device address of the scratch array on the current device (resolved at the first call on that device).
static int scratch_on_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TMAN_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return TMAN_ERR_LAUNCH;
        }
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return TMAN_OK;
}

}  // namespace tman

using namespace tman;

extern "C" {

int tman_noalloc_init(void) {
    void* p = nullptr;
    return scratch_on_current_device(&p);
}

int tman_mpgemv_noalloc(const tman_shape_t* shape, const void* packed, const void* lut, int32_t N, void* y,
                        void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !lut || !y) return TMAN_ERR_NULL;
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS) return TMAN_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(lut)) return TMAN_ERR_ALIGN;
    if (tman_mpgemv_workspace_bytes(shape, N) > (size_t)TMAN_NOALLOC_SCRATCH_BYTES) return TMAN_ERR_WORKSPACE;
    void* ws = nullptr;
    rc = scratch_on_current_device(&ws);
    if (rc != TMAN_OK) return rc;
    // The tickets at the start of the array are zero when the library is loaded and every call returns them
    // to zero; the partial sums are written before they are read.  Nothing needs clearing between calls.
    return launch_mpgemv(make_layout(shape), packed, lut, N, y, ws, (hipStream_t)stream);
}

}  // extern "C"
