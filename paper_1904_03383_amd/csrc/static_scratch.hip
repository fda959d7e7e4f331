// The library's own scratch buffer, for the one entry point that serves callers who cannot
// allocate device memory (code under graph capture, serving loops with a no-allocation rule):
// a file-scope device array of fixed size that every GPU the library runs on holds until the
// process ends.  It takes the place of the caller's workspace for split-K partial products.
//
// In host code the array's name is only a handle for the runtime; its device address is asked
// for once per device (each GPU holds its own copy at its own address) and that address is what
// kernels, fills and copies are given.
#include "tg_internal.h"

#include <mutex>

namespace tg {

namespace {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_scratch_mutex;
void *g_scratch_ptr[64] = {nullptr};   // device address of `scratch`, per device index

}  // namespace

hipError_t static_scratch(void **ptr) {
    *ptr = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // with device `dev` current: that device's copy
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace tg
