// The scratch buffer of the entry point that allocates nothing (nm_conv2d_static): the
// partial sums of a K-split variant live here instead of in the library's growable
// workspace.  The array is part of the library's device image, so every GPU the library
// runs on holds its own copy, at its own address, until the process ends.
#include <mutex>

#include "nm_internal.h"

static __device__ __align__(256) unsigned char scratch[nm::kStaticScratchBytes];

namespace nm {

// Device address of the copy of `scratch` on device `dev`, which must be the current
// device.  In host code the array's name is only a handle for the runtime: the address
// a kernel can use comes from hipGetSymbolAddress, looked up once per device and kept.
int static_scratch(int dev, float** out)
{
    static std::mutex mu;
    static std::map<int, float*> ptrs;
    std::lock_guard<std::mutex> lk(mu);
    auto it = ptrs.find(dev);
    if (it == ptrs.end()) {
        int cur = -1;
        NM_HIP_CHECK(hipGetDevice(&cur));
        if (cur != dev) {
            set_error("device %d is not the current device (%d)", dev, cur);
            return NM_ERR_ARG;
        }
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_error("hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
            return NM_ERR_HIP;
        }
        it = ptrs.emplace(dev, reinterpret_cast<float*>(ptr)).first;
    }
    *out = it->second;
    return NM_OK;
}

}  // namespace nm
