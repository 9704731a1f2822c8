// The library's own staging chunk, for callers that cannot allocate device memory
// (code under HIP-graph capture, serving loops, harnesses that forbid hipMalloc).
//
// The staged path needs one chunk of device memory beyond the source and target
// shards.  liver_pack / liver_unpack take it from the caller; liver_reshard_static
// takes it from the file-scope array below, which every GPU the library is loaded on
// holds from module load until the process ends.  Host code never uses the array's
// name as an address (on the host it is only a handle of the symbol): the address
// on a device is looked up once, with that device current, and kept per device.
#include <hip/hip_runtime.h>

#include <mutex>

#include "launch.hpp"

namespace liver {
namespace {

static __device__ __align__(256) unsigned char scratch[STATIC_STAGING_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void* g_ptr[MAX_DEVICES] = {};  // per device: where `scratch` lives there

}  // namespace

hipError_t static_staging(int device, void** ptr) {
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;  // the lookup answers for the current device
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || (uintptr_t)p % 256) return hipErrorInvalidSymbol;
        g_ptr[device] = p;
    }
    *ptr = g_ptr[device];
    return hipSuccess;
}

}  // namespace liver
