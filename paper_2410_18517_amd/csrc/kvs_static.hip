// kvs_decode_attention for callers that cannot allocate (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): the same kernels, with the split-context
// scratch (arrival counters and partial states) in a file-scope device array of this library
// instead of a workspace the caller brings.  Nothing here allocates or frees.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "../../include/kvs.h"
#include "kvs_internal.h"

namespace {

// Every GPU the library's code is loaded on holds one copy of this array until the process ends.
// The runtime zero-fills it when the code object is loaded, and every attention call leaves the
// counter region at its start at zero again, so it is never cleared here.
constexpr size_t kScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code the array's name is only a handle for the runtime, not a device address: the
// address of each GPU's own copy is asked for once per device and kept.
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_of_device[kMaxDevices] = {};

int scratch_of_current_device(void** ptr)
{
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_of_device[dev]) {
        void* p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return (int)e;
        g_scratch_of_device[dev] = p;
    }
    *ptr = g_scratch_of_device[dev];
    return 0;
}

}  // namespace

extern "C" {

size_t kvs_noalloc_scratch_bytes(void) { return kScratchBytes; }

int kvs_decode_attention_noalloc(const kvs_store* store, int layer, const void* q, const int32_t* seq_lens,
                                 int B, float* out, void* stream)
{
    if (!store) return kvs::report_error(KVS_ERR_INVALID_ARG, "store is NULL");
    if (B <= 0) return kvs::report_error(KVS_ERR_INVALID_ARG, "B must be positive");
    const size_t need = kvs_workspace_bytes(&store->desc, B, 1);
    if (need == 0) return KVS_ERR_INVALID_ARG;                    // the descriptor was refused: kvs_last_error says why
    if (need > kScratchBytes) {
        char msg[160];
        snprintf(msg, sizeof msg, "this shape needs %zu bytes of scratch, the built-in array holds %zu: use kvs_decode_attention",
                 need, kScratchBytes);
        return kvs::report_error(KVS_ERR_CAPACITY, msg);
    }
    // the remaining argument checks are those of kvs_decode_attention and precede its launch; a
    // device address is needed to pass it the scratch, so the device is asked for first
    void* ptr = nullptr;
    if (int e = scratch_of_current_device(&ptr)) {
        char msg[160];
        snprintf(msg, sizeof msg, "address of the built-in scratch: %s", kvs::hip_error_string(e));
        return kvs::report_error(KVS_ERR_HIP, msg);
    }
    return kvs_decode_attention(store, layer, q, seq_lens, B, out, ptr, kScratchBytes, stream);
}

}  // extern "C"
