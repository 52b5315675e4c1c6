// varlen_attn_bwd for callers that cannot provide scratch memory: the backward's workspace (delta, the
// rescaled LSE and the partial sums of split key tiles) lives in a device array of this library.
#include <atomic>

#include "kernels.h"

namespace {

constexpr size_t kStaticWorkspaceBytes = VA_STATIC_WORKSPACE_BYTES;

// One copy per GPU the library's code is loaded on, at an address of its own there.  In host code the name
// is only a handle for hipGetSymbolAddress; kernels and the entry point use the address that call returns.
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_of_device[kMaxDevices];

// Address of `scratch` on the current device (looked up once per device), or nullptr with *err set.
void* scratch_on_current_device(hipError_t* err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    void* ptr = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !ptr) {
        if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
        return nullptr;
    }
    g_scratch_of_device[dev].store(ptr, std::memory_order_release);
    return ptr;
}

}  // namespace

extern "C" int varlen_attn_bwd_static(const void* q, const void* k, const void* v, const void* out, const float* lse,
                                      const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                                      const void* worklist_dkdv, const void* worklist_dkdv_host,
                                      const void* worklist_dq, const void* worklist_dq_host,
                                      const va_shape* shape, float scale, void* dq, void* dk, void* dv, void* stream) {
    const char* who = "varlen_attn_bwd_static";
    if (!shape) return va::fail(VA_EINVAL, "%s: null shape", who);
    const size_t need = varlen_attn_bwd_workspace_bytes(shape);
    if (need > kStaticWorkspaceBytes)
        return va::fail(VA_ESIZE, "%s: these shapes need %zu bytes of scratch, the built-in buffer holds %zu "
                                  "(use varlen_attn_bwd with a workspace of the caller's)", who, need, kStaticWorkspaceBytes);
    hipError_t err = hipSuccess;
    void* ws = scratch_on_current_device(&err);
    if (!ws) return va::fail(VA_EHIP, "%s: the address of the built-in scratch buffer is not available: %s", who,
                             hipGetErrorString(err));
    return varlen_attn_bwd(q, k, v, out, lse, dout, cu_seqlens, prefix_lens, worklist_dkdv, worklist_dkdv_host,
                           worklist_dq, worklist_dq_host, shape, scale, dq, dk, dv, ws, kStaticWorkspaceBytes, stream);
}
