// fea_decode_attention_static: decode attention for callers that cannot allocate and
// have no workspace to hand over (code under graph capture, tight serving loops).
// The plan and the partial results live in a buffer that is part of the library's
// device image; everything else is fea_decode_attention.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/fea.h"
#include "fea_internal.h"

namespace fea {

// One copy per GPU, at an address of its own on each; it lives until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress - never a device
// address: the kernels are given the pointer looked up below.
static __device__ __align__(256) unsigned char scratch[FEA_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, once looked up
static std::mutex g_scratch_mu;

// The buffer's address on the current device (looked up once per device, with that
// device current).  Returns nullptr after storing the error message.
static void* scratch_on_current_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(FEA_EHIP, "fea_decode_attention_static: no current device (%s)", e == hipSuccess ? "index out of range" : hipGetErrorString(e));
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            fail(FEA_EHIP, "fea_decode_attention_static: the workspace symbol has no address on device %d (%s)", dev, hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace fea

using namespace fea;

extern "C" int32_t fea_decode_attention_static(const fea_attn_params* p, const void* q, const void* k_cache, const void* v_cache,
                                               const int32_t* block_tables, int32_t table_stride, const int32_t* seq_lens,
                                               int32_t B, void* out, void* hip_stream) {
    size_t need = 0;
    const int32_t rc = decode_workspace_bytes(p, B, table_stride, &need, "fea_decode_attention_static");
    if (rc != FEA_OK) return rc;
    if (p->flags & (FEA_FLAG_REUSE_PLAN | FEA_FLAG_PLAN_ONLY | FEA_FLAG_REFRESH_PLAN))
        return fail(FEA_EINVAL, "fea_decode_attention_static: FEA_FLAG_REUSE_PLAN, FEA_FLAG_PLAN_ONLY and FEA_FLAG_REFRESH_PLAN need a workspace of the caller's "
                                "(the built-in one is shared by every call on the GPU)");
    if (need > (size_t)FEA_STATIC_WORKSPACE_BYTES)
        return fail(FEA_ERANGE, "fea_decode_attention_static: this batch needs a workspace of %zu bytes, the built-in one has %zu; "
                                "use fea_decode_attention with a workspace of your own",
                    need, (size_t)FEA_STATIC_WORKSPACE_BYTES);
    if (B == 0) return FEA_OK;
    void* ws = scratch_on_current_device();
    if (!ws) return FEA_EHIP;
    return decode_impl(p, q, k_cache, v_cache, block_tables, table_stride, seq_lens, B, out, ws, need, hip_stream);
}
