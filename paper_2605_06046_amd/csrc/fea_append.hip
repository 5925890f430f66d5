// Appending one decoded token's K and V per request to the paged cache: the write
// that precedes every decode-attention call (Section 2.1: each step extends every
// request's KV history by one token; Section 3: the history lives in 16-token blocks).
//
// Request i's new token sits at position seq_lens[i] - 1 (the lengths already count
// it), i.e. in block block_tables[i][pos / 16], slot pos % 16, for every KV head.
// One thread moves 16 bytes; the whole launch moves 2 B Hkv d elements.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "../../include/fea.h"
#include "fea_internal.h"
#include "fea_plan.h"

namespace fea {

struct AppendArgs {
    const char* k_new;
    const char* v_new;
    char* k_cache;
    char* v_cache;
    const int32_t* bt;
    const int32_t* seq_lens;
    int32_t stride, B, Hkv;
    int32_t row_bytes;     // head_dim * element size: one token of one KV head
};

__global__ __launch_bounds__(256) void append_kernel(AppendArgs a) {
    const int chunks = a.row_bytes / 16;
    const long long per_cache = (long long)a.B * a.Hkv * chunks;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= 2 * per_cache) return;
    const bool is_v = idx >= per_cache;
    long long r = is_v ? idx - per_cache : idx;
    const int c = (int)(r % chunks); r /= chunks;
    const int g = (int)(r % a.Hkv);
    const int i = (int)(r / a.Hkv);
    const int L = a.seq_lens[i];
    if (L <= 0 || (L - 1) / kBlock >= a.stride) return;   // nothing to write / no such column
    const int pos = L - 1;
    const int b = a.bt[(size_t)i * a.stride + pos / kBlock];
    if (b < 0) return;                                    // padding entry: the caller's table is short
    const size_t src = ((size_t)i * a.Hkv + g) * a.row_bytes + (size_t)c * 16;
    const size_t dst = (((size_t)b * a.Hkv + g) * kBlock + pos % kBlock) * a.row_bytes + (size_t)c * 16;
    const uint4 v = *reinterpret_cast<const uint4*>((is_v ? a.v_new : a.k_new) + src);
    *reinterpret_cast<uint4*>((is_v ? a.v_cache : a.k_cache) + dst) = v;
}

}  // namespace fea

using namespace fea;

extern "C" int32_t fea_kv_append(const fea_attn_params* p, const void* k_new, const void* v_new, void* k_cache,
                                 void* v_cache, const int32_t* block_tables, int32_t table_stride,
                                 const int32_t* seq_lens, int32_t B, void* hip_stream) {
    if (!p) return fail(FEA_EINVAL, "fea_kv_append: params is NULL");
    if (p->num_kv_heads <= 0 || p->head_dim <= 0 || p->block_size != FEA_BLOCK_TOKENS)
        return fail(FEA_EINVAL, "fea_kv_append: bad shape (num_kv_heads=%d, head_dim=%d, block_size=%d)", p->num_kv_heads, p->head_dim, p->block_size);
    if (p->dtype != FEA_DTYPE_F32 && p->dtype != FEA_DTYPE_BF16) return fail(FEA_EINVAL, "fea_kv_append: unknown dtype %d", p->dtype);
    const int es = p->dtype == FEA_DTYPE_F32 ? 4 : 2;
    if ((p->head_dim * es) % 16 != 0) return fail(FEA_EINVAL, "fea_kv_append: head_dim=%d gives rows that are not a multiple of 16 bytes", p->head_dim);
    if (B < 0 || table_stride < 0) return fail(FEA_EINVAL, "fea_kv_append: negative B or table_stride");
    if (B == 0) return FEA_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_tables || !seq_lens) return fail(FEA_EINVAL, "fea_kv_append: NULL device pointer");
    if (((uintptr_t)k_new & 15) || ((uintptr_t)v_new & 15) || ((uintptr_t)k_cache & 15) || ((uintptr_t)v_cache & 15))
        return fail(FEA_EINVAL, "fea_kv_append: new rows and caches must be 16-byte aligned");
    AppendArgs a;
    a.k_new = static_cast<const char*>(k_new);
    a.v_new = static_cast<const char*>(v_new);
    a.k_cache = static_cast<char*>(k_cache);
    a.v_cache = static_cast<char*>(v_cache);
    a.bt = block_tables;
    a.seq_lens = seq_lens;
    a.stride = table_stride;
    a.B = B;
    a.Hkv = p->num_kv_heads;
    a.row_bytes = p->head_dim * es;
    const long long threads = 2ll * B * a.Hkv * (a.row_bytes / 16);
    if (threads > 0x7FFFFFFFll * 256) return fail(FEA_EINVAL, "fea_kv_append: problem too large");
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FEA_EHIP, "fea_kv_append: launch failed: %s", hipGetErrorString(e));
    return FEA_OK;
}
