// Cumulative chunk hashes on the device: the chunk-parallel formulation of the
// prefix hash computation (appendix "Prefix Hash Computation", Algorithm 2).
// Every 16-token chunk is hashed on its own into a leaf (the parallel phase, one
// thread per chunk), then the leaves of a request are chained in order (the
// sequential phase, O(C) per request, one thread).  One workgroup per request;
// leaves pass through LDS in tiles so the chaining thread never waits on global
// memory.  The arithmetic is the one documented at fea_chunk_hashes; the host
// function and this kernel must agree bit for bit.
#include <hip/hip_runtime.h>

#include "../../include/fea.h"
#include "fea_internal.h"

namespace fea {

namespace {

constexpr unsigned long long kGammaD = 0x9E3779B97F4A7C15ull;
constexpr unsigned long long kH0D = 0x243F6A8885A308D3ull;
constexpr int kChunk = FEA_BLOCK_TOKENS;
constexpr int kLeafTile = 2048;     // leaves staged per pass: 16 KB of LDS

__device__ __forceinline__ unsigned long long mixd(unsigned long long x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

struct HashArgs {
    const int32_t* tokens;
    const int64_t* tok_offsets;
    const int64_t* hash_offsets;
    unsigned long long* hashes;
    int64_t n_tokens, n_hashes;
};

__global__ __launch_bounds__(256) void chunk_hash_kernel(HashArgs a) {
    __shared__ unsigned long long s_leaf[kLeafTile];
    const int i = blockIdx.x, tid = threadIdx.x;
    const int64_t t0 = a.tok_offsets[i], t1 = a.tok_offsets[i + 1];
    if (t0 < 0 || t1 < t0 || t1 > a.n_tokens) return;            // inconsistent offsets: the row is skipped
    const int64_t T = t1 - t0, C = (T + kChunk - 1) / kChunk;
    const int64_t h0 = a.hash_offsets[i];
    if (h0 < 0 || h0 + C > a.n_hashes) return;
    const int32_t* tok = a.tokens + t0;
    unsigned long long h = kH0D;                                  // carried by thread 0 across tiles
    for (int64_t base = 0; base < C; base += kLeafTile) {
        const int n = (int)(C - base < kLeafTile ? C - base : kLeafTile);
        for (int c = tid; c < n; c += 256) {                      // parallel phase: independent leaves
            const int64_t first = (base + c) * kChunk;
            const int len = (int)(T - first < kChunk ? T - first : kChunk);
            unsigned long long x = mixd(kGammaD ^ (unsigned long long)len);
            for (int j = 0; j < len; ++j) x = mixd(x ^ (unsigned long long)(uint32_t)tok[first + j]);
            s_leaf[c] = x;
        }
        __syncthreads();
        if (tid == 0) {                                           // sequential phase: the chain
            for (int c = 0; c < n; ++c) {
                h = mixd(mixd(h + kGammaD) ^ s_leaf[c]);
                s_leaf[c] = h;
            }
        }
        __syncthreads();
        for (int c = tid; c < n; c += 256) a.hashes[h0 + base + c] = s_leaf[c];
        __syncthreads();
    }
}

}  // namespace
}  // namespace fea

using namespace fea;

extern "C" int32_t fea_chunk_hashes_device(const int32_t* tokens, int64_t n_tokens, const int64_t* tok_offsets,
                                           int32_t B, const int64_t* hash_offsets, uint64_t* hashes,
                                           int64_t n_hashes, void* hip_stream) {
    if (B < 0 || n_tokens < 0 || n_hashes < 0) return fail(FEA_EINVAL, "fea_chunk_hashes_device: negative size");
    if (B == 0) return FEA_OK;
    if (!tok_offsets || !hash_offsets || (n_tokens > 0 && !tokens) || (n_hashes > 0 && !hashes))
        return fail(FEA_EINVAL, "fea_chunk_hashes_device: NULL device pointer");
    HashArgs a;
    a.tokens = tokens;
    a.tok_offsets = tok_offsets;
    a.hash_offsets = hash_offsets;
    a.hashes = reinterpret_cast<unsigned long long*>(hashes);
    a.n_tokens = n_tokens;
    a.n_hashes = n_hashes;
    hipLaunchKernelGGL(chunk_hash_kernel, dim3((unsigned)B), dim3(256), 0, static_cast<hipStream_t>(hip_stream), a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FEA_EHIP, "fea_chunk_hashes_device: launch failed: %s", hipGetErrorString(e));
    return FEA_OK;
}
