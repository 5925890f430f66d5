// Measurement aid: what this GPU delivers to the KV sweep's own fetch path.
//
// The sweep is a gather-scan bound by HBM bandwidth; its roofline is quoted against
// the published peak, and next to it belongs what the box at hand can actually
// stream.  This kernel reads a buffer exactly once the way the sweep does - one
// single-wave workgroup per SIMD, 16 KB tiles made of four 4 KB chunks (one KV block
// of one head each), fetched global -> LDS with two tiles in flight - and nothing
// else, so its rate is the ceiling for any sweep built on that path.
#include <hip/hip_runtime.h>

#include "../../include/fea.h"
#include "fea_internal.h"

namespace fea {

constexpr uint32_t kChunk = 4096;
constexpr uint32_t kTile = 4 * kChunk;

__device__ __forceinline__ const char* uniform_ptr(const char* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return reinterpret_cast<const char*>(lo | (hi << 32));
}

// Four wave-wide 16-byte-per-lane loads (one 4 KB chunk) into LDS at `lds` (wave-uniform).
__device__ __forceinline__ void fetch_chunk(const char* base, uint32_t lane_off, uint32_t lds) {
    asm volatile(
        "s_nop 4\n\t"
        "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\t"
        "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024\n\t"
        "s_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048\n\t"
        "s_mov_b32 m0, %5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072"
        :: "v"(lane_off), "s"(base), "s"(lds), "s"(lds + 1024), "s"(lds + 2048), "s"(lds + 3072)
        : "memory", "m0");
}

// n_chunks is a power of two; chunk c of the stream sits at ((c * mult) mod n_chunks) * 4 KB,
// mult odd, hence every chunk is read exactly once.  mult == 1 is a linear sweep.
__global__ __launch_bounds__(64) void stream_read_kernel(const char* buf, uint32_t n_chunks, uint32_t mult, uint32_t* sink) {
    __shared__ __attribute__((aligned(1024))) char stage[2 * kTile];
    const uint32_t lds = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)stage);
    const uint32_t lane_off = threadIdx.x * 16;
    const uint32_t n_tiles = n_chunks / 4;
    uint32_t it = 0;
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x, ++it) {
        const uint32_t st = lds + (it & 1) * kTile;
#pragma unroll
        for (uint32_t x = 0; x < 4; ++x) {
            const uint32_t c = ((t * 4 + x) * mult) & (n_chunks - 1);
            fetch_chunk(uniform_ptr(buf + (size_t)c * kChunk), lane_off, st + x * kChunk);
        }
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");   // the tile before this one has landed
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (reinterpret_cast<const uint32_t*>(stage)[threadIdx.x] == 0x9E3779B9u && sink) sink[0] = 1;   // keeps the stage observable
}

}  // namespace fea

using namespace fea;

extern "C" int32_t fea_stream_read_gbs(const void* buffer, size_t bytes, int32_t scattered, int32_t repeats, void* hip_stream,
                                       double* gbs) {
    if (!buffer || !gbs) return fail(FEA_EINVAL, "fea_stream_read_gbs: NULL pointer");
    if (((uintptr_t)buffer & 15) != 0) return fail(FEA_EINVAL, "fea_stream_read_gbs: buffer must be 16-byte aligned");
    if (repeats < 1 || repeats > 1000) return fail(FEA_EINVAL, "fea_stream_read_gbs: repeats=%d out of range", repeats);
    uint64_t n_chunks = 1;
    while (n_chunks * 2 * kChunk <= bytes && n_chunks < (1ull << 30)) n_chunks *= 2;
    if (n_chunks < 1024) return fail(FEA_EINVAL, "fea_stream_read_gbs: at least 4 MiB are needed, %zu bytes given", bytes);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    float ms = 0.f;
    if (e == hipSuccess) {
        const uint32_t mult = scattered ? 2654435761u : 1u;
        hipLaunchKernelGGL(stream_read_kernel, dim3(4 * cus), dim3(64), 0, st, static_cast<const char*>(buffer), (uint32_t)n_chunks, mult,
                           (uint32_t*)nullptr);   // warm-up: page tables, clocks
        e = hipEventRecord(e0, st);
        for (int r = 0; r < repeats; ++r)
            hipLaunchKernelGGL(stream_read_kernel, dim3(4 * cus), dim3(64), 0, st, static_cast<const char*>(buffer), (uint32_t)n_chunks,
                               mult, (uint32_t*)nullptr);
        if (e == hipSuccess) e = hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess) e = hipGetLastError();
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(FEA_EHIP, "fea_stream_read_gbs: %s", hipGetErrorString(e));
    if (!(ms > 0.f)) return fail(FEA_EHIP, "fea_stream_read_gbs: no time elapsed");
    *gbs = (double)n_chunks * kChunk * repeats / (ms * 1e-3) / 1e9;
    return FEA_OK;
}
