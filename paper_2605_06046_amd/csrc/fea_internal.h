// Internal glue between the host bookkeeping and the HIP launch code.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <new>

#include "../../include/fea.h"

namespace fea {
// Stores a printf-style message for fea_last_error() and returns `code`.
int32_t fail(int32_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// fea_decode_attention and fea_decode_workspace_bytes behind the C entry points (the
// variant that brings its own workspace calls them too).
int32_t decode_workspace_bytes(const fea_attn_params* p, int32_t B, int32_t table_stride, size_t* out_bytes, const char* who);
int32_t decode_impl(const fea_attn_params* p, const void* q, const void* k_cache, const void* v_cache,
                    const int32_t* block_tables, int32_t table_stride, const int32_t* seq_lens, int32_t B,
                    void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

// Runs the body of an entry point so that no C++ exception crosses the C boundary:
// memory exhaustion on the host becomes FEA_ENOMEM, anything else FEA_EINVAL.
template <class F> int32_t guarded(const char* who, F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(FEA_ENOMEM, "%s: out of host memory", who);
    } catch (...) {
        return fail(FEA_EINVAL, "%s: unexpected exception", who);
    }
}
}  // namespace fea
