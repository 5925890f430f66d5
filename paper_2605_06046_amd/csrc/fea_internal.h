// Internal glue between the host bookkeeping and the HIP launch code.
#pragma once
#include <cstdarg>
#include <cstdint>

namespace fea {
// Stores a printf-style message for fea_last_error() and returns `code`.
int32_t fail(int32_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}  // namespace fea
