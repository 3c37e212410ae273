// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/pipefill.h"

namespace pf {

// Records a thread-local message and returns `code` (so call sites can `return pf::fail(...)`).
int32_t fail(int32_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline int32_t esize(int32_t dtype) { return dtype == PF_DTYPE_BF16 ? 2 : 4; }

}  // namespace pf
