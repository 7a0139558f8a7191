// Shared by the translation units behind the C ABI.
#pragma once
#include "hcl.h"

namespace hcl {
// Stores a printf-style message where hcl_last_error() finds it (thread-local) and returns `st`.
hcl_status_t fail(hcl_status_t st, const char* fmt, ...);
}  // namespace hcl
