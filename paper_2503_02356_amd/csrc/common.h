// Shared host-side helpers of the library: error reporting.
#pragma once
#include <cstdarg>
#include <cstdio>

#include "chunkflow.h"

namespace cf {

// Records a printf-style message for cf_last_error() on this thread and returns `code`.
int fail(int code, const char *fmt, ...);

}  // namespace cf
