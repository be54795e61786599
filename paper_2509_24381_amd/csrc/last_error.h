// The thread-local message behind rs_last_error(), shared by the library's translation units (not exported).
#pragma once
#include "../../include/rserve_prefill.h"

// Stores a printf-style message for rs_last_error() and returns `st`.
__attribute__((visibility("hidden"))) rs_status rs_internal_fail(rs_status st, const char* fmt, ...)
    __attribute__((format(printf, 2, 3)));
