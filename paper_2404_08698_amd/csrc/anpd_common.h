// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "anpd.h"

namespace anpd {

// Thread-local message behind anpd_last_error().
char *error_buffer();
constexpr int kErrorBufferBytes = 512;

inline int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), kErrorBufferBytes, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace anpd
