// Internal helpers shared by the translation units of libcanz.so (not part of the ABI).
#pragma once
#include <cstdarg>
#include <cstdint>

namespace canz {

// Records a printf-style message for canz_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace canz
