// Error reporting shared by the translation units of libscheinfer (host-only header).
#pragma once

namespace si {
// Stores the formatted text as the calling thread's last error (read by si_last_error) and returns `code`.
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}  // namespace si
