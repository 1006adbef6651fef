// Thread-local error text shared by the library's translation units.
#pragma once
namespace relaygr {
// Stores a printf-formatted message as the calling thread's last error and returns code.
int fail(int code, const char* fmt, ...);
}  // namespace relaygr
