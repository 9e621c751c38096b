// Error text of the C ABI, shared by the host-side source files.
#pragma once

namespace fmha_host {

extern thread_local char g_err[512];  // what fmha_last_error() returns on this thread

// Formats the message and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace fmha_host
