// Shared by the translation units that implement the C ABI.
#pragma once

namespace msrl {

// Records the message msrl_last_error() returns on this thread and passes `code` through.
int fail(int code, const char* fmt, ...);

}  // namespace msrl
