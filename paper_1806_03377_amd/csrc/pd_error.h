// Error reporting shared by the host-side sources: records the message pd_last_error() returns (thread-local)
// and hands back the status code, so that a caller can write `return pd::fail(PD_EINVAL, "...", ...)`.
#pragma once

namespace pd {
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}
