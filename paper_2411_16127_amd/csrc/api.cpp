// Status strings, thread-local error text and version of libdfgnn.
#include <cstdarg>
#include <cstdio>

#include "../../include/dfgnn.h"

namespace dfgnn {
static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}
void clear_error() { g_error[0] = '\0'; }
}  // namespace dfgnn

extern "C" const char* dfgnn_status_string(int status) {
    switch (status) {
    case DFGNN_OK: return "DFGNN_OK";
    case DFGNN_EINVAL: return "DFGNN_EINVAL: invalid argument";
    case DFGNN_EUNSUPPORTED: return "DFGNN_EUNSUPPORTED: shape, dtype or alignment not supported";
    case DFGNN_EWORKSPACE: return "DFGNN_EWORKSPACE: caller-provided buffer too small";
    case DFGNN_EHIP: return "DFGNN_EHIP: HIP runtime error";
    default: return "unknown dfgnn status";
    }
}

extern "C" const char* dfgnn_last_error(void) { return dfgnn::g_error; }

extern "C" int dfgnn_version(int* major, int* minor) {
    if (major) *major = 0;
    if (minor) *minor = 1;
    return DFGNN_OK;
}
