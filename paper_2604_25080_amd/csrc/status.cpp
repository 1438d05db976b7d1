// Status strings and the thread-local error message.
#include "cf_common.h"

namespace cf {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

}  // namespace cf

extern "C" const char* cf_status_str(int status) {
    switch (status) {
        case CF_OK: return "ok";
        case CF_ERR_INVALID_ARG: return "invalid argument";
        case CF_ERR_INVALID_PLAN: return "invalid restoration split";
        case CF_ERR_OUT_OF_PAGES: return "out of KV pages";
        case CF_ERR_HIP: return "HIP runtime error";
        case CF_ERR_UNKNOWN_REQUEST: return "unknown or duplicate request id";
        case CF_ERR_WORKSPACE: return "workspace or context limit exceeded";
        case CF_ERR_UNSUPPORTED: return "unsupported model shape";
        default: return "unknown status";
    }
}

extern "C" const char* cf_last_error(void) { return cf::g_err; }
