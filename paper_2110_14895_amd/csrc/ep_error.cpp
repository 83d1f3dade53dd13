#include "ep_error.h"

#include <cstdarg>
#include <cstdio>

namespace {
thread_local char g_err[512] = "";
}

ep_status ep_fail(ep_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

void ep_clear_error() { g_err[0] = '\0'; }

extern "C" const char *ep_last_error(void) { return g_err; }

extern "C" const char *ep_status_string(ep_status s)
{
    switch (s) {
    case EP_OK: return "EP_OK";
    case EP_ERR_INVALID_ARG: return "EP_ERR_INVALID_ARG";
    case EP_ERR_UNSUPPORTED: return "EP_ERR_UNSUPPORTED";
    case EP_ERR_OOM: return "EP_ERR_OOM";
    case EP_ERR_HIP: return "EP_ERR_HIP";
    case EP_ERR_INFEASIBLE: return "EP_ERR_INFEASIBLE";
    }
    return "EP_ERR_UNKNOWN";
}
