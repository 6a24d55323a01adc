// Thread-local last-error text and the version query.
#include <cstdarg>
#include <cstdio>

#include "common.h"

namespace {
thread_local char g_error[512] = "";
}

namespace rlhf {

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return code;
}

void clear_error()
{
    g_error[0] = '\0';
}

}  // namespace rlhf

extern "C" const char *rlhf_last_error_string(void)
{
    return g_error;
}

extern "C" int rlhf_version(void)
{
    return 1;
}
