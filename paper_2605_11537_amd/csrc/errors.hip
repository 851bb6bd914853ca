// Thread-local error text behind moe_last_error().
#include <stdarg.h>

#include "common.h"

namespace moe {
static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
}  // namespace moe

extern "C" const char *moe_last_error(void) { return moe::g_err; }
extern "C" int moe_version(void) { return 200; }

#ifndef MOE_BUILD_ID
#define MOE_BUILD_ID "unknown"
#endif
extern "C" const char *moe_build_id(void) { return MOE_BUILD_ID; }
