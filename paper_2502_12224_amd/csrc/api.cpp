// Error string, version.
#include <cstdarg>
#include <cstdio>
#include "../../include/fate.h"

namespace fate {
static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
}  // namespace fate

extern "C" const char* fate_last_error(void) { return fate::g_err; }
extern "C" const char* fate_version(void) { return "libfate 0.1 (gfx950)"; }
