// Thread-local last-error string and version of the fise library.
#include <cstdarg>
#include <cstdio>
#include "../../include/fise.h"

namespace fise {
static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
}
int fail(int code, const char* fmt, ...) {
    va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
    return code;
}
}  // namespace fise

extern "C" const char* fise_last_error(void) { return fise::g_err; }
extern "C" int fise_version(void) { return 1; }
