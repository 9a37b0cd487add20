// Error text and version of the C ABI.
#include <string.h>

#include "st_internal.h"

namespace st {
static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}
const char* get_error() { return g_error; }
}  // namespace st

extern "C" const char* st_last_error(void) { return st::get_error(); }
extern "C" int32_t st_version(void) { return 1; }
