// Thread-local error text behind laser_last_error().
#include <cstdarg>
#include <cstdio>

#include "../../include/laser.h"

namespace laser {
static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
}  // namespace laser

extern "C" const char* laser_last_error(void) { return laser::g_err; }
extern "C" const char* laser_version(void) { return "laser-gfx950 0.1"; }
