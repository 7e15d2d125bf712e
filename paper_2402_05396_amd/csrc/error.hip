// Thread-local error text behind taser_last_error().
#include <cstdarg>
#include <cstdio>

#include "taser_internal.h"

namespace {
thread_local char g_error[512] = "";
}

int taser_fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

int taser_fail_hip(hipError_t e, const char* what) {
    (void)hipGetLastError();   // do not leave the error behind for the caller's next HIP call
    return taser_fail(e == hipErrorOutOfMemory ? TASER_E_OOM : TASER_E_HIP, "%s failed: %s", what,
                      hipGetErrorString(e));
}

extern "C" const char* taser_last_error(void) { return g_error; }
