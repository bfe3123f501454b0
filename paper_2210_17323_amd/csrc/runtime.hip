// Library-wide helpers: version, thread-local error text.
#include "common.h"

#include <cstring>

namespace gptq {

static thread_local char g_err[512] = "";

int fail_v(int code, const char* fmt, va_list ap) {
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    return code;
}

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

}  // namespace gptq

extern "C" int gptq_version(void) { return 100; }
extern "C" const char* gptq_last_error(void) { return gptq::g_err; }
