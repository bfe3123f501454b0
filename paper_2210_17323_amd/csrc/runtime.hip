// Library-wide helpers: version, thread-local error text, the look-ahead stream.
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

int lookahead_get(Lookahead** out) {
    constexpr int MAXDEV = 64;
    static thread_local Lookahead table[MAXDEV];
    int dev = 0;
    GPTQ_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAXDEV) return fail(GPTQ_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    Lookahead& l = table[dev];
    if (!l.stream) {
        hipStream_t st = nullptr;
        GPTQ_HIP_CHECK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
        for (hipEvent_t& e : l.ev) {
            const hipError_t err = hipEventCreateWithFlags(&e, hipEventDisableTiming);
            if (err != hipSuccess) {            // give back what was created: the next call starts from nothing
                for (hipEvent_t& d : l.ev) { if (d) (void)hipEventDestroy(d); d = nullptr; }
                (void)hipStreamDestroy(st);
                return fail(GPTQ_ERR_HIP, "hipEventCreateWithFlags failed: %s", hipGetErrorString(err));
            }
        }
        l.stream = st;
    }
    *out = &l;
    return GPTQ_OK;
}

}  // namespace gptq

extern "C" int gptq_version(void) { return 100; }
extern "C" const char* gptq_last_error(void) { return gptq::g_err; }
