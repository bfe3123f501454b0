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

namespace {
constexpr int MAXDEV = 64;
thread_local Lookahead table[MAXDEV];
}

int lookahead_get(Lookahead** out) {
    int dev = 0;
    GPTQ_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAXDEV) return fail(GPTQ_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    Lookahead& l = table[dev];
    if (!l.stream) {
        hipStream_t st = nullptr, st2 = nullptr, st3 = nullptr;
        GPTQ_HIP_CHECK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
        hipError_t err = hipStreamCreateWithFlags(&st2, hipStreamNonBlocking);
        if (err == hipSuccess) err = hipStreamCreateWithFlags(&st3, hipStreamNonBlocking);
        for (hipEvent_t& e : l.ev) {
            if (err == hipSuccess) err = hipEventCreateWithFlags(&e, hipEventDisableTiming);
        }
        if (err != hipSuccess) {                // give back what was created: the next call starts from nothing
            for (hipEvent_t& d : l.ev) { if (d) (void)hipEventDestroy(d); d = nullptr; }
            if (st3) (void)hipStreamDestroy(st3);
            if (st2) (void)hipStreamDestroy(st2);
            (void)hipStreamDestroy(st);
            return fail(GPTQ_ERR_HIP, "creating the helper streams and events failed: %s", hipGetErrorString(err));
        }
        l.stream = st;
        l.stream2 = st2;
        l.stream3 = st3;
    }
    *out = &l;
    return GPTQ_OK;
}

}  // namespace gptq

extern "C" int gptq_version(void) { return 100; }

extern "C" int gptq_release_thread_resources(void) {
    using namespace gptq;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return GPTQ_OK;      // no usable device: nothing can have been created
    if (dev < 0 || dev >= MAXDEV) return GPTQ_OK;
    Lookahead& l = table[dev];
    if (!l.stream) return GPTQ_OK;                      // nothing was created on this thread for this device
    hipError_t err = hipSuccess;
    for (hipStream_t st : {l.stream, l.stream2, l.stream3}) {
        // every call joins the helpers back into the caller's stream, but their last event records may still be pending
        hipError_t e = hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipStreamDestroy(st);
        if (e != hipSuccess && err == hipSuccess) err = e;
    }
    for (hipEvent_t& e : l.ev) {
        if (e) { const hipError_t d = hipEventDestroy(e); if (d != hipSuccess && err == hipSuccess) err = d; }
        e = nullptr;
    }
    l = Lookahead{};
    if (err != hipSuccess) return fail(GPTQ_ERR_HIP, "releasing the helper streams and events failed: %s", hipGetErrorString(err));
    return GPTQ_OK;
}
extern "C" const char* gptq_last_error(void) { return gptq::g_err; }
