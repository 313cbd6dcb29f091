// Version and status strings of libw4a4, and the timing hook.
#include "common.hpp"

extern "C" const char *w4a4_version(void) { return "w4a4 0.1 (gfx950)"; }

extern "C" const char *w4a4_status_string(int status) {
    switch (status) {
        case W4A4_OK: return "ok";
        case W4A4_ERR_INVALID_ARG: return "invalid argument";
        case W4A4_ERR_UNSUPPORTED_SHAPE: return "unsupported shape or alignment";
        case W4A4_ERR_WORKSPACE: return "workspace missing or too small";
        case W4A4_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

namespace w4a4 {
KernelTimer &kernel_timer() {
    static thread_local KernelTimer t;
    return t;
}
}  // namespace w4a4

extern "C" int w4a4_time_next_gemm(void *start_event, void *stop_event) {
    w4a4::KernelTimer &t = w4a4::kernel_timer();
    t.start = reinterpret_cast<hipEvent_t>(start_event);
    t.stop = reinterpret_cast<hipEvent_t>(stop_event);
    return W4A4_OK;
}
