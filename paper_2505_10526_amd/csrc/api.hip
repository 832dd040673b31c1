// Status strings and ABI version of libmassv_verify.
#include "kernels.h"

extern "C" const char* massv_status_string(int status) {
    switch (status) {
        case MASSV_OK: return "ok";
        case MASSV_EINVAL: return "invalid argument";
        case MASSV_EUNSUPPORTED: return "shape or dtype not supported by the gfx950 kernels";
        case MASSV_EWORKSPACE: return "workspace missing or too small";
        case MASSV_ELAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}

extern "C" int massv_abi_version(void) { return 3; }

namespace massv {
TraceRequest& trace_request() {
    static thread_local TraceRequest req = {-1, nullptr, nullptr};
    return req;
}
}  // namespace massv

extern "C" int massv_trace_kernel(int kernel_id, void* start_event, void* stop_event) {
    massv::TraceRequest& t = massv::trace_request();
    if (kernel_id < 0) { t.kid = -1; return MASSV_OK; }
    if (kernel_id > MASSV_K_LINEAR || !start_event || !stop_event) return MASSV_EINVAL;
    t.kid = kernel_id; t.start = (hipEvent_t)start_event; t.stop = (hipEvent_t)stop_event;
    return MASSV_OK;
}
