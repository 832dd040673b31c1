// Status strings and ABI version of libmassv_verify.
#include "common.h"

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

extern "C" int massv_abi_version(void) { return 1; }
