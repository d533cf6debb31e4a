// Version and status strings of the MXInt library.
#include "mx_common.h"

extern "C" int32_t mx_version(void) { return 100; }

extern "C" const char* mx_status_string(mx_status s) {
    switch (s) {
        case MX_OK: return "ok";
        case MX_ERR_BAD_ARG: return "bad argument";
        case MX_ERR_UNSUPPORTED: return "unsupported combination";
        case MX_ERR_DEVICE: return "HIP launch failed";
    }
    return "unknown status";
}
