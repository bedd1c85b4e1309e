// Version and error strings of the ARRoL C ABI.
#include "common.h"

extern "C" int arrol_version(void) { return 200; }

extern "C" const char* arrol_error_string(int code) {
    switch (code) {
        case ARROL_OK: return "ok";
        case ARROL_EINVAL: return "invalid argument (null pointer, bad shape or misaligned base)";
        case ARROL_EWORKSPACE: return "workspace missing, misaligned or too small";
        case ARROL_EHIP: return "the HIP runtime refused a kernel launch";
        default: return "unknown error code";
    }
}
