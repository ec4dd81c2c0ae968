// Version and status strings of libsquat.
#include "squat.h"

extern "C" int squat_version(void) { return 100; /* 0.1.0 */ }

extern "C" const char* squat_strerror(int status) {
    switch (status) {
        case SQUAT_OK: return "ok";
        case SQUAT_E_NULLPTR: return "a required pointer is NULL";
        case SQUAT_E_BADSHAPE: return "unsupported shape, size or stride";
        case SQUAT_E_BADDTYPE: return "unsupported dtype";
        case SQUAT_E_ALIGN: return "pointer or stride not aligned as required";
        case SQUAT_E_WORKSPACE: return "workspace missing or too small";
        case SQUAT_E_HIP: return "HIP runtime error at launch";
        case SQUAT_E_BADVALUE: return "lambda must be >= 0 (or +inf)";
    }
    return "unknown status";
}
