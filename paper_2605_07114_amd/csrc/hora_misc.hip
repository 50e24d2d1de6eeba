// Status strings and version of the HORA library.
#include "hora.h"

extern "C" const char* hora_status_string(int status) {
    switch (status) {
        case HORA_OK: return "ok";
        case HORA_ERR_INVALID_ARG: return "invalid argument";
        case HORA_ERR_INFEASIBLE: return "budget cannot be placed";
        case HORA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case HORA_ERR_RANGE: return "device data out of range";
        case HORA_ERR_HIP: return "HIP runtime error";
        case HORA_ERR_UNSUPPORTED: return "size not supported";
        default: return "unknown status";
    }
}

extern "C" int hora_version(void) { return 100; }
