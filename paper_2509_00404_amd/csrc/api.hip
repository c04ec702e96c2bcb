// Status strings and version of the C ABI.
#include "common.h"

extern "C" const char* metis_status_string(int status) {
    switch (status) {
        case METIS_OK: return "ok";
        case METIS_INVALID_ARG: return "invalid argument";
        case METIS_BAD_SHAPE: return "bad shape";
        case METIS_WORKSPACE_TOO_SMALL: return "workspace too small";
        case METIS_HIP_ERROR: return "HIP launch error";
        case METIS_UNSUPPORTED: return "unsupported size or dtype";
        default: return "unknown status";
    }
}

extern "C" int metis_version(void) { return 1; }
