// Status strings and version of the C ABI.
#include "common.h"
#include <math.h>

extern "C" const char* metis_status_string(int status) {
    switch (status) {
        case METIS_OK: return "ok";
        case METIS_INVALID_ARG: return "invalid argument";
        case METIS_BAD_SHAPE: return "bad shape";
        case METIS_WORKSPACE_TOO_SMALL: return "workspace too small";
        case METIS_HIP_ERROR: return "HIP launch error";
        case METIS_UNSUPPORTED: return "unsupported size or dtype";
        case METIS_SCRATCH_TOO_SMALL: return "input exceeds the built-in scratch array";
        default: return "unknown status";
    }
}

extern "C" int metis_version(void) { return 2; }

// Smallest power of two g with 6 * 448 * g >= amax (host arithmetic only).  frexp gives amax = m 2^e with
// 0.5 <= m < 1; 2688 = 0.65625 * 2^12, so g = 2^(e - 12) covers amax when m <= 0.65625 and 2^(e - 11) otherwise.
extern "C" float metis_tensor_scale(float amax) {
    if (!(amax > 0.0f) || amax > 3.0e38f) return 1.0f;
    int e = 0;
    const float m = frexpf(amax, &e);
    return ldexpf(1.0f, m <= 0.65625f ? e - 12 : e - 11);
}

MetisProfSlot g_metis_prof[METIS_PROF_COUNT] = {};

extern "C" int metis_profile_events(int kernel_id, void** start, void** stop, int n) {
    if (kernel_id < 0 || kernel_id >= METIS_PROF_COUNT || n < 0) return METIS_INVALID_ARG;
    if (n > 0 && (!start || !stop)) return METIS_INVALID_ARG;
    MetisProfSlot& p = g_metis_prof[kernel_id];
    p.start = (hipEvent_t*)start;
    p.stop = (hipEvent_t*)stop;
    p.n = n;
    p.next = 0;
    return METIS_OK;
}
