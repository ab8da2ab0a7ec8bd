// Status strings and version of the C ABI.
#include "common.h"

extern "C" const char* specvlm_status_string(int status)
{
    switch (status) {
        case SPECVLM_OK:           return "ok";
        case SPECVLM_EINVAL:       return "invalid argument";
        case SPECVLM_EUNSUPPORTED: return "unsupported shape";
        case SPECVLM_EWORKSPACE:   return "workspace missing, misaligned or too small";
        case SPECVLM_ELAUNCH:      return "kernel launch failed";
        default:                   return "unknown status";
    }
}

extern "C" int specvlm_version(void) { return 100; }
