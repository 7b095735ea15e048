// Status strings and version of libkvcomm.
#include "kvcomm.h"

extern "C" const char *kvcomm_status_string(int status)
{
    switch (status) {
        case KVCOMM_OK: return "ok";
        case KVCOMM_EINVAL: return "invalid argument";
        case KVCOMM_EUNSUPPORTED: return "unsupported shape or dtype";
        case KVCOMM_EWORKSPACE: return "workspace missing, misaligned or too small";
        case KVCOMM_EHIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

extern "C" int kvcomm_version(void) { return 200; }  // 0.2.0: batched 8-bit update, static-scratch weights, confined attention
