// Library-level entry points: version, status strings, last launch error.
#include "etv_common.h"

namespace etv {
thread_local int32_t g_last_hip_error = 0;
}

extern "C" const char *etv_version(void) { return "eagletv 0.1 (gfx950)"; }

extern "C" int32_t etv_last_hip_error(void) { return etv::g_last_hip_error; }

extern "C" const char *etv_status_string(int32_t status) {
    switch (status) {
        case ETV_OK: return "ok";
        case ETV_ERR_INVALID_ARG: return "invalid argument";
        case ETV_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case ETV_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case ETV_ERR_HIP: return "HIP launch error";
        case ETV_ERR_UNIMPLEMENTED: return "not implemented";
        default: return "unknown status";
    }
}
