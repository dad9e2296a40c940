// Status strings and build information.
#include "common.h"

extern "C" const char* lamp_status_string(lamp_status s) {
    switch (s) {
        case LAMP_OK: return "ok";
        case LAMP_ERR_NULL: return "a required pointer is NULL";
        case LAMP_ERR_SHAPE: return "bad or mismatching shape";
        case LAMP_ERR_ALIGN: return "pointer or stride not aligned";
        case LAMP_ERR_DTYPE: return "unknown or mismatching dtype";
        case LAMP_ERR_WORKSPACE: return "workspace missing or too small";
        case LAMP_ERR_UNSUPPORTED: return "unsupported request";
        case LAMP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* lamp_build_info(void) { return "liblamp 0.1 gfx950"; }
