// Status texts of the C ABI.
#include "common.h"

extern "C" const char* chipmunk_status_string(int32_t status) {
    switch (status) {
        case CHIPMUNK_OK: return "ok";
        case CHIPMUNK_ERR_NULL: return "a required pointer is NULL";
        case CHIPMUNK_ERR_SHAPE: return "a size or scalar argument is out of range";
        case CHIPMUNK_ERR_ALIGN: return "a pointer or leading dimension is misaligned";
        case CHIPMUNK_ERR_UNSUPPORTED: return "unsupported parameter (E, c, D, F or act)";
        case CHIPMUNK_ERR_WORKSPACE: return "workspace missing or too small";
        case CHIPMUNK_ERR_LAUNCH: return "the HIP runtime refused the launch";
        default: return "unknown status";
    }
}
