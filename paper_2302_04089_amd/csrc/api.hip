// Version and status strings of the C ABI.
#include "common.h"

extern "C" int ziplm_version(void) { return 100; }

extern "C" const char *ziplm_status_string(int status) {
    switch (status) {
        case ZIPLM_OK: return "ok";
        case ZIPLM_ERR_INVALID_ARG: return "invalid argument";
        case ZIPLM_ERR_NOT_PD: return "matrix not positive definite";
        case ZIPLM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case ZIPLM_ERR_DEVICE: return "device error";
        case ZIPLM_ERR_UNSUPPORTED: return "unsupported request";
        default: return "unknown status";
    }
}
