// Status strings and version of the fk C ABI.
#include "fk_common.h"

extern "C" const char* fk_status_string(fk_status s) {
    switch (s) {
        case FK_OK: return "ok";
        case FK_ERR_INVALID_ARG: return "invalid argument";
        case FK_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case FK_ERR_WORKSPACE: return "workspace missing or too small";
        case FK_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

extern "C" const char* fk_version(void) { return "fk 0.1 gfx950"; }
