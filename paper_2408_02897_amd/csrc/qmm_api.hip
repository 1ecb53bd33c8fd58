// Small host-only entry points of the C ABI.
#include "qmm.h"

extern "C" const char* qmm_status_string(qmm_status s)
{
    switch (s) {
    case QMM_OK: return "ok";
    case QMM_ERR_NULL: return "required pointer is NULL";
    case QMM_ERR_SHAPE: return "invalid shape or stride";
    case QMM_ERR_ENUM: return "invalid enum value";
    case QMM_ERR_ALIGN: return "alignment rule violated";
    case QMM_ERR_UNSUPPORTED: return "not supported by this build";
    case QMM_ERR_WORKSPACE: return "workspace missing or too small";
    case QMM_ERR_LAUNCH: return "kernel launch failed";
    case QMM_ERR_LIMIT: return "input exceeds a fixed capacity of the call";
    }
    return "unknown status";
}

extern "C" int qmm_version(void) { return 100; }
