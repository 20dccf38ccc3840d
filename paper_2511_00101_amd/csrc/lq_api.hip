// Entry points that launch nothing: status strings.
#include "lq_common.h"

extern "C" const char* lora_status_string(lq_status status)
{
    switch (status) {
        case LQ_OK: return "ok";
        case LQ_ERR_INVALID_ARG: return "invalid argument";
        case LQ_ERR_UNSUPPORTED: return "unsupported shape, alignment, rank or adapter count";
        case LQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LQ_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}
