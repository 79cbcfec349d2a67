// Names of the status codes of singlequant.h.
#include "singlequant.h"

extern "C" const char *sq_status_string(sq_status status)
{
    switch (status) {
        case SQ_OK: return "ok";
        case SQ_ERR_NULL: return "a required pointer is NULL";
        case SQ_ERR_SHAPE: return "unsupported or inconsistent shape";
        case SQ_ERR_INDEX: return "Givens index out of range or i == j";
        case SQ_ERR_ALIGN: return "pointer or leading dimension is misaligned";
        case SQ_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}
