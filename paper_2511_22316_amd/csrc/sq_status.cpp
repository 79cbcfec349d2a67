// Names of the status codes of singlequant.h, and the store behind sq_debug_set_option.
#include "singlequant.h"

#include <atomic>

namespace sq {

static std::atomic<int32_t> debug_options[SQ_DEBUG_OPTION_COUNT] = {};

// Current value of a debug option (0 unless sq_debug_set_option has set it).
int32_t debug_option(sq_debug_option option) { return debug_options[option].load(std::memory_order_relaxed); }

}  // namespace sq

extern "C" sq_status sq_debug_set_option(sq_debug_option option, int32_t value)
{
    if ((int)option < 0 || (int)option >= SQ_DEBUG_OPTION_COUNT) return SQ_ERR_SHAPE;
    sq::debug_options[option].store(value, std::memory_order_relaxed);
    return SQ_OK;
}

extern "C" const char *sq_status_string(sq_status status)
{
    switch (status) {
        case SQ_OK: return "ok";
        case SQ_ERR_NULL: return "a required pointer is NULL";
        case SQ_ERR_SHAPE: return "unsupported or inconsistent shape";
        case SQ_ERR_INDEX: return "Givens index out of range or i == j";
        case SQ_ERR_ALIGN: return "pointer or leading dimension is misaligned";
        case SQ_ERR_LAUNCH: return "HIP launch failed";
        case SQ_ERR_TIMEOUT: return "a workgroup of sq_decode_layer gave up waiting for the rotated tokens";
    }
    return "unknown status";
}
