// Status strings and the per-thread record of the last failing HIP call.
#include "bload_common.hpp"

namespace bload {
thread_local int g_last_hip_error = 0;
}

extern "C" const char* bload_status_string(bload_status status)
{
    switch (status) {
        case BLOAD_OK: return "BLOAD_OK";
        case BLOAD_EINVAL: return "BLOAD_EINVAL: invalid argument";
        case BLOAD_ELENGTH: return "BLOAD_ELENGTH: a sequence length is outside [1, t_blk]";
        case BLOAD_EWORKSPACE: return "BLOAD_EWORKSPACE: workspace too small";
        case BLOAD_EALIGN: return "BLOAD_EALIGN: misaligned buffer";
        case BLOAD_EOVERFLOW: return "BLOAD_EOVERFLOW: size beyond the supported range";
        case BLOAD_EHIP: return "BLOAD_EHIP: a HIP runtime call failed";
    }
    return "unknown bload_status";
}

extern "C" int bload_last_hip_error(void) { return bload::g_last_hip_error; }
