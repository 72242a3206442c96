// Version and status strings of the railsched C ABI.
#include "common.h"

extern "C" const char *railsched_version(void) { return "railsched 0.1 (gfx950)"; }

extern "C" const char *railsched_strerror(int status)
{
    switch (status) {
        case RAILSCHED_OK: return "ok";
        case RAILSCHED_ERR_INVALID_ARG: return "invalid argument: a size or count is out of range";
        case RAILSCHED_ERR_NULL_PTR: return "null pointer";
        case RAILSCHED_ERR_UNSUPPORTED: return "unsupported: beyond the limits of this build";
        case RAILSCHED_ERR_CAPACITY: return "record arrays smaller than the chunk count";
        case RAILSCHED_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case RAILSCHED_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}
