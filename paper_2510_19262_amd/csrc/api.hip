// Version and status strings of the railsched C ABI.
#include "common.h"

extern "C" const char *railsched_version(void) { return "railsched 0.2 (gfx950)"; }

extern "C" const char *railsched_strerror(int status)
{
    switch (status) {
        case RAILSCHED_OK: return "ok";
        case RAILSCHED_ERR_INVALID_ARG: return "invalid argument: a size or count is out of range";
        case RAILSCHED_ERR_NULL_PTR: return "null pointer";
        case RAILSCHED_ERR_UNSUPPORTED: return "unsupported: beyond the limits of this library";
        case RAILSCHED_ERR_CAPACITY: return "more chunks than the record arrays hold";
        case RAILSCHED_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case RAILSCHED_ERR_HIP: return "HIP runtime error";
        case RAILSCHED_ERR_SCRATCH: return "the batch needs more scratch memory than the library's static buffer holds";
        default: return "unknown status";
    }
}

// The one call that waits for the device: the chunk count only exists there.
extern "C" int railsched_check_capacity(const int64_t *chunk_off, int32_t batch, const railsched_topo_t *h_topo, int64_t capacity,
                                        int64_t *h_total, void *stream)
{
    using namespace rs;
    if (int rc = check_topo(h_topo)) return rc;
    if (batch < 0 || capacity < 0) return RAILSCHED_ERR_INVALID_ARG;
    if (!chunk_off) return RAILSCHED_ERR_NULL_PTR;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t total = 0;
    if (hipMemcpyAsync(&total, chunk_off + (int64_t)batch * h_topo->nodes, sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return RAILSCHED_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return RAILSCHED_ERR_HIP;
    if (h_total) *h_total = total;
    return total > capacity ? RAILSCHED_ERR_CAPACITY : RAILSCHED_OK;
}
