// An aggregation entry point for callers that cannot allocate: the scratch memory of the long-row
// kernels (partial sums of row segments, CSR-based kernel of Sec. 3.2 with rows split across
// wavefronts) lives in a static device array instead of memory obtained at plan creation.
#include <hip/hip_runtime.h>

#include <atomic>

#include "ag_internal.h"

namespace {

// One copy per GPU, held from the first use of the library on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[AG_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU

// Device address of this GPU's copy of `scratch` (looked up once per device; in host code the
// array's name is only a handle for the lookup, never an address to hand to a kernel).
int scratch_address(void **out)
{
    int dev = -1;
    int rc = ag::hip_fail((int)hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    if (dev < 0 || dev >= kMaxDevices) {
        ag::set_error("device index out of range");
        return AG_ERR_UNSUPPORTED;
    }
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        rc = ag::hip_fail((int)hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc) return rc;
        if (!ptr) {
            ag::set_error("the static scratch buffer has no device address");
            return AG_ERR_HIP;
        }
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return AG_OK;
}

}  // namespace

extern "C" int ag_aggregate_static(ag_plan *p, const float *H_dev, float *Y_dev, void *hip_stream)
{
    void *ptr = nullptr;
    int rc = scratch_address(&ptr);
    if (rc) return rc;
    // every segment's partial row is written before it is read, so nothing has to be cleared
    return ag::aggregate_settled(p, H_dev, Y_dev, (float *)ptr, (size_t)AG_STATIC_SCRATCH_BYTES, hip_stream);
}
