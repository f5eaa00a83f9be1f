// Stand-ins for everything the host plan code links against but never calls in AG_FLAG_HOST_ONLY
// mode: the kernel launchers of the .hip files and the few HIP runtime calls of api.cpp.  With
// them the plan code (ingest, transpose, reorder, split, formats, statistics, export) builds as a
// plain host program that can run under AddressSanitizer / UBSan without a GPU runtime.
// A call to any of them means that host-only mode touched the device path: abort loudly.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#include "ag_internal.h"

#define TOUCHED() do { std::fprintf(stderr, "host-only build reached %s\n", __func__); std::abort(); } while (0)

extern "C" {
hipError_t hipMalloc(void **, size_t) { TOUCHED(); }
hipError_t hipFree(void *) { TOUCHED(); }
hipError_t hipMemcpy(void *, const void *, size_t, hipMemcpyKind) { TOUCHED(); }
hipError_t hipDeviceSynchronize(void) { TOUCHED(); }
hipError_t hipEventCreate(hipEvent_t *) { TOUCHED(); }
hipError_t hipEventDestroy(hipEvent_t) { TOUCHED(); }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { TOUCHED(); }
hipError_t hipEventSynchronize(hipEvent_t) { TOUCHED(); }
hipError_t hipEventElapsedTime(float *, hipEvent_t, hipEvent_t) { TOUCHED(); }
const char *hipGetErrorString(hipError_t) { return "stub"; }
}

namespace ag {
int launch_csr_rows(const CsrDev &, const float *, float *, int32_t, int32_t, int32_t, int32_t, int, void *) { TOUCHED(); }
int launch_csr_long(const CsrDev &, const float *, float *, int32_t, float *, int32_t, void *) { TOUCHED(); }
int launch_coo(const CsrDev &, const float *, float *, int32_t, int32_t, void *) { TOUCHED(); }
int launch_block_sparse(const BlocksDev &, const int32_t *, int32_t, const CsrDev *, const float *, float *, int32_t, void *) { TOUCHED(); }
int launch_block_dense(const BlocksDev &, const CsrDev *, const float *, float *, int32_t, int, void *) { TOUCHED(); }
int launch_csr_max(const CsrDev &, const float *, float *, int32_t *, int32_t, void *) { TOUCHED(); }
int launch_csr_max_t(const CsrDev &, const float *, const int32_t *, float *, int32_t, void *) { TOUCHED(); }
int launch_permute_rows(const int32_t *, int64_t, int32_t, const float *, float *, bool, void *) { TOUCHED(); }
int launch_axpy(int64_t, float, const float *, float *, void *) { TOUCHED(); }
}  // namespace ag
