// COO-based kernel (paper Sec. 3.2 "COO-based kernel", Algorithm 1): one lane group per edge,
// every feature of the source row is added to the destination row with an atomic add.  No
// shared memory, maximal parallelism, atomic destination updates; a candidate for the
// inter-community subgraph only.  Algorithm 1 is weight-free; here the edge value multiplies
// the source features (unit weights reproduce it exactly).  The sum order is not fixed, so
// results vary in the last bits from run to run.
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include "kernels_common.h"

namespace ag {
namespace {

template <int G, int VEC>
__global__ __launch_bounds__(kWG) void k_coo_edges(CsrDev A, const float *__restrict__ H,
                                                   float *__restrict__ Y, int F, int n_edges)
{
    constexpr int TEAMS = kWG / G;
    const int tid = threadIdx.x, team = tid / G, gl = tid % G;
    const int e = (blockIdx.x * TEAMS + team);
    if (e >= n_edges) return;
    const int f = blockIdx.y * (G * VEC) + gl * VEC;
    if (f >= F) return;
    const int dst = A.row[e], src = A.col[e];
    const float a = A.val ? A.val[e] : 1.f;
    float h[VEC];
    load_vec<VEC>(H + (size_t)src * F + f, h);
    float *y = Y + (size_t)dst * F + f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) unsafeAtomicAdd(y + j, a * h[j]);
}

template <int G, int VEC>
void run(const CsrDev &A, const float *H, float *Y, int F, int n_edges, hipStream_t st)
{
    const int teams = kWG / G;
    dim3 grid((n_edges + teams - 1) / teams, (F + G * VEC - 1) / (G * VEC));
    hipLaunchKernelGGL((k_coo_edges<G, VEC>), grid, dim3(kWG), 0, st, A, H, Y, F, n_edges);
}

}  // namespace

int launch_coo(const CsrDev &A, const float *H, float *Y, int32_t F, int32_t zero_from, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (!A.row) { set_error("COO form was not built for this matrix"); return AG_ERR_UNSUPPORTED; }
    int rc = launch_fill_zero((int64_t)(A.n - zero_from) * F, Y + (size_t)zero_from * F, stream);
    if (rc) return rc;
    const int n_edges = A.nnz;
    if (n_edges == 0) return AG_OK;
    const int VEC = vec_width(F);
    const int need = (F + VEC - 1) / VEC, cap = (VEC == 4) ? 32 : 64;
    int G = 4;
    while (G < need && G < cap) G <<= 1;
#define AG_CASE(g, v) if (G == g && VEC == v) { run<g, v>(A, H, Y, F, n_edges, st); return hip_fail((int)hipGetLastError(), "coo launch"); }
    AG_CASE(4, 4) AG_CASE(8, 4) AG_CASE(16, 4) AG_CASE(32, 4)
    AG_CASE(4, 2) AG_CASE(8, 2) AG_CASE(16, 2) AG_CASE(32, 2) AG_CASE(64, 2)
    AG_CASE(4, 1) AG_CASE(8, 1) AG_CASE(16, 1) AG_CASE(32, 1) AG_CASE(64, 1)
#undef AG_CASE
    set_error("coo: no kernel shape for this feature width");
    return AG_ERR_UNSUPPORTED;
}

}  // namespace ag
