// Aggregate-max and its adjoint (paper Sec. 2.1 lists sum, mean and max as the Aggregate
// choices; the paper's kernels cover the sum).  Edge values play no part.  Both kernels walk the
// CSR of the reordered matrix with one team of G lanes per row, the team covering a tile of
// G * VEC features with full-width vector loads; the row's column indices are fetched once per
// tile by the team and passed round with lane shuffles, four feature-row loads in flight.
//   forward : Y[i][k] = max over the stored entries (i, j) of H[j][k]; arg[i][k] = the smallest
//             such j (columns are ascending, and only a strictly larger value replaces the
//             current one); rows without entries give 0 and -1.  NaN inputs are not supported.
//   adjoint : dH[j][k] = sum of G[i][k] over the rows i with arg[i][k] == j, gathered along
//             row j of the transposed pattern in a fixed order (no atomics, reproducible).
#include "kernels_common.h"

namespace ag {
namespace {

template <int G, int VEC>
__global__ __launch_bounds__(kWG) void k_csr_max(CsrDev A, const float *__restrict__ H, float *__restrict__ Y,
                                                 int32_t *__restrict__ arg, int F, int n)
{
    constexpr int TEAMS = kWG / G, U = 4;
    const int tid = threadIdx.x, team = tid / G, gl = tid % G;
    const int row = xcd_contiguous(blockIdx.x, gridDim.x) * TEAMS + team;
    if (row >= n) return;                               // the whole team leaves together
    const int beg = A.rowptr[row], end = A.rowptr[row + 1];
    for (int f0 = 0; f0 < F; f0 += G * VEC) {
        const int f = f0 + gl * VEC;
        const bool ok = f < F;
        float best[VEC];
        int who[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) { best[j] = 0.f; who[j] = -1; }
        for (int base = beg; base < end; base += G) {
            const int e = base + gl;
            const int c = e < end ? A.col[e] : 0;
            const int cnt = min(G, end - base);
            for (int k0 = 0; k0 < cnt; k0 += U) {
                int ck[U];
                float h[U][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) ck[u] = __shfl(c, (k0 + u) & (G - 1), G);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (k0 + u < cnt && ok) {
                        load_vec<VEC>(H + (size_t)ck[u] * F + f, h[u]);
                    } else {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) h[u][j] = 0.f;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!(k0 + u < cnt)) continue;
#pragma unroll
                    for (int j = 0; j < VEC; ++j)
                        if (who[j] < 0 || h[u][j] > best[j]) { best[j] = h[u][j]; who[j] = ck[u]; }
                }
            }
        }
        if (ok) {
            store_vec<VEC>(Y + (size_t)row * F + f, best);
            if (arg) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) arg[(size_t)row * F + f + j] = who[j];
            }
        }
    }
}

template <int G, int VEC>
__global__ __launch_bounds__(kWG) void k_csr_max_t(CsrDev At, const float *__restrict__ Gm,
                                                   const int32_t *__restrict__ arg, float *__restrict__ dH,
                                                   int F, int n)
{
    constexpr int TEAMS = kWG / G, U = 4;
    const int tid = threadIdx.x, team = tid / G, gl = tid % G;
    const int row = xcd_contiguous(blockIdx.x, gridDim.x) * TEAMS + team;
    if (row >= n) return;
    const int beg = At.rowptr[row], end = At.rowptr[row + 1];
    for (int f0 = 0; f0 < F; f0 += G * VEC) {
        const int f = f0 + gl * VEC;
        const bool ok = f < F;
        float acc[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
        for (int base = beg; base < end; base += G) {
            const int e = base + gl;
            const int c = e < end ? At.col[e] : 0;
            const int cnt = min(G, end - base);
            for (int k0 = 0; k0 < cnt; k0 += U) {
                int ck[U];
                float g[U][VEC], a[U][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) ck[u] = __shfl(c, (k0 + u) & (G - 1), G);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (k0 + u < cnt && ok) {
                        load_vec<VEC>(reinterpret_cast<const float *>(arg) + (size_t)ck[u] * F + f, a[u]);
                        load_vec<VEC>(Gm + (size_t)ck[u] * F + f, g[u]);
                    } else {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) { a[u][j] = __int_as_float(-1); g[u][j] = 0.f; }
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int j = 0; j < VEC; ++j)
                        if (__float_as_int(a[u][j]) == row) acc[j] += g[u][j];
            }
        }
        if (ok) store_vec<VEC>(dH + (size_t)row * F + f, acc);
    }
}

template <int G, int VEC>
int run(bool adjoint, const CsrDev &A, const float *X, const int32_t *arg_in, float *Yo, int32_t *arg_out,
        int F, hipStream_t st)
{
    constexpr int TEAMS = kWG / G;
    const int n = A.n;
    dim3 grid((unsigned)((n + TEAMS - 1) / TEAMS));
    if (adjoint)
        hipLaunchKernelGGL((k_csr_max_t<G, VEC>), grid, dim3(kWG), 0, st, A, X, arg_in, Yo, F, n);
    else
        hipLaunchKernelGGL((k_csr_max<G, VEC>), grid, dim3(kWG), 0, st, A, X, Yo, arg_out, F, n);
    return hip_fail((int)hipGetLastError(), "csr_max launch");
}

template <int VEC>
int pick(bool adjoint, const CsrDev &A, const float *X, const int32_t *arg_in, float *Yo, int32_t *arg_out,
         int F, hipStream_t st)
{
    const int need = F / VEC;                           // vectors per feature row
    if (need > 32) return run<64, VEC>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    if (need > 16) return run<32, VEC>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    if (need > 8) return run<16, VEC>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    if (need > 4) return run<8, VEC>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    return run<4, VEC>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
}

int dispatch(bool adjoint, const CsrDev &A, const float *X, const int32_t *arg_in, float *Yo, int32_t *arg_out,
             int F, void *stream)
{
    if (A.n <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    switch (vec_width(F)) {
    case 4: return pick<4>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    case 2: return pick<2>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    default: return pick<1>(adjoint, A, X, arg_in, Yo, arg_out, F, st);
    }
}

}  // namespace

int launch_csr_max(const CsrDev &A, const float *H, float *Y, int32_t *arg, int32_t F, void *stream)
{
    return dispatch(false, A, H, nullptr, Y, arg, F, stream);
}

int launch_csr_max_t(const CsrDev &At, const float *G, const int32_t *arg, float *dH, int32_t F, void *stream)
{
    return dispatch(true, At, G, arg, dH, nullptr, F, stream);
}

}  // namespace ag
