// CSR-based kernel for the intra-community subgraph (paper Sec. 3.2, second half of "CSR-based
// kernel"): one work-group per community (diagonal block).  The block's source rows coincide
// with its destination rows, so their feature rows are loaded once into LDS and every entry
// of the block reads from there; the feature dimension is tiled when it exceeds the LDS tile.
// The topology of the block uses one-byte block-local column indices.
// With FUSED the same lanes go on to add their rows' inter-community entries (gathered from
// global memory), so each output row is written exactly once and no merge pass is needed.
#include "kernels_common.h"

namespace ag {
namespace {

template <int G, int VEC, bool FUSED>
__global__ __launch_bounds__(kWG) void k_block_sparse(BlocksDev B, const int32_t *__restrict__ list,
                                                      CsrDev R, const float *__restrict__ H,
                                                      float *__restrict__ Y, int F)
{
    constexpr int FT = G * VEC, TEAMS = kWG / G, U = 4;
    __shared__ float sH[kMaxBlock * FT];
    const int tid = threadIdx.x;
    const int b = list[blockIdx.x];
    const int r0 = B.blk_ptr[b], nr = B.blk_ptr[b + 1] - r0;
    const int f0 = blockIdx.y * FT;
    for (int idx = tid; idx < nr * G; idx += kWG) {
        const int r = idx / G, g = idx % G, f = f0 + g * VEC;
        float h[VEC];
        if (f < F) {
            load_vec<VEC>(H + (size_t)(r0 + r) * F + f, h);
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) h[j] = 0.f;
        }
        store_vec<VEC>(sH + r * FT + g * VEC, h);
    }
    __syncthreads();
    const int team = tid / G, gl = tid % G;
    const int f = f0 + gl * VEC;
    const bool fok = f < F;
    for (int r = team; r < nr; r += TEAMS) {
        const int row = r0 + r;
        const int beg = B.i_rowptr[row], end = B.i_rowptr[row + 1];
        float acc[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
        for (int base = beg; base < end; base += G) {
            const int e = base + gl;
            int c = 0;
            float v = 0.f;
            if (e < end) {
                c = B.i_col8[e];
                v = B.i_val ? B.i_val[e] : 1.f;
            }
            const int cnt = min(G, end - base);
            for (int k0 = 0; k0 < cnt; k0 += U) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int kk = k0 + u;
                    const int ck = __shfl(c, kk & (G - 1), G);
                    const float vk = __shfl(v, kk & (G - 1), G);
                    if (kk < cnt) {
                        float h[VEC];
                        load_vec<VEC>(sH + ck * FT + gl * VEC, h);
#pragma unroll
                        for (int j = 0; j < VEC; ++j) acc[j] = fmaf(vk, h[j], acc[j]);
                    }
                }
            }
        }
        if constexpr (FUSED) {
            const int rb = R.rowptr[row], re = R.rowptr[row + 1];
            if (re - rb <= kLongThresh)
                team_row_gather<G, G, VEC>(R.col, R.val, rb, re, H, F, f, fok, gl, acc);
        }
        if (fok) store_vec<VEC>(Y + (size_t)row * F + f, acc);
    }
}

template <int G, int VEC>
int run(const BlocksDev &B, const int32_t *list, int nlist, const CsrDev *rem, const float *H,
        float *Y, int F, hipStream_t st)
{
    dim3 grid(nlist, (F + G * VEC - 1) / (G * VEC));
    if (rem)
        hipLaunchKernelGGL((k_block_sparse<G, VEC, true>), grid, dim3(kWG), 0, st, B, list, *rem, H, Y, F);
    else
        hipLaunchKernelGGL((k_block_sparse<G, VEC, false>), grid, dim3(kWG), 0, st, B, list, CsrDev(), H, Y, F);
    return hip_fail((int)hipGetLastError(), "block_sparse launch");
}

}  // namespace

int launch_block_sparse(const BlocksDev &B, const int32_t *list, int32_t nlist, const CsrDev *fused_rem,
                        const float *H, float *Y, int32_t F, void *stream)
{
    if (nlist <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    const int VEC = (F % 4 == 0) ? 4 : 1;
    const int need = (F + VEC - 1) / VEC, cap = (VEC == 4) ? 32 : 64;
    int G = 4;
    while (G < need && G < cap) G <<= 1;
#define AG_CASE(g, v) if (G == g && VEC == v) return run<g, v>(B, list, nlist, fused_rem, H, Y, F, st);
    AG_CASE(4, 4) AG_CASE(8, 4) AG_CASE(16, 4) AG_CASE(32, 4)
    AG_CASE(4, 1) AG_CASE(8, 1) AG_CASE(16, 1) AG_CASE(32, 1) AG_CASE(64, 1)
#undef AG_CASE
    set_error("block_sparse: no kernel shape for this feature width");
    return AG_ERR_UNSUPPORTED;
}

}  // namespace ag
