// Dense-based kernel (paper Sec. 3.2 "Dense-based kernel"): a work-group takes one community's
// adjacency block in dense form and multiplies it with the block's feature rows as a small
// GEMM, which equals the aggregate-sum over the block's edges.  Here the GEMM runs on the
// fp32 matrix instruction v_mfma_f32_32x32x2_f32 with full fp32 operands (no reduced-mantissa
// mode).  Unit-weight blocks are stored as 128 x 128 bit maps and expanded to 0/1 operands in
// registers; weighted blocks carry their values pre-arranged in operand order.
// Note: a dense product multiplies non-neighbours by zero, so non-finite feature values in a
// block spread to every row of that block; finite inputs are required.
#include "kernels_common.h"

namespace ag {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Operand / result layout of the 32x32x2 fp32 instruction for lane l:
//   A operand = A[l & 31][l >> 5], B operand = B[l >> 5][l & 31],
//   result register r holds D[8 (r / 4) + 4 (l >> 5) + (r & 3)][l & 31].
template <int NT, bool WEIGHTED>
__global__ __launch_bounds__(kWG) void k_block_dense(BlocksDev B, const float *__restrict__ H,
                                                     float *__restrict__ Y, int F)
{
    constexpr int FT = 32 * NT;
    __shared__ float sH[kMaxBlock * FT];
    const int tid = threadIdx.x;
    const int slot = xcd_contiguous(blockIdx.x, gridDim.x);   // neighbouring blocks share an XCD (L2)
    const int b = B.list_dense[slot];
    const int r0 = B.blk_ptr[b], nr = B.blk_ptr[b + 1] - r0;
    const int f0 = blockIdx.y * FT;
    const int kpad = (nr + 31) & ~31;                 // source rows rounded up, extras are zero
    if (F % 4 == 0) stage_tile<FT, 4>(H, F, r0, nr, kpad, f0, sH, tid);
    else if (F % 2 == 0) stage_tile<FT, 2>(H, F, r0, nr, kpad, f0, sH, tid);
    else stage_tile<FT, 1>(H, F, r0, nr, kpad, f0, sH, tid);
    __syncthreads();
    const int w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    if (32 * w >= nr) return;
    const uint4 bits = *reinterpret_cast<const uint4 *>(B.bitmap + ((size_t)slot * kMaxBlock + 32 * w + lo) * 4);
    const float *tile = WEIGHTED ? B.tiles + (size_t)slot * (kMaxBlock * kMaxBlock) + w * 4096 + l : nullptr;
    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    const int nwords = kpad >> 5;
    for (int wd = 0; wd < nwords; ++wd) {
        const uint32_t word = (wd == 0) ? bits.x : (wd == 1) ? bits.y : (wd == 2) ? bits.z : bits.w;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int step = wd * 16 + j;
            const int k = 2 * step + hi;
            float a;
            if constexpr (WEIGHTED) a = tile[step * 64];
            else a = ((word >> (2 * j + hi)) & 1u) ? 1.f : 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float bv = sH[k * FT + 32 * t + lo];
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[t], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int f = f0 + 32 * t + lo;
        if (f >= F) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3);
            if (i < nr) Y[(size_t)(r0 + i) * F + f] = acc[t][r];
        }
    }
}

template <int NT>
int run(const BlocksDev &B, const float *H, float *Y, int F, hipStream_t st)
{
    dim3 grid(B.n_dense, (F + 32 * NT - 1) / (32 * NT));
    if (B.tiles)
        hipLaunchKernelGGL((k_block_dense<NT, true>), grid, dim3(kWG), 0, st, B, H, Y, F);
    else
        hipLaunchKernelGGL((k_block_dense<NT, false>), grid, dim3(kWG), 0, st, B, H, Y, F);
    return hip_fail((int)hipGetLastError(), "block_dense launch");
}

}  // namespace

int launch_block_dense(const BlocksDev &B, const float *H, float *Y, int32_t F, void *stream)
{
    if (B.n_dense <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    if (F <= 32) return run<1>(B, H, Y, F, st);
    if (F <= 64) return run<2>(B, H, Y, F, st);
    return run<4>(B, H, Y, F, st);
}

}  // namespace ag
