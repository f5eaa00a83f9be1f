// Dense-based kernel (paper Sec. 3.2 "Dense-based kernel"): a work-group takes one community's
// adjacency block in dense form and multiplies it with the block's feature rows as a small
// GEMM, which equals the aggregate-sum over the block's edges.  Here the GEMM runs on the
// fp32 matrix instruction v_mfma_f32_32x32x2_f32 with full fp32 operands (no reduced-mantissa
// mode).  Unit-weight blocks are stored as 128 x 128 bit maps and expanded to 0/1 operands in
// registers; weighted blocks carry their values pre-arranged in operand order.
// A second form for unit-weight blocks runs on the bf16 matrix instruction at fp32 accuracy: the
// 0/1 adjacency operand is exact in bf16 and every fp32 feature value is cut into three bf16
// pieces that add up to it exactly, so three bf16 products accumulated in fp32 give the fp32
// result (the mixed-precision direction the paper names as future work in Sec. 3.2, without
// giving up accuracy).
// Note: a dense product multiplies non-neighbours by zero, so non-finite feature values in a
// block spread to every row of that block; finite inputs are required.
#include "kernels_common.h"

namespace ag {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Write-out shared by both forms.  Result register r of lane l holds D[8 (r / 4) + 4 (l >> 5)
// + (r & 3)][l & 31] of the wave's 32 x 32 tile.  Plain: every lane stores its values (32
// consecutive features per row and instruction).  FUSED: the tile goes to LDS (the operand tile
// is no longer needed) and the rows are finished with their remainder entries, one store per row.
template <int NT, int VEC, bool FUSED, bool SCALED>
__device__ __forceinline__ void write_out(const floatx16 (&acc)[NT], bool wave_has_rows, float *sOut,
                                          RemainderRows<32 * NT, VEC> &rem, const CsrDev &R,
                                          const float *__restrict__ H, float *__restrict__ Y,
                                          int F, int r0, int nr, int f0, int tid,
                                          const float *__restrict__ out_scale)
{
    constexpr int FT = 32 * NT;
    const int w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    float osc[SCALED ? 16 : 1];                         // factored values: the factor of each of the lane's 16 rows
    if constexpr (SCALED) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3);
            osc[r] = (out_scale && i < nr) ? out_scale[r0 + i] : 1.f;
        }
    }
    if constexpr (!FUSED) {
        if (!wave_has_rows) return;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int f = f0 + 32 * t + lo;
            if (f >= F) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (i < nr) Y[(size_t)(r0 + i) * F + f] = SCALED ? acc[t][r] * osc[SCALED ? r : 0] : acc[t][r];
            }
        }
    } else {
        __syncthreads();                                // every wave is done with the operand tile
        if (wave_has_rows) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3);
                    sOut[i * FT + 32 * t + lo] = SCALED ? acc[t][r] * osc[SCALED ? r : 0] : acc[t][r];
                }
        }
        __syncthreads();
        rem.finish(R, sOut, r0, H, Y, F);
    }
}

// Operand / result layout of the 32x32x2 fp32 instruction for lane l:
//   A operand = A[l & 31][l >> 5], B operand = B[l >> 5][l & 31],
//   result register r holds D[8 (r / 4) + 4 (l >> 5) + (r & 3)][l & 31].
// All global loads that do not depend on the staged tile (bit map, remainder row pointers and
// first topology chunks) are issued before the staging, so they overlap with it.
template <int NT, int VEC, bool WEIGHTED, bool FUSED, bool SCALED>
__global__ __launch_bounds__(kWG) void k_block_dense(BlocksDev B, CsrDev R, const float *__restrict__ H,
                                                     float *__restrict__ Y, int F)
{
    constexpr int FT = 32 * NT;
    static_assert(!FUSED || NT <= 2, "the fused write-out handles tiles of up to 64 features");
    __shared__ float sH[kMaxBlock * FT];
    const int tid = threadIdx.x;
    const int slot = xcd_contiguous(blockIdx.x, gridDim.x);   // neighbouring blocks share an XCD (L2)
    const int b = B.list_dense[slot];
    const int r0 = B.blk_ptr[b], nr = B.blk_ptr[b + 1] - r0;
    const int f0 = blockIdx.y * FT;
    const int kpad = (nr + 31) & ~31;                 // source rows rounded up, extras are zero
    const int w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const bool has_rows = 32 * w < nr;
    const uint4 bits = *reinterpret_cast<const uint4 *>(B.bitmap + ((size_t)slot * kMaxBlock + 32 * w + lo) * 4);
    RemainderRows<FT, VEC> rem;
    if constexpr (FUSED) rem.prepare(R, r0, nr, F, f0, tid);
    stage_tile<FT, VEC>(H, F, r0, nr, kpad, f0, sH, tid, SCALED ? B.in_scale : nullptr);
    __syncthreads();
    if (!FUSED && !has_rows) return;
    const float *tile = WEIGHTED ? B.tiles + (size_t)slot * (kMaxBlock * kMaxBlock) + w * 4096 + l : nullptr;
    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    const int nwords = has_rows ? kpad >> 5 : 0;
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
    write_out<NT, VEC, FUSED, SCALED>(acc, has_rows, sH, rem, R, H, Y, F, r0, nr, f0, tid, B.out_scale);
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// h = p[0] + p[1] + p[2] exactly, each piece having at most 8 significant bits (the upper half
// of an fp32 word is a bf16 number): cut off the low 16 bits, subtract (exact), repeat.  Pieces
// below the normal range may flush; the error is then far below the absolute tolerance.
__device__ __forceinline__ void cut3(float h, uint32_t (&p)[3])
{
    p[0] = __float_as_uint(h) & 0xffff0000u;
    const float r1 = h - __uint_as_float(p[0]);
    p[1] = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(p[1]);
    p[2] = __float_as_uint(r2) & 0xffff0000u;
}

// Stage rows [r0, r0+nr) x columns [f0, f0+FT) of H as three bf16 tiles, transposed:
// sT[(piece * FT + f) * kKS + j] holds piece `piece` of H[r0 + j][f0 + f]; rows j >= nr and
// columns beyond F are zero.  A thread handles two consecutive rows so it writes whole 32-bit
// words.  kKS (bf16 elements per tile row) keeps 16-byte operand reads of 8 lanes on distinct banks.
constexpr int kKS = kMaxBlock + 8;

template <int FT, int VEC>
__device__ __forceinline__ void stage_tile_bf16x3(const float *__restrict__ H, int F, int r0, int nr, int f0,
                                                  uint32_t *sT, int tid, const float *__restrict__ scale)
{
    constexpr int UPR = FT / VEC;
    constexpr int ITER = (kMaxBlock / 2 * UPR) / kWG;
    static_assert((kMaxBlock / 2 * UPR) % kWG == 0, "tile must divide among the threads");
    float h[ITER][2][VEC];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = tid + it * kWG, jp = idx / UPR, ff = f0 + (idx % UPR) * VEC;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (2 * jp + q < nr && ff < F) {
                load_vec<VEC>(H + (size_t)(r0 + 2 * jp + q) * F + ff, h[it][q]);
                if (scale) {                            // factored values: the source row's factor, in fp32, before the cut
                    const float sc = scale[r0 + 2 * jp + q];
#pragma unroll
                    for (int j = 0; j < VEC; ++j) h[it][q][j] *= sc;
                }
            } else {
#pragma unroll
                for (int j = 0; j < VEC; ++j) h[it][q][j] = 0.f;
            }
        }
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = tid + it * kWG, jp = idx / UPR, fl = (idx % UPR) * VEC;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            uint32_t a[3], b[3];
            cut3(h[it][0][j], a);
            cut3(h[it][1][j], b);
#pragma unroll
            for (int s = 0; s < 3; ++s) sT[((s * FT + fl + j) * kKS) / 2 + jp] = (a[s] >> 16) | b[s];
        }
    }
}

// Operand / result layout of v_mfma_f32_32x32x16_bf16 for lane l (8 bf16 per operand register
// group): A = A[l & 31][8 (l >> 5) + 0..7], B = B[8 (l >> 5) + 0..7][l & 31], result as above.
// A is the adjacency block (rows = destinations, 8 consecutive sources = one byte of the row's
// bit map), B the transposed feature pieces.
template <int NT, int VEC, bool FUSED, bool SCALED>
__global__ __launch_bounds__(kWG) void k_block_dense_bf16x3(BlocksDev B, CsrDev R, const float *__restrict__ H,
                                                            float *__restrict__ Y, int F)
{
    constexpr int FT = 32 * NT;
    __shared__ __attribute__((aligned(16))) uint32_t sT[3 * FT * kKS / 2];
    static_assert(3 * FT * kKS / 2 >= kMaxBlock * FT, "the result tile reuses the operand tile");
    const int tid = threadIdx.x;
    const int slot = xcd_contiguous(blockIdx.x, gridDim.x);
    const int b = B.list_dense[slot];
    const int r0 = B.blk_ptr[b], nr = B.blk_ptr[b + 1] - r0;
    const int f0 = blockIdx.y * FT;
    const int w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const bool has_rows = 32 * w < nr;
    const uint4 bits = *reinterpret_cast<const uint4 *>(B.bitmap + ((size_t)slot * kMaxBlock + 32 * w + lo) * 4);
    RemainderRows<FT, VEC> rem;
    if constexpr (FUSED) rem.prepare(R, r0, nr, F, f0, tid);
    stage_tile_bf16x3<FT, VEC>(H, F, r0, nr, f0, sT, tid, SCALED ? B.in_scale : nullptr);
    __syncthreads();
    if (!FUSED && !has_rows) return;
    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    const int nsteps = has_rows ? (nr + 15) >> 4 : 0;   // 16 source rows per instruction
    for (int s16 = 0; s16 < nsteps; ++s16) {
        const int byte_idx = 2 * s16 + hi;              // sources 16 s16 + 8 hi .. + 7
        const uint32_t word = (byte_idx < 4) ? bits.x : (byte_idx < 8) ? bits.y : (byte_idx < 12) ? bits.z : bits.w;
        const uint32_t m = (word >> ((byte_idx & 3) * 8)) & 0xffu;
        uint4 av;                                       // bit -> bf16 1.0 (0x3f80) or 0, two per word
        av.x = ((m & 1u) ? 0x3f80u : 0u) | ((m & 2u) ? 0x3f800000u : 0u);
        av.y = ((m & 4u) ? 0x3f80u : 0u) | ((m & 8u) ? 0x3f800000u : 0u);
        av.z = ((m & 16u) ? 0x3f80u : 0u) | ((m & 32u) ? 0x3f800000u : 0u);
        av.w = ((m & 64u) ? 0x3f80u : 0u) | ((m & 128u) ? 0x3f800000u : 0u);
        const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int pc = 2; pc >= 0; --pc) {           // smallest pieces first
                const uint4 bv = *reinterpret_cast<const uint4 *>(
                    sT + ((pc * FT + 32 * t + lo) * kKS + 16 * s16 + 8 * hi) / 2);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bv), acc[t], 0, 0, 0);
            }
        }
    }
    write_out<NT, VEC, FUSED, SCALED>(acc, has_rows, reinterpret_cast<float *>(sT), rem, R, H, Y, F, r0, nr, f0, tid, B.out_scale);
}

// ---- launchers -----------------------------------------------------------------------------
template <int NT, int VEC, bool FUSED>
int run_bf16x3(const BlocksDev &B, const CsrDev &R, const float *H, float *Y, int F, hipStream_t st)
{
    dim3 grid(B.n_dense, (F + 32 * NT - 1) / (32 * NT));
    if (B.in_scale || B.out_scale)                      // factored values: a separate instantiation keeps the plain path lean
        hipLaunchKernelGGL((k_block_dense_bf16x3<NT, VEC, FUSED, true>), grid, dim3(kWG), 0, st, B, R, H, Y, F);
    else
        hipLaunchKernelGGL((k_block_dense_bf16x3<NT, VEC, FUSED, false>), grid, dim3(kWG), 0, st, B, R, H, Y, F);
    return hip_fail((int)hipGetLastError(), "block_dense_bf16x3 launch");
}

template <int NT, int VEC, bool FUSED>
int run_f32(const BlocksDev &B, const CsrDev &R, const float *H, float *Y, int F, hipStream_t st)
{
    dim3 grid(B.n_dense, (F + 32 * NT - 1) / (32 * NT));
    if (B.tiles)                                        // weighted and not factored
        hipLaunchKernelGGL((k_block_dense<NT, VEC, true, FUSED, false>), grid, dim3(kWG), 0, st, B, R, H, Y, F);
    else if (B.in_scale || B.out_scale)
        hipLaunchKernelGGL((k_block_dense<NT, VEC, false, FUSED, true>), grid, dim3(kWG), 0, st, B, R, H, Y, F);
    else
        hipLaunchKernelGGL((k_block_dense<NT, VEC, false, FUSED, false>), grid, dim3(kWG), 0, st, B, R, H, Y, F);
    return hip_fail((int)hipGetLastError(), "block_dense launch");
}

template <int VEC, bool FUSED>
int pick(const BlocksDev &B, const CsrDev &R, const float *H, float *Y, int F, int variant, hipStream_t st)
{
    if (variant == AG_K_BLOCK_DENSE_BF16X3)
        return (F <= 32) ? run_bf16x3<1, VEC, FUSED>(B, R, H, Y, F, st) : run_bf16x3<2, VEC, FUSED>(B, R, H, Y, F, st);
    if (F <= 32) return run_f32<1, VEC, FUSED>(B, R, H, Y, F, st);
    if (FUSED || F <= 64) return run_f32<2, VEC, FUSED>(B, R, H, Y, F, st);
    if constexpr (!FUSED) return run_f32<4, VEC, false>(B, R, H, Y, F, st);
    return AG_ERR_INVALID;                              // not reached
}

template <bool FUSED>
int pick_vec(const BlocksDev &B, const CsrDev &R, const float *H, float *Y, int F, int variant, hipStream_t st)
{
    switch (vec_width(F)) {
    case 4: return pick<4, FUSED>(B, R, H, Y, F, variant, st);
    case 2: return pick<2, FUSED>(B, R, H, Y, F, variant, st);
    default: return pick<1, FUSED>(B, R, H, Y, F, variant, st);
    }
}

}  // namespace

int launch_block_dense(const BlocksDev &B, const CsrDev *fused_rem, const float *H, float *Y, int32_t F,
                       int variant, void *stream)
{
    if (B.n_dense <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    if (variant == AG_K_BLOCK_DENSE_BF16X3 && B.tiles) {
        set_error("the bf16x3 dense kernel takes unit-weight or factored blocks only");
        return AG_ERR_UNSUPPORTED;
    }
    if (fused_rem) return pick_vec<true>(B, *fused_rem, H, Y, F, variant, st);
    return pick_vec<false>(B, CsrDev(), H, Y, F, variant, st);
}

}  // namespace ag
