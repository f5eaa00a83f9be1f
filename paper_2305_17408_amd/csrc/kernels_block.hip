// CSR-based kernel for the intra-community subgraph (paper Sec. 3.2, second half of "CSR-based
// kernel"): one work-group per community (diagonal block).  The block's source rows coincide
// with its destination rows, so their feature rows are loaded once into LDS and every entry
// of the block reads from there; the feature dimension is tiled when it exceeds the LDS tile.
// The topology of the block uses one-byte block-local column indices.
// With FUSED the same lanes go on to add their rows' inter-community entries (gathered from
// global memory), so each output row is written exactly once and no merge pass is needed.
//
// Mapping: a team of G lanes owns a contiguous run of the block's rows; a lane owns NV vectors
// of VEC floats, vector v at feature offset (v*G + lane)*VEC of the tile, so every load of a
// team is one contiguous G*VEC-float piece of a feature row.  The team's entries are one
// contiguous range of the topology arrays and are streamed through a 3-deep ring of register
// chunks (G entries each, fetched ahead of use) independent of the row boundaries; the row
// pointers of the team's rows sit in its lanes.  The kernel is bound by vector-ALU issue, not
// by LDS or HBM, which is why a lane carries NV = 2 vectors for wide features (half the
// shuffles and address arithmetic per FMA).
#include <algorithm>
#include <atomic>

#include "kernels_common.h"

namespace ag {
namespace {

constexpr int kWantGroups = 4096;   // work-groups a block-sparse launch should have before blocks stop being shared out

// Entries lo..hi-1 of a register chunk (lane k of the team holds entry k); feature rows come
// from the LDS tile.  Entries beyond hi belong to other rows: they are redirected to the zero
// row of the tile with weight 0, so nothing of them reaches the sum (not even 0 * Inf).
template <int G, int NV, int VEC, int MAXR>
__device__ __forceinline__ void chunk_range_lds(int c, float v, int lo, int hi, const float *sH, int gl,
                                                float (&acc)[NV][VEC])
{
    constexpr int FT = G * VEC * NV, U = 4;
    for (int k0 = lo; k0 < hi; k0 += U) {
        int row[U];
        float w[U], h[U][NV][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = k0 + u < hi;
            const int ck = __shfl(c, (k0 + u) & (G - 1), G);
            const float vk = __shfl(v, (k0 + u) & (G - 1), G);
            row[u] = ok ? ck : MAXR;                    // the zero row behind the tile
            w[u] = ok ? vk : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < NV; ++q) load_vec<VEC>(sH + row[u] * FT + (q * G + gl) * VEC, h[u][q]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[q][j] = fmaf(w[u], h[u][q][j], acc[q][j]);
    }
}

template <int G, int NV, int VEC, bool FUSED, bool SCALED, int MAXR>
__global__ __launch_bounds__(kWG) void k_block_sparse(BlocksDev B, const int32_t *__restrict__ list,
                                                      CsrDev R, const float *__restrict__ H,
                                                      float *__restrict__ Y, int F, int parts)
{
    constexpr int FT = G * VEC * NV, TEAMS = kWG / G;
    static_assert(kMaxBlock / TEAMS + 1 <= G, "row pointers of a team must fit in its lanes");
    static_assert(MAXR % kMaxBlock == 0 && MAXR <= 256, "one-byte block-local columns");
    extern __shared__ float sH[];                       // (MAXR + 1) x FT: feature tile + a zero row
    const int tid = threadIdx.x;
    // `parts` work-groups share a block (each stages the whole tile and serves its share of the rows):
    // more work-groups when a plan has few blocks.  Neighbouring ids -> the same block, the same XCD (L2).
    const int slot = xcd_contiguous(blockIdx.x, gridDim.x);
    const int b = list[slot / parts];
    const int r0 = B.blk_ptr[b], nr = B.blk_ptr[b + 1] - r0;
    const int part = slot % parts;
    const int pr0 = (int)((long)nr * part / parts), pr1 = (int)((long)nr * (part + 1) / parts);   // this work-group's rows
    const int f0 = blockIdx.y * FT;
    const int team = tid / G, gl = tid % G;
    const int f = f0 + gl * VEC;                        // first feature of vector 0
    bool fok[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) fok[q] = f + q * G * VEC < F;
    // The block's rows are served in runs of kMaxBlock (blocks of up to 128 rows: one run); within a
    // run every team takes a contiguous share of the rows.  State of the team for the current run:
    int first, myrows, irp, ie1, iq, ic0, ic1, ic2;
    float osc, iv0, iv1, iv2;
    int rrp = 0, re1 = 0, rq = 0, rc0 = 0, rc1 = 0, rc2 = 0;
    float rv0 = 0.f, rv1 = 0.f, rv2 = 0.f;
    auto ld_i = [&](int e, int &c, float &v) {
        c = 0;
        v = 0.f;
        if (e < ie1) {
            c = B.i_col8[e];
            v = B.i_val ? B.i_val[e] : 1.f;
        }
    };
    auto ld_r = [&](int e, int &c, float &v) {
        c = 0;
        v = 0.f;
        if (e < re1) {
            c = R.col[e];
            v = R.val ? R.val[e] : 1.f;
        }
    };
    auto begin_run = [&](int c0) {                      // row pointers and the first topology chunks of a run
        const int cn = min(kMaxBlock, pr1 - c0);
        const int rpt = (cn + TEAMS - 1) / TEAMS;       // rows per team
        first = c0 + min(team * rpt, cn);
        myrows = min(rpt, c0 + cn - first);
        irp = B.i_rowptr[r0 + first + min(gl, myrows)];
        // factored values: lane gl keeps the output factor of the team's row gl (fetched with the row pointers)
        osc = (SCALED && B.out_scale && gl < myrows) ? B.out_scale[r0 + first + gl] : 1.f;
        ie1 = __shfl(irp, myrows, G);
        iq = __shfl(irp, 0, G);                         // entry held by lane 0 of ring chunk 0
        ld_i(iq + gl, ic0, iv0);
        ld_i(iq + G + gl, ic1, iv1);
        ld_i(iq + 2 * G + gl, ic2, iv2);
        if constexpr (FUSED) {
            rrp = R.rowptr[r0 + first + min(gl, myrows)];
            re1 = __shfl(rrp, myrows, G);
            rq = __shfl(rrp, 0, G);
            ld_r(rq + gl, rc0, rv0);
            ld_r(rq + G + gl, rc1, rv1);
            ld_r(rq + 2 * G + gl, rc2, rv2);
        }
    };
    begin_run(pr0);
    stage_tile<FT, VEC, MAXR>(H, F, r0, nr, nr, f0, sH, tid, SCALED ? B.in_scale : nullptr);
    for (int j = tid; j < FT; j += kWG) sH[MAXR * FT + j] = 0.f;
    __syncthreads();
    for (int c0 = pr0;;) {
    for (int i = 0; i < myrows; ++i) {
        const int row = r0 + first + i;
        float acc[NV][VEC];
#pragma unroll
        for (int q = 0; q < NV; ++q)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[q][j] = 0.f;
        {
            const int rb = __shfl(irp, i, G), re = __shfl(irp, i + 1, G);
            int k = rb;
            while (k < re) {
                if (k >= iq + G) {                      // move on to the next chunk of the ring
                    ic0 = ic1; iv0 = iv1; ic1 = ic2; iv1 = iv2;
                    iq += G;
                    ld_i(iq + 2 * G + gl, ic2, iv2);
                }
                const int hi = min(re, iq + G) - iq;
                chunk_range_lds<G, NV, VEC, MAXR>(ic0, iv0, k - iq, hi, sH, gl, acc);
                k = iq + hi;
            }
        }
        if (SCALED && B.out_scale) {                    // factored values: the row's factor on its block sum
            const float sc = __shfl(osc, i, G);
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[q][j] *= sc;
        }
        if constexpr (FUSED) {
            const int rb = __shfl(rrp, i, G), re = __shfl(rrp, i + 1, G);
            int k = rb;
            if (re - rb > kLongThresh) k = re;          // long rows: the segment kernels add them
            while (k < re) {
                if (k >= rq + 3 * G) {                  // skipped far ahead: restart the ring here
                    rq = k;
                    ld_r(rq + gl, rc0, rv0);
                    ld_r(rq + G + gl, rc1, rv1);
                    ld_r(rq + 2 * G + gl, rc2, rv2);
                } else if (k >= rq + G) {
                    rc0 = rc1; rv0 = rv1; rc1 = rc2; rv1 = rv2;
                    rq += G;
                    ld_r(rq + 2 * G + gl, rc2, rv2);
                    continue;                           // may have to advance once more
                }
                const int hi = min(re, rq + G) - rq;
                chunk_range_global<G, NV, VEC>(rc0, rv0, k - rq, hi, H, F, f, fok, acc);
                k = rq + hi;
            }
        }
#pragma unroll
        for (int q = 0; q < NV; ++q)
            if (fok[q]) {
                // fused: the row is final and nobody reads it again soon -> non-temporal store (2.7 % faster
                // at configs[3]); split: the remainder kernel adds to it next
                if constexpr (FUSED) store_vec_nt<VEC>(Y + (size_t)row * F + f + q * G * VEC, acc[q]);
                else store_vec<VEC>(Y + (size_t)row * F + f + q * G * VEC, acc[q]);
            }
    }
    c0 += kMaxBlock;
    if (MAXR == kMaxBlock || c0 >= pr1) break;          // uniform over the work-group
    begin_run(c0);
    }
}

template <int G, int NV, int VEC, bool FUSED, bool SCALED, int MAXR>
int launch_one(const BlocksDev &B, const int32_t *list, int nlist, const CsrDev &R, const float *H, float *Y,
               int F, hipStream_t st)
{
    constexpr int FT = G * VEC * NV;
    constexpr size_t lds = (size_t)(MAXR + 1) * FT * sizeof(float);
    if (lds > 65536) {
        // more than the default 64 KB of dynamic LDS has to be requested once per device
        static std::atomic<bool> prepared[64];          // per instantiation and device
        int dev = 0;
        (void)hipGetDevice(&dev);
        if (dev < 0 || dev >= 64 || !prepared[dev].load(std::memory_order_acquire)) {
            int rc = hip_fail((int)hipFuncSetAttribute((const void *)k_block_sparse<G, NV, VEC, FUSED, SCALED, MAXR>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                              "LDS size attribute");
            if (rc) return rc;
            if (dev >= 0 && dev < 64) prepared[dev].store(true, std::memory_order_release);
        }
    }
    // few blocks: up to four work-groups per block until about kWantGroups of them are in flight
    const int tiles = (F + FT - 1) / FT;
    const int parts = std::max(1, std::min(4, kWantGroups / std::max(1, nlist * tiles)));
    dim3 grid(nlist * parts, tiles);
    hipLaunchKernelGGL((k_block_sparse<G, NV, VEC, FUSED, SCALED, MAXR>), grid, dim3(kWG), lds, st, B, list, R, H, Y, F, parts);
    return hip_fail((int)hipGetLastError(), "block_sparse launch");
}

template <int G, int NV, int VEC, int MAXR>
int run_sized(const BlocksDev &B, const int32_t *list, int nlist, const CsrDev *rem, const float *H,
              float *Y, int F, hipStream_t st)
{
    const bool scaled = B.in_scale || B.out_scale;      // factored values: a separate instantiation keeps the plain path lean
    if (rem) return scaled ? launch_one<G, NV, VEC, true, true, MAXR>(B, list, nlist, *rem, H, Y, F, st)
                           : launch_one<G, NV, VEC, true, false, MAXR>(B, list, nlist, *rem, H, Y, F, st);
    return scaled ? launch_one<G, NV, VEC, false, true, MAXR>(B, list, nlist, CsrDev(), H, Y, F, st)
                  : launch_one<G, NV, VEC, false, false, MAXR>(B, list, nlist, CsrDev(), H, Y, F, st);
}

// plans whose blocks all have at most 128 rows keep the smaller LDS tile (more work-groups per CU)
template <int G, int NV, int VEC>
int run(const BlocksDev &B, const int32_t *list, int nlist, const CsrDev *rem, const float *H,
        float *Y, int F, hipStream_t st)
{
    if (B.max_block_rows > kMaxBlock) return run_sized<G, NV, VEC, kMaxBlockWide>(B, list, nlist, rem, H, Y, F, st);
    return run_sized<G, NV, VEC, kMaxBlock>(B, list, nlist, rem, H, Y, F, st);
}

}  // namespace

int launch_block_sparse(const BlocksDev &B, const int32_t *list, int32_t nlist, const CsrDev *fused_rem,
                        const float *H, float *Y, int32_t F, void *stream)
{
    if (nlist <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    if (F % 4 == 0) {
        const int need = F / 4;                         // float4 vectors per row
        // 64-feature tiles (33 KB of LDS, 4 work-groups per CU) beat 128-feature tiles (2 per CU)
        if (need >= 32) return run<8, 2, 4>(B, list, nlist, fused_rem, H, Y, F, st);
        if (need >= 16) return run<8, 2, 4>(B, list, nlist, fused_rem, H, Y, F, st);
        if (need > 8) return run<16, 1, 4>(B, list, nlist, fused_rem, H, Y, F, st);
        if (need > 4) return run<8, 1, 4>(B, list, nlist, fused_rem, H, Y, F, st);
        return run<4, 1, 4>(B, list, nlist, fused_rem, H, Y, F, st);
    }
    if (F % 2 == 0) {                                   // 8-byte vectors, up to 128 features per tile
        const int need = F / 2;
        if (need > 32) return run<64, 1, 2>(B, list, nlist, fused_rem, H, Y, F, st);
        if (need > 16) return run<32, 1, 2>(B, list, nlist, fused_rem, H, Y, F, st);
        if (need > 8) return run<16, 1, 2>(B, list, nlist, fused_rem, H, Y, F, st);
        if (need > 4) return run<8, 1, 2>(B, list, nlist, fused_rem, H, Y, F, st);
        return run<4, 1, 2>(B, list, nlist, fused_rem, H, Y, F, st);
    }
    if (F > 32) return run<64, 1, 1>(B, list, nlist, fused_rem, H, Y, F, st);
    if (F > 16) return run<32, 1, 1>(B, list, nlist, fused_rem, H, Y, F, st);
    if (F > 8) return run<16, 1, 1>(B, list, nlist, fused_rem, H, Y, F, st);
    if (F > 4) return run<8, 1, 1>(B, list, nlist, fused_rem, H, Y, F, st);
    return run<4, 1, 1>(B, list, nlist, fused_rem, H, Y, F, st);
}

}  // namespace ag
