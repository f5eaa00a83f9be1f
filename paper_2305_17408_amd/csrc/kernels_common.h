// Device helpers shared by the aggregation kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>

#include "ag_internal.h"

namespace ag {

constexpr int kWG = 256;   // work-group size of every aggregation kernel (4 wavefronts)

template <int VEC>
__device__ __forceinline__ void load_vec(const float *__restrict__ p, float (&h)[VEC])
{
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        h[0] = t.x; h[1] = t.y; h[2] = t.z; h[3] = t.w;
    } else if constexpr (VEC == 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        h[0] = t.x; h[1] = t.y;
    } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) h[j] = p[j];
    }
}

// Non-temporal forms for data that is touched once (stores of finished output rows).
template <int VEC>
__device__ __forceinline__ void load_vec_nt(const float *__restrict__ p, float (&h)[VEC])
{
    if constexpr (VEC == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
        h[0] = t.x; h[1] = t.y; h[2] = t.z; h[3] = t.w;
    } else {
        load_vec<VEC>(p, h);
    }
}
template <int VEC>
__device__ __forceinline__ void store_vec_nt(float *__restrict__ p, const float (&h)[VEC])
{
    if constexpr (VEC == 4) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        f4 t = {h[0], h[1], h[2], h[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<f4 *>(p));
    } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) p[j] = h[j];
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float *__restrict__ p, const float (&h)[VEC])
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(h[0], h[1], h[2], h[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(h[0], h[1]);
    } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) p[j] = h[j];
    }
}

// Widest vector (floats) every row of an F-column fp32 matrix can be moved with: rows start at
// multiples of 4F bytes, so 16-byte vectors need F % 4 == 0 and 8-byte vectors F % 2 == 0.
inline int vec_width(int F) { return (F % 4 == 0) ? 4 : (F % 2 == 0) ? 2 : 1; }

// Work-groups are handed to the 8 XCDs round-robin.  This maps the hardware block id to a
// logical id such that each XCD walks one contiguous eighth of the logical range, so rows
// that share neighbours (same community) meet in the same L2.
__device__ __forceinline__ int xcd_contiguous(int bid, int nb)
{
    const int x = bid & 7, i = bid >> 3, per = nb >> 3, rem = nb & 7;
    return x * per + (x < rem ? x : rem) + i;
}

// Copy rows [r0, r0+nr) x columns [f0, f0+FT) of the row-major matrix H (F columns) into the LDS
// tile sH[row][FT]; rows nr..pad_rows-1 and columns beyond F are zero-filled.  All loads of a
// thread are issued before its first LDS store, so a tile costs one memory latency, not one per
// row.  With `scale` every row is multiplied by scale[row] on the way (factored edge values).
// Must be called by the whole work-group; the caller synchronises afterwards.
template <int FT, int VEC, int MAXR = kMaxBlock>
__device__ __forceinline__ void stage_tile(const float *__restrict__ H, int F, int r0, int nr, int pad_rows,
                                           int f0, float *sH, int tid, const float *__restrict__ scale = nullptr)
{
    constexpr int UPR = FT / VEC;                       // load units per tile row
    constexpr int ITER = (MAXR * UPR + kWG - 1) / kWG;  // the tile holds at most MAXR rows
    float h[ITER][VEC];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = tid + it * kWG, r = idx / UPR, ff = f0 + (idx % UPR) * VEC;
        if (r < nr && ff < F) {
            load_vec<VEC>(H + (size_t)(r0 + r) * F + ff, h[it]);
            if (scale) {
                const float sc = scale[r0 + r];
#pragma unroll
                for (int j = 0; j < VEC; ++j) h[it][j] *= sc;
            }
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) h[it][j] = 0.f;
        }
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = tid + it * kWG, r = idx / UPR;
        if (r < pad_rows) store_vec<VEC>(sH + r * FT + (idx % UPR) * VEC, h[it]);
    }
}

// One chunk of a CSR row held in registers: lane tl of the team holds entry tl's column `c` and
// value `v` (cnt <= W entries are valid).  The W/G lane groups (G lanes, each lane owning NV
// vectors of VEC features, vector q starting at column f + q*G*VEC) pass the entries round with
// lane shuffles and gather the feature rows of their share from global memory, U*NV independent
// loads in flight per lane.  All W lanes of the team must call this together.
template <int G, int W, int NV, int VEC>
__device__ __forceinline__ void team_chunk_gather(int c, float v, int cnt, const float *__restrict__ H,
                                                  int F, int f, const bool (&fok)[NV], int tl,
                                                  float (&acc)[NV][VEC])
{
    constexpr int NSG = W / G, U = 8 / NV;
    const int sg = tl / G;
    for (int k0 = 0; k0 < cnt; k0 += NSG * U) {
        int ck[U];
        float vk[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kk = k0 + u * NSG + sg;
            ck[u] = __shfl(c, kk & (W - 1), W);
            vk[u] = __shfl(v, kk & (W - 1), W);
        }
        float h[U][NV][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kk = k0 + u * NSG + sg;
            if (!(kk < cnt)) vk[u] = 0.f;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (kk < cnt && fok[q]) {
                    load_vec<VEC>(H + (size_t)ck[u] * F + f + q * G * VEC, h[u][q]);
                } else {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) h[u][q][j] = 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[q][j] = fmaf(vk[u], h[u][q][j], acc[q][j]);
    }
}

// Sum of p[q * stride] for q = q0, q0 + step, ... < q1 with eight loads in flight (eight running
// sums, combined pairwise): the additions always happen in the same order, so the result is
// bitwise reproducible, and a reduction over a few hundred partial results does not wait for one
// memory latency per term.
__device__ __forceinline__ float sum_strided(const float *__restrict__ p, size_t stride, int q0, int q1, int step)
{
    float a[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] = 0.f;
    int q = q0;
    for (; q + 7 * step < q1; q += 8 * step) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(size_t)(q + u * step) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] += v[u];
    }
#pragma unroll
    for (int u = 0; u < 7; ++u)
        if (q + u * step < q1) a[u] += p[(size_t)(q + u * step) * stride];
    return ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
}

// Accumulate entries [beg,end) of one CSR row into acc, W entries per chunk (see above).
template <int G, int W, int NV, int VEC>
__device__ __forceinline__ void team_row_gather(const int32_t *__restrict__ col,
                                                const float *__restrict__ val, int beg, int end,
                                                const float *__restrict__ H, int F, int f,
                                                const bool (&fok)[NV], int tl, float (&acc)[NV][VEC])
{
    for (int base = beg; base < end; base += W) {
        const int e = base + tl;
        int c = 0;
        float v = 0.f;
        if (e < end) {
            c = col[e];
            v = val ? val[e] : 1.f;
        }
        team_chunk_gather<G, W, NV, VEC>(c, v, min(W, end - base), H, F, f, fok, tl, acc);
    }
}

// Entries lo..hi-1 of a register chunk (lane k of a G-lane team holds entry k: column c, value v);
// the feature rows are gathered from global memory, U * NV loads in flight per lane.  A lane owns
// NV vectors of VEC floats, vector q starting at column f + q*G*VEC.
template <int G, int NV, int VEC>
__device__ __forceinline__ void chunk_range_global(int c, float v, int lo, int hi, const float *__restrict__ H,
                                                   int F, int f, const bool (&fok)[NV], float (&acc)[NV][VEC])
{
    constexpr int U = 4;
    for (int k0 = lo; k0 < hi; k0 += U) {
        int ck[U];
        float vk[U], h[U][NV][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ck[u] = __shfl(c, (k0 + u) & (G - 1), G);
            vk[u] = __shfl(v, (k0 + u) & (G - 1), G);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!(k0 + u < hi)) vk[u] = 0.f;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (k0 + u < hi && fok[q]) {
                    load_vec<VEC>(H + (size_t)ck[u] * F + f + q * G * VEC, h[u][q]);
                } else {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) h[u][q][j] = 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[q][j] = fmaf(vk[u], h[u][q][j], acc[q][j]);
    }
}

// Second half of a fused block kernel.  The work-group's partial sums for rows r0..r0+nr-1 and
// columns f0..f0+FT-1 sit in the LDS tile sOut[row][FT].  A team of G = FT/VEC lanes takes a
// contiguous run of those rows, adds the rows' entries of the remainder matrix R (feature rows
// gathered from global memory, topology streamed through a 3-deep ring of register chunks) and
// stores each output row exactly once.  Rows with more than kLongThresh remainder entries are
// stored without them; the segment kernels add those afterwards.
// prepare() issues the row-pointer and first topology loads and can run long before the partial
// sums exist (it hides two dependent memory latencies behind the block's own work); finish()
// needs the LDS tile complete.  The whole work-group must call both.
template <int FT, int VEC>
struct RemainderRows {
    static constexpr int G = FT / VEC, TEAMS = kWG / (G <= kWG ? G : kWG);
    int gl, f, first, myrows, rrp, re1, rq, rc0, rc1, rc2;
    float rv0, rv1, rv2;
    bool fok[1];

    __device__ __forceinline__ void ld(const CsrDev &R, int e, int &c, float &v) const
    {
        c = 0;
        v = 0.f;
        if (e < re1) {
            c = R.col[e];
            v = R.val ? R.val[e] : 1.f;
        }
    }

    __device__ __forceinline__ void prepare(const CsrDev &R, int r0, int nr, int F, int f0, int tid)
    {
        static_assert(G <= 64 && kMaxBlock / TEAMS + 1 <= G, "row pointers of a team must fit in its lanes");
        const int team = tid / G;
        gl = tid % G;
        f = f0 + gl * VEC;
        fok[0] = f < F;
        const int rpt = (nr + TEAMS - 1) / TEAMS;
        first = min(team * rpt, nr);
        myrows = min(rpt, nr - first);
        rrp = R.rowptr[r0 + first + min(gl, myrows)];
        re1 = __shfl(rrp, myrows, G);
        rq = __shfl(rrp, 0, G);
        ld(R, rq + gl, rc0, rv0);
        ld(R, rq + G + gl, rc1, rv1);
        ld(R, rq + 2 * G + gl, rc2, rv2);
    }

    __device__ __forceinline__ void finish(const CsrDev &R, const float *sOut, int r0,
                                           const float *__restrict__ H, float *__restrict__ Y, int F)
    {
        for (int i = 0; i < myrows; ++i) {
            float acc[1][VEC];
            load_vec<VEC>(sOut + (first + i) * FT + gl * VEC, acc[0]);
            const int rb = __shfl(rrp, i, G), re = __shfl(rrp, i + 1, G);
            int k = rb;
            if (re - rb > kLongThresh) k = re;
            while (k < re) {
                if (k >= rq + 3 * G) {                  // skipped far ahead: restart the ring here
                    rq = k;
                    ld(R, rq + gl, rc0, rv0);
                    ld(R, rq + G + gl, rc1, rv1);
                    ld(R, rq + 2 * G + gl, rc2, rv2);
                } else if (k >= rq + G) {
                    rc0 = rc1; rv0 = rv1; rc1 = rc2; rv1 = rv2;
                    rq += G;
                    ld(R, rq + 2 * G + gl, rc2, rv2);
                    continue;                           // may have to advance once more
                }
                const int hi = min(re, rq + G) - rq;
                chunk_range_global<G, 1, VEC>(rc0, rv0, k - rq, hi, H, F, f, fok, acc);
                k = rq + hi;
            }
            if (fok[0]) store_vec<VEC>(Y + (size_t)(r0 + first + i) * F + f, acc[0]);
        }
    }
};

// Sum the partial accumulators of the W/G lane groups of a team; every group ends with the total.
template <int G, int W, int NV, int VEC>
__device__ __forceinline__ void team_reduce(float (&acc)[NV][VEC])
{
#pragma unroll
    for (int off = G; off < W; off <<= 1)
#pragma unroll
        for (int q = 0; q < NV; ++q)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[q][j] += __shfl_xor(acc[q][j], off, W);
}

}  // namespace ag
