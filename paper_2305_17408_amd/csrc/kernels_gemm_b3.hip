// Layer transform C[N x n] = epilogue(A[N x k] W[k x n]) on the bf16 matrix instruction at fp32
// accuracy (the dense Update of paper Sec. 2.1; mixed precision is the direction Sec. 3.2 names
// as future work, here without giving up accuracy).
//
// Every fp32 operand is cut into three bf16 pieces that add up to it exactly (8 + 8 + 8 mantissa
// bits, by truncation with the remainder computed exactly, so |a2| <= 2^-7 |a| and |a3| <= 2^-14 |a|
// in the worst case).  Of the nine piece products the six with weight >= 2^-16 are accumulated in
// fp32, smallest first:
//     a b ~= a3 b1 + a1 b3 + a2 b2 + a2 b1 + a1 b2 + a1 b1
// The dropped terms a2 b3 + a3 b2 + a3 b3 are bounded by 2^-20 |a b| and reach about 2^-21 |a b|
// (4.7e-7 |a b| for mantissas of the form 1 + 2^-7 - 2^-23); the cuts being truncations, they always point towards
// zero (mean bias about 4e-8 |a b|): a little below the accuracy of a true fp32 product, far
// inside the 1e-5 acceptance band, at 6/16 of the fp32 matrix-pipe time.
// W is split once by a small kernel into K-contiguous piece rows; A is split while its tile is
// staged into LDS.  Operand layout of v_mfma_f32_32x32x16_bf16 for lane l: A[l & 31][8 (l >> 5) +
// 0..7], B[8 (l >> 5) + 0..7][l & 31]; result register r holds D[8 (r / 4) + 4 (l >> 5) + (r & 3)][l & 31].
#include <algorithm>

#include "kernels_common.h"
#include "mfma_b3.h"

namespace ag {
namespace {

enum { EPI_NONE = 0, EPI_BIAS_RELU = 1, EPI_RELU_MASK = 2 };

constexpr int kStage = 32;              // k values staged per step (two matrix instructions deep)
constexpr int kRowB = kStage * 2 + 16;  // bytes per LDS operand row: 64 of data + 16 of padding, so
                                        // the eight lanes of a 16-byte read phase hit distinct banks

// Wp[(piece * npad + col) * kpad + kk] = piece of W[kk][col]; zero for kk >= k or col >= n
__global__ __launch_bounds__(kWG) void k_split_w(const float *__restrict__ W, uint16_t *__restrict__ Wp,
                                                 int k, int kpad, int n, int npad)
{
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i >= (int64_t)kpad * npad) return;
    const int kk = (int)(i / npad), col = (int)(i % npad);
    uint32_t p[3] = {0u, 0u, 0u};
    if (kk < k && col < n) cut3(W[(size_t)kk * n + col], p);
#pragma unroll
    for (int s = 0; s < 3; ++s) Wp[((size_t)s * npad + col) * kpad + kk] = (uint16_t)(p[s] >> 16);
}

// WVM x WVN wavefronts, each owning WM x WN tiles of 32 x 32.  Work-groups that share rows of A (the
// column tiles of one row tile) have neighbouring ids, so the second read of those rows is served
// by the memory-side cache.
template <int WVM, int WVN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WVM * WVN * 64) void k_gemm_nn_b3(const float *__restrict__ A, const uint16_t *__restrict__ Wp,
                                                      float *__restrict__ C, int64_t N, int k, int kpad, int n,
                                                      int npad, int ncol_tiles, const float *__restrict__ aux)
{
    constexpr int kWG = WVM * WVN * 64;                       // threads of this kernel's work-group
    constexpr int TM = WVM * WM * 32, TN = WVN * WN * 32;
    constexpr int UA = TM * kStage / 4 / kWG;                 // float4 loads of A per thread and stage
    constexpr int NW = 3 * TN * kStage / 8;                   // 16-byte units of the W pieces per stage
    constexpr int UW = (NW + kWG - 1) / kWG;                  // ... per thread
    static_assert(TM * kStage / 4 % kWG == 0, "tile must divide among the threads");
    __shared__ __attribute__((aligned(16))) unsigned char sA[3 * TM * kRowB];
    __shared__ __attribute__((aligned(16))) unsigned char sW[3 * TN * kRowB];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int wm = w / WVN, wn = w % WVN;
    // Persistent work-groups: each walks the output tiles t, t + gridDim.x, ...; the loads of the
    // next stage are always in flight during the current one, also across the end of a tile, so
    // a tile's first memory latency and its write-out overlap with its neighbours' work.
    const int64_t ntiles = ((N + TM - 1) / TM) * ncol_tiles;

    float4 ra[UA];
    u32x4 rw[UW];
    auto fetch = [&](int64_t tile, int k0) {
        const int64_t r0 = (tile / ncol_tiles) * TM;
        const int n0 = (int)(tile % ncol_tiles) * TN;
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (kStage / 4), c = (idx % (kStage / 4)) * 4;
            ra[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r0 + r < N && k0 + c < k) ra[u] = *reinterpret_cast<const float4 *>(A + (r0 + r) * k + k0 + c);
        }
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int idx = tid + u * kWG, pc = idx / (TN * kStage / 8), rem = idx % (TN * kStage / 8);
            const int col = rem / (kStage / 8), c = (rem % (kStage / 8)) * 8;
            rw[u] = u32x4{0u, 0u, 0u, 0u};
            if (idx < NW) rw[u] = *reinterpret_cast<const u32x4 *>(Wp + ((size_t)pc * npad + n0 + col) * kpad + k0 + c);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (kStage / 4), c = (idx % (kStage / 4)) * 4;
            uint32_t px[3], py[3], pz[3], pw[3];
            cut3(ra[u].x, px); cut3(ra[u].y, py); cut3(ra[u].z, pz); cut3(ra[u].w, pw);
#pragma unroll
            for (int s = 0; s < 3; ++s)
                *reinterpret_cast<uint2 *>(sA + (s * TM + r) * kRowB + c * 2) =
                    make_uint2((px[s] >> 16) | py[s], (pz[s] >> 16) | pw[s]);
        }
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int idx = tid + u * kWG, pc = idx / (TN * kStage / 8), rem = idx % (TN * kStage / 8);
            const int col = rem / (kStage / 8), c = (rem % (kStage / 8)) * 8;
            if (idx < NW) *reinterpret_cast<u32x4 *>(sW + (pc * TN + col) * kRowB + c * 2) = rw[u];
        }
    };

    fetch(blockIdx.x, 0);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int64_t r0 = (tile / ncol_tiles) * TM;
    const int n0 = (int)(tile % ncol_tiles) * TN;
    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int k0 = 0; k0 < kpad; k0 += kStage) {
        __syncthreads();                       // everyone is done reading the previous tiles
        stash();
        __syncthreads();
        if (k0 + kStage < kpad) fetch(tile, k0 + kStage);
        else if (tile + gridDim.x < ntiles) fetch(tile + gridDim.x, 0);
#pragma unroll
        for (int ks = 0; ks < kStage / 16; ++ks) {
            u32x4 a[WM][3], b[WN][3];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int s = 0; s < 3; ++s)
                    a[i][s] = *reinterpret_cast<const u32x4 *>(
                        sA + (s * TM + (wm * WM + i) * 32 + lo) * kRowB + (ks * 16 + 8 * hi) * 2);
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int s = 0; s < 3; ++s)
                    b[j][s] = *reinterpret_cast<const u32x4 *>(
                        sW + (s * TN + (wn * WN + j) * 32 + lo) * kRowB + (ks * 16 + 8 * hi) * 2);
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    floatx16 c = acc[i][j];
                    c = mfma16(a[i][2], b[j][0], c);
                    c = mfma16(a[i][0], b[j][2], c);
                    c = mfma16(a[i][1], b[j][1], c);
                    c = mfma16(a[i][1], b[j][0], c);
                    c = mfma16(a[i][0], b[j][1], c);
                    c = mfma16(a[i][0], b[j][0], c);
                    acc[i][j] = c;
                }
        }
    }
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int col = n0 + (wn * WN + j) * 32 + lo;
            if (col >= n) continue;
            float bias = 0.f;
            if constexpr (EPI == EPI_BIAS_RELU) bias = aux[col];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = r0 + (wm * WM + i) * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (row >= N) continue;
                float v = acc[i][j][r];
                if constexpr (EPI == EPI_BIAS_RELU) v = fmaxf(v + bias, 0.f);
                if constexpr (EPI == EPI_RELU_MASK) v = (aux[row * n + col] > 0.f) ? v : 0.f;
                C[row * n + col] = v;
            }
        }
    }
}

// The same transform for k <= 128 with the weights RESIDENT IN REGISTERS: a work-group of NW =
// ceil(n / 32) wavefronts covers all output columns of a block of 32 rows; wavefront w keeps the
// three bf16 pieces of W[:, 32 w .. 32 w + 31] for all KT k-steps of 16 in 12 KT registers for the
// whole kernel (the split copy Wp is K-contiguous: one 16-byte load per k-step and piece), so no
// shared operand has to be fetched again for every tile.  The block of A is read once per
// work-group (float4 loads, one block ahead), cut into pieces and written to LDS as
// sA[piece][row][k] (lines of 2 KP + 16 bytes); lane (row, hi) reads its operand of a k-step with
// one 16-byte LDS load per piece.  Two LDS buffers, one barrier per block, unconditional loads
// with clamped rows.  (Two work-groups of four wavefronts per row block, to have them on one CU in
// different phases, were slower: 0.52 against 0.46 ms on the 1 M x 128 x 256 transform.)  The 32 x 32 result tile gets its epilogue in registers and is stored with
// 128-byte row pieces.
template <int KT, int NW, int EPI>
__global__ __launch_bounds__(64 * NW, 1) void k_gemm_nn_b3_resident(const float *__restrict__ A, const uint16_t *__restrict__ Wp,
                                                                    float *__restrict__ C, int64_t N, int k, int kpad, int n,
                                                                    int npad, const float *__restrict__ aux, int rows_per_wg)
{
    constexpr int KP = 16 * KT, T = 64 * NW, kLine = 2 * KP + 16;
    constexpr int NV = 32 * KP / 4;                        // float4 units of a block of A
    constexpr int UA = (NV + T - 1) / T;                   // ... per thread
    __shared__ __attribute__((aligned(16))) unsigned char sA[2][3 * 32 * kLine];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int col = 32 * w + lo;                           // < npad: Wp is zero beyond n
    u32x4 bw[KT][3];
#pragma unroll
    for (int ks = 0; ks < KT; ++ks)
#pragma unroll
        for (int s = 0; s < 3; ++s)
            bw[ks][s] = (16 * ks + 8 * hi < kpad)
                            ? *reinterpret_cast<const u32x4 *>(Wp + ((size_t)s * npad + col) * kpad + 16 * ks + 8 * hi)
                            : u32x4{0u, 0u, 0u, 0u};
    float bias = 0.f;
    if constexpr (EPI == EPI_BIAS_RELU) bias = col < n ? aux[col] : 0.f;
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg, re = min(N, rb + rows_per_wg);
    const bool vec = (k % 4 == 0);

    float4 ra[UA];
    auto fetch = [&](int64_t R0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * T, r = idx / (KP / 4), c = (idx % (KP / 4)) * 4;
            const int64_t row = min(R0 + min(r, 31), N - 1);
            const float *p = A + row * k;
            if (vec) {
                ra[u] = *reinterpret_cast<const float4 *>(p + min(c, k - 4));
            } else {
                ra[u] = make_float4(p[min(c, k - 1)], p[min(c + 1, k - 1)], p[min(c + 2, k - 1)], p[min(c + 3, k - 1)]);
            }
        }
    };
    auto stash = [&](int buf, int64_t R0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * T, r = idx / (KP / 4), c = (idx % (KP / 4)) * 4;
            if (idx >= NV) continue;
            const bool ok = R0 + r < re;
            uint32_t px[3], py[3], pz[3], pw[3];
            cut3((ok && c < k) ? ra[u].x : 0.f, px);
            cut3((ok && c + 1 < k) ? ra[u].y : 0.f, py);
            cut3((ok && c + 2 < k) ? ra[u].z : 0.f, pz);
            cut3((ok && c + 3 < k) ? ra[u].w : 0.f, pw);
#pragma unroll
            for (int s = 0; s < 3; ++s)
                *reinterpret_cast<uint2 *>(&sA[buf][(s * 32 + r) * kLine + c * 2]) =
                    make_uint2((px[s] >> 16) | py[s], (pz[s] >> 16) | pw[s]);
        }
    };

    int buf = 0;
    if (rb < re) {                                         // uniform over the work-group
        fetch(rb);
        stash(0, rb);
    }
    for (int64_t R0 = rb; R0 < re; R0 += 32, buf ^= 1) {
        __syncthreads();                                   // buffer `buf` is complete; the other one is free
        fetch(R0 + 32);                                    // always (clamped): no branch between loads and work
        float mask[EPI == EPI_RELU_MASK ? 16 : 1];         // the mask entries travel while the matrix pipe works
        if constexpr (EPI == EPI_RELU_MASK) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = min(R0 + 8 * (r >> 2) + 4 * hi + (r & 3), N - 1);
                mask[r] = aux[row * n + min(col, n - 1)];
            }
        }
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KT; ++ks) {
            u32x4 a[3];
#pragma unroll
            for (int s = 0; s < 3; ++s)
                a[s] = *reinterpret_cast<const u32x4 *>(&sA[buf][(s * 32 + lo) * kLine + (16 * ks + 8 * hi) * 2]);
            acc = mfma16_b3(a, bw[ks], acc);
        }
        if (col < n) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = R0 + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (row >= re) continue;
                float v = acc[r];
                if constexpr (EPI == EPI_BIAS_RELU) v = fmaxf(v + bias, 0.f);
                if constexpr (EPI == EPI_RELU_MASK) v = (mask[r] > 0.f) ? v : 0.f;
                C[row * n + col] = v;
            }
        }
        stash(buf ^ 1, R0 + 32);
    }
}

// Two chained transforms of a GCN layer pair (paper Sec. 2.1, Update of layer 1 followed by the
// product that layer 2 aggregates): H = relu(A W + b) [N x n] and Q = H W2 [N x c], c <= 16, in
// one pass, H never being read back.  Same frame as k_gemm_nn_b3_resident (weights resident in
// registers, the block of A cut into LDS once per work-group), with the operands of the matrix
// instruction swapped: it then yields the TRANSPOSED tile, lane (row, hi) holding H[row][32 w +
// 8 g + 4 hi + q] in register 4 g + q.  In that layout
//   * a lane stores its row of the tile with four 16-byte stores, and
//   * registers 8 s .. 8 s + 7 are, as they stand, the operand "8 consecutive k values of column
//     `row`" of a second matrix instruction whose k index runs over the wavefront's 32 hidden
//     columns in the order 16 s + 8 (t / 4) + 4 hi + (t & 3); the rows of W2 are loaded into the
//     other operand in that same order, so Q^T(partial) = W2^T H^T needs no data movement at all.
// The eight wavefronts' partial products (each over its own 32 hidden columns) meet in LDS and are
// summed and stored by 128 threads during the next block.
template <int KT, int NW>
__global__ __launch_bounds__(64 * NW, 1) void k_gemm_chain_b3(const float *__restrict__ A, const uint16_t *__restrict__ Wp,
                                                              const float *__restrict__ bias, const float *__restrict__ W2,
                                                              float *__restrict__ C, float *__restrict__ Q, int64_t N,
                                                              int k, int kpad, int n, int npad, int c, int rows_per_wg)
{
    constexpr int KP = 16 * KT, T = 64 * NW, kLine = 2 * KP + 16;
    constexpr int NV = 32 * KP / 4;                        // float4 units of a block of A
    constexpr int UA = (NV + T - 1) / T;                   // ... per thread
    constexpr int kQLine = 20;                             // floats per row of a partial Q tile: 16 + 4 of padding
    __shared__ __attribute__((aligned(16))) unsigned char sA[2][3 * 32 * kLine];
    __shared__ __attribute__((aligned(16))) float sQ[2][NW][32 * kQLine];
    __shared__ __attribute__((aligned(16))) float sBias[32 * NW];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int col = 32 * w + lo;                           // < npad: Wp is zero beyond n
    u32x4 bw[KT][3];
#pragma unroll
    for (int ks = 0; ks < KT; ++ks)
#pragma unroll
        for (int s = 0; s < 3; ++s)
            bw[ks][s] = (16 * ks + 8 * hi < kpad)
                            ? *reinterpret_cast<const u32x4 *>(Wp + ((size_t)s * npad + col) * kpad + 16 * ks + 8 * hi)
                            : u32x4{0u, 0u, 0u, 0u};
    // W2^T operand: lane (class lo, hi), slot t of step s <-> hidden column 32 w + 16 s + 8 (t / 4) + 4 hi + (t & 3)
    u32x4 w2p[2][3];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int hc = 32 * w + 16 * s + 8 * (t >> 2) + 4 * hi + (t & 3);
            v[t] = (lo < c && hc < n) ? W2[(size_t)hc * c + lo] : 0.f;
        }
        cut3x8(v, w2p[s]);
    }
    for (int i = tid; i < 32 * NW; i += T) sBias[i] = i < n ? bias[i] : 0.f;
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg, re = min(N, rb + rows_per_wg);

    // Addresses advance by a constant per block (no multiplications in the loop); a load that would
    // start beyond the last row is redirected to the last row (its values are not used).
    float4 ra[UA];
    const float *pa[UA], *pa_last[UA];
#pragma unroll
    for (int u = 0; u < UA; ++u) {
        const int idx = tid + u * T, r = idx / (KP / 4), cc = (idx % (KP / 4)) * 4;
        pa[u] = A + (rb + min(r, 31)) * k + min(cc, k - 4);
        pa_last[u] = A + (N - 1) * k + min(cc, k - 4);
    }
    const int64_t a_step = (int64_t)32 * k;
    auto fetch = [&]() {                                   // the next block of A, in order
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            ra[u] = *reinterpret_cast<const float4 *>(min(pa[u], pa_last[u]));
            pa[u] += a_step;
        }
    };
    auto stash = [&](int buf, int64_t R0) {
        const int left = (int)min<int64_t>(re - R0, 32);   // rows of this block (<= 0: none)
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * T, r = idx / (KP / 4), cc = (idx % (KP / 4)) * 4;
            if (idx >= NV) continue;
            const bool ok = r < left && cc < k;            // k is a multiple of 4
            uint32_t px[3], py[3], pz[3], pw[3];
            cut3(ok ? ra[u].x : 0.f, px);
            cut3(ok ? ra[u].y : 0.f, py);
            cut3(ok ? ra[u].z : 0.f, pz);
            cut3(ok ? ra[u].w : 0.f, pw);
#pragma unroll
            for (int s = 0; s < 3; ++s)
                *reinterpret_cast<uint2 *>(&sA[buf][(s * 32 + r) * kLine + cc * 2]) =
                    make_uint2((px[s] >> 16) | py[s], (pz[s] >> 16) | pw[s]);
        }
    };
    // sum of the wavefronts' partial tiles of the block that started at row R0, by threads 0 .. 127
    float *pq = Q + (rb + (tid >> 2)) * c + (tid & 3) * 4;  // threads 0 .. 127: row tid / 4 of the block, four classes
    auto reduce_q = [&](int qbuf, int64_t R0) {
        if (tid >= 128) return;
        const int r = tid >> 2, c4 = (tid & 3) * 4;
        float *q = pq;
        pq += 32 * c;
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            const float4 v = *reinterpret_cast<const float4 *>(&sQ[qbuf][ww][r * kQLine + c4]);
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        if (R0 + r >= re) return;
        if (c % 4 == 0) {
            if (c4 < c) *reinterpret_cast<float4 *>(q) = sum;
        } else {
            if (c4 < c) q[0] = sum.x;
            if (c4 + 1 < c) q[1] = sum.y;
            if (c4 + 2 < c) q[2] = sum.z;
            if (c4 + 3 < c) q[3] = sum.w;
        }
    };

    if (rb >= re) return;                                  // uniform over the work-group
    fetch();
    stash(0, rb);
    float *pc = C + (rb + lo) * n + 32 * w + 4 * hi;       // this lane's row of the tile; + 8 g for register group g
    int buf = 0;
    for (int64_t R0 = rb; R0 < re; R0 += 32, buf ^= 1) {
        __syncthreads();                                   // sA[buf] and the previous block's sQ[buf ^ 1] are complete
        fetch();                                           // always (clamped): no branch between loads and work
        if (R0 > rb) reduce_q(buf ^ 1, R0 - 32);
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KT; ++ks) {
            u32x4 a[3];
#pragma unroll
            for (int s = 0; s < 3; ++s)
                a[s] = *reinterpret_cast<const u32x4 *>(&sA[buf][(s * 32 + lo) * kLine + (16 * ks + 8 * hi) * 2]);
            acc = mfma16_b3(bw[ks], a, acc);               // acc[4 g + q] = (A W)[R0 + lo][32 w + 8 g + 4 hi + q]
        }
        const bool row_ok = lo < re - R0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int hc = 32 * w + 8 * g + 4 * hi;
            const float4 b = *reinterpret_cast<const float4 *>(&sBias[hc]);
            acc[4 * g] = fmaxf(acc[4 * g] + b.x, 0.f);
            acc[4 * g + 1] = fmaxf(acc[4 * g + 1] + b.y, 0.f);
            acc[4 * g + 2] = fmaxf(acc[4 * g + 2] + b.z, 0.f);
            acc[4 * g + 3] = fmaxf(acc[4 * g + 3] + b.w, 0.f);
            if (row_ok && hc < n)                          // n is a multiple of 4
                *reinterpret_cast<float4 *>(pc + 8 * g) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
        }
        pc += (int64_t)32 * n;
        floatx16 qa;
#pragma unroll
        for (int r = 0; r < 16; ++r) qa[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            float v[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = acc[8 * s + t];
            u32x4 hb[3];
            cut3x8(v, hb);
            qa = mfma16_b3(w2p[s], hb, qa);                // qa[4 g + q] = Q^T(partial)[class 8 g + 4 hi + q][row lo]
        }
#pragma unroll
        for (int g = 0; g < 2; ++g)
            *reinterpret_cast<float4 *>(&sQ[buf][w][lo * kQLine + 8 * g + 4 * hi]) =
                make_float4(qa[4 * g], qa[4 * g + 1], qa[4 * g + 2], qa[4 * g + 3]);
        stash(buf ^ 1, R0 + 32);
    }
    __syncthreads();
    reduce_q(buf ^ 1, rb + ((re - rb - 1) / 32) * 32);     // the last block's partial tiles
}

constexpr int kResidentRowsPerWg = 4096;

template <int KT, int EPI>
bool run_resident(int64_t N, int k, int kpad, int n, int npad, const float *A, const uint16_t *Wp, float *C,
                  const float *aux, hipStream_t st)
{
    const int nw = (n + 31) / 32;
    // rows per work-group: about 256 x 8 wavefronts over the chip whatever the work-group's size
    const int rows = std::max(kResidentRowsPerWg * nw / 8, 256);
    const dim3 grid((unsigned)((N + rows - 1) / rows));
#define AG_RES(w) case w: hipLaunchKernelGGL((k_gemm_nn_b3_resident<KT, w, EPI>), grid, dim3(64 * w), 0, st, A, Wp, C, N, k, kpad, n, npad, aux, rows); return true;
    switch (nw) {                                         // the common widths; others take the tiled kernel
    AG_RES(1) AG_RES(2) AG_RES(4) AG_RES(8)
    default: return false;
    }
#undef AG_RES
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

template <int EPI>
void run_b3(int64_t N, int k, int n, const float *A, const uint16_t *Wp, float *C, const float *aux, hipStream_t st)
{
    const int kpad = round_up(k, kStage), npad = round_up(n, 256);
    // k <= 128 and up to 256 output columns: the weights stay in registers
    if (k <= 64 && run_resident<4, EPI>(N, k, kpad, n, npad, A, Wp, C, aux, st)) return;
    if (k > 64 && k <= 128 && run_resident<8, EPI>(N, k, kpad, n, npad, A, Wp, C, aux, st)) return;
    if (n > 128) {
        // 128 x 256 tile, 16 waves: a row tile of A is staged (and cut) once for 256 output columns
        const int ct = (n + 255) / 256;
        dim3 grid((unsigned)std::min<int64_t>(((N + 127) / 128) * ct, 256));
        hipLaunchKernelGGL((k_gemm_nn_b3<4, 4, 1, 2, EPI>), grid, dim3(1024), 0, st, A, Wp, C, N, k, kpad, n, npad, ct, aux);
    } else {
        dim3 grid((unsigned)std::min<int64_t>((N + 127) / 128, 512));
        hipLaunchKernelGGL((k_gemm_nn_b3<4, 2, 1, 2, EPI>), grid, dim3(512), 0, st, A, Wp, C, N, k, kpad, n, npad, 1, aux);
    }
}

}  // namespace

// floats of scratch the split copy of W needs (0 if the shape is not served by this path: outputs
// of up to 16 columns, and of up to 64 columns unless the weights fit the register-resident
// kernel, stay on the fp32 kernels)
size_t gemm_nn_b3_scratch_floats(int32_t k, int32_t n)
{
    if (k < 32 || k % 4 || n <= 16 || (n <= 64 && k > 128)) return 0;
    return ((size_t)3 * round_up(n, 256) * round_up(k, kStage) * sizeof(uint16_t) + 3) / 4 + 4;
}

// Returns AG_ERR_UNSUPPORTED when the shape is not served here (the caller then uses the fp32 kernels).
int launch_gemm_nn_b3(int64_t N, int32_t k, int32_t n, const float *A, const float *W, float *C, int epilogue,
                      const float *aux, float *wsplit, void *stream)
{
    if (!wsplit || gemm_nn_b3_scratch_floats(k, n) == 0) return AG_ERR_UNSUPPORTED;
    if (N <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    const int kpad = round_up(k, kStage), npad = round_up(n, 256);
    uint16_t *Wp = reinterpret_cast<uint16_t *>(wsplit);
    const int64_t cells = (int64_t)kpad * npad;
    hipLaunchKernelGGL(k_split_w, dim3((unsigned)((cells + kWG - 1) / kWG)), dim3(kWG), 0, st, W, Wp, k, kpad, n, npad);
    if (epilogue == EPI_BIAS_RELU) run_b3<EPI_BIAS_RELU>(N, k, n, A, Wp, C, aux, st);
    else if (epilogue == EPI_RELU_MASK) run_b3<EPI_RELU_MASK>(N, k, n, A, Wp, C, aux, st);
    else run_b3<EPI_NONE>(N, k, n, A, Wp, C, aux, st);
    return hip_fail((int)hipGetLastError(), "gemm_nn_b3 launch");
}

// H = relu(A W + b) and Q = H W2 in one pass (see k_gemm_chain_b3).  `wsplit` holds at least
// gemm_nn_b3_scratch_floats(k, n) floats.  Returns AG_ERR_UNSUPPORTED for shapes the kernel does
// not serve: the caller then runs the two transforms one after the other.
int launch_gemm_chain_b3(int64_t N, int32_t k, int32_t n, int32_t c, const float *A, const float *W, const float *bias,
                         const float *W2, float *H, float *Q, float *wsplit, void *stream)
{
    const bool fits = wsplit && k >= 32 && k <= 128 && k % 4 == 0 && (n == 128 || n == 256) && c >= 1 && c <= 16;
    if (!fits || gemm_nn_b3_scratch_floats(k, n) == 0) return AG_ERR_UNSUPPORTED;
    if (N <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    const int kpad = round_up(k, kStage), npad = round_up(n, 256);
    uint16_t *Wp = reinterpret_cast<uint16_t *>(wsplit);
    const int64_t cells = (int64_t)kpad * npad;
    hipLaunchKernelGGL(k_split_w, dim3((unsigned)((cells + kWG - 1) / kWG)), dim3(kWG), 0, st, W, Wp, k, kpad, n, npad);
    const int nw = n / 32, rows = kResidentRowsPerWg * nw / 8;
    const dim3 grid((unsigned)((N + rows - 1) / rows));
#define AG_CHAIN(kt, w) hipLaunchKernelGGL((k_gemm_chain_b3<kt, w>), grid, dim3(64 * w), 0, st, A, Wp, bias, W2, H, Q, N, k, kpad, n, npad, c, rows)
    if (k <= 64) { if (nw == 4) AG_CHAIN(4, 4); else AG_CHAIN(4, 8); }
    else         { if (nw == 4) AG_CHAIN(8, 4); else AG_CHAIN(8, 8); }
#undef AG_CHAIN
    return hip_fail((int)hipGetLastError(), "gemm_chain_b3 launch");
}

// The layer transform on the fastest path that serves the shape: bf16 pieces when `wsplit` (at least
// gemm_nn_b3_scratch_floats(k, n) floats) is given and the shape fits, else the fp32 kernels.
int launch_gemm_nn_auto(int64_t N, int32_t k, int32_t n, const float *A, const float *W, float *C, int epilogue,
                        const float *aux, float *wsplit, void *stream)
{
    const int rc = launch_gemm_nn_b3(N, k, n, A, W, C, epilogue, aux, wsplit, stream);
    if (rc != AG_ERR_UNSUPPORTED) return rc;
    return launch_gemm_nn(N, k, n, A, W, C, epilogue, aux, stream);
}

}  // namespace ag
