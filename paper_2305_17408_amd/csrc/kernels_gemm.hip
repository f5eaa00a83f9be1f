// fp32 MFMA GEMMs for the dense Update part of the GCN step (paper Sec. 2.1 "Update", Sec. 5).
//
// gemm_tn:  C[m x n] = A^T B  with A [K x m], B [K x n] row-major and K = number of vertices
//           (the weight gradients dW = X^T dY).  K is split across work-groups; each writes a
//           partial m x n tile and a second kernel adds the partials in a fixed order.
//           Both MFMA operands are rows of A and B, so they are read coalesced and staged in LDS
//           without any transposition.  Optionally the column sums of B (the bias gradient)
//           are accumulated on the way from the values each thread loads anyway.
// gemm_nn:  C[N x n] = epilogue(A[N x k] W[k x n]) with N = number of vertices: the layer
//           transforms.  Epilogues: none, + bias then ReLU, or masking by a ReLU activation
//           (the backward through the ReLU), fused so the N x n result is written once.
#include "kernels_common.h"
#include "mfma_b3.h"

namespace ag {
namespace {


constexpr int kKSdef = 16;         // K rows staged per step
constexpr int kMaxChunks = 512;    // K-splits (partials) per output tile
constexpr int kMaxChunksSmall = 2048;   // ... for the 64 x 64 tile: short steps need more work-groups in flight

inline bool tn_small_tile(int32_t m, int32_t n) { return n > 32 && n <= 64 && m <= 64; }
inline int tn_max_chunks(int32_t m, int32_t n) { return tn_small_tile(m, n) ? kMaxChunksSmall : kMaxChunks; }

// load 4 consecutive floats of row `r` starting at column c (zero beyond `cols` / `rows`)
__device__ __forceinline__ float4 guarded_load4(const float *__restrict__ M, int64_t r, int64_t rows,
                                                int c, int cols, bool vec_ok)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r >= rows || c >= cols) return v;
    const float *p = M + r * cols + c;
    if (vec_ok && c + 3 < cols) return *reinterpret_cast<const float4 *>(p);
    v.x = p[0];
    if (c + 1 < cols) v.y = p[1];
    if (c + 2 < cols) v.z = p[2];
    if (c + 3 < cols) v.w = p[3];
    return v;
}

// WAVES_M x WAVES_N wavefronts (= 4), each owning WM x WN tiles of 32 x 32.
template <int WAVES_M, int WAVES_N, int WM, int WN, int kKS>
__global__ __launch_bounds__(kWG) void k_gemm_tn(const float *__restrict__ A, const float *__restrict__ B,
                                                 float *__restrict__ part, int64_t K, int m, int n,
                                                 int64_t rows_per_chunk, float *__restrict__ colsum_part)
{
    constexpr int TM = WAVES_M * WM * 32, TN = WAVES_N * WN * 32;
    constexpr int NA = kKS * TM / 4, NB = kKS * TN / 4;                 // float4 units per stage
    constexpr int UA = (NA + kWG - 1) / kWG, UB = (NB + kWG - 1) / kWG; // ... per thread
    __shared__ float sA[2][kKS][TM];
    __shared__ float sB[2][kKS][TN];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int wm = w / WAVES_N, wn = w % WAVES_N;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.z * TN;
    const int64_t k_begin = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t k_end = min(K, k_begin + rows_per_chunk);
    const bool va = (m % 4 == 0), vb = (n % 4 == 0);

    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[UA], rb[UB], cs[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) cs[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool want_cs = colsum_part != nullptr && blockIdx.y == 0;
    // interior tiles (all columns present, 16-byte aligned rows) take unguarded 16-byte loads
    const bool interior = va && vb && m0 + TM <= m && n0 + TN <= n;
    auto fetch_fast = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (TM / 4), c = (idx % (TM / 4)) * 4;
            if (idx < NA) ra[u] = *reinterpret_cast<const float4 *>(A + (k0 + r) * m + m0 + c);
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NB) {
                rb[u] = *reinterpret_cast<const float4 *>(B + (k0 + r) * n + n0 + c);
                cs[u].x += rb[u].x; cs[u].y += rb[u].y; cs[u].z += rb[u].z; cs[u].w += rb[u].w;
            }
        }
    };
    auto fetch_safe = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (TM / 4), c = (idx % (TM / 4)) * 4;
            if (idx < NA) ra[u] = guarded_load4(A, k0 + r, k_end, m0 + c, m, va);
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NB) {
                rb[u] = guarded_load4(B, k0 + r, k_end, n0 + c, n, vb);
                cs[u].x += rb[u].x; cs[u].y += rb[u].y; cs[u].z += rb[u].z; cs[u].w += rb[u].w;
            }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (TM / 4), c = (idx % (TM / 4)) * 4;
            if (idx < NA) *reinterpret_cast<float4 *>(&sA[buf][r][c]) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NB) *reinterpret_cast<float4 *>(&sB[buf][r][c]) = rb[u];
        }
    };

    auto fetch = [&](int64_t k0) {
        if (interior && k0 + kKS <= k_end) fetch_fast(k0);
        else fetch_safe(k0);
    };
    if (k_begin < k_end) {
        fetch(k_begin);
        stash(0);
    }
    __syncthreads();
    int buf = 0;
    for (int64_t k0 = k_begin; k0 < k_end; k0 += kKS) {
        const bool more = k0 + kKS < k_end;
        if (more) fetch(k0 + kKS);
#pragma unroll
        for (int s = 0; s < kKS / 2; ++s) {
            float a[WM], b[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) a[i] = sA[buf][2 * s + hi][(wm * WM + i) * 32 + lo];
#pragma unroll
            for (int j = 0; j < WN; ++j) b[j] = sB[buf][2 * s + hi][(wn * WN + j) * 32 + lo];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    if (want_cs) {
        // threads that loaded the same columns (different staged rows) are combined through LDS
        float *red = &sB[0][0][0];                    // kKS x TN floats, free after the last barrier
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NB) *reinterpret_cast<float4 *>(&red[r * TN + c]) = cs[u];
        }
        __syncthreads();
        for (int c = tid; c < TN; c += kWG) {
            float t = 0.f;
#pragma unroll
            for (int r = 0; r < kKS; ++r) t += red[r * TN + c];
            if (n0 + c < n) colsum_part[(size_t)blockIdx.x * n + n0 + c] = t;
        }
    }
    float *out = part + (size_t)blockIdx.x * m * n;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int col = n0 + (wn * WN + j) * 32 + lo;
            if (col >= n) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * WM + i) * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (row < m) out[(size_t)row * n + col] = acc[i][j][r];
            }
        }
}

// The same product without LDS: the fp32 matrix instruction takes A[k + (l >> 5)][m0 + (l & 31)] and
// B[k + (l >> 5)][n0 + (l & 31)] as operands of lane l, which are plain coalesced 4-byte loads of
// the two row-major inputs, so every wave streams its own operands from global memory (the
// neighbouring wave's copy comes from L1) with KU k-steps of loads in flight and no barrier.
template <int WM, int WN, int KU>
__global__ __launch_bounds__(kWG) void k_gemm_tn_direct(const float *__restrict__ A, const float *__restrict__ B,
                                                        float *__restrict__ part, int64_t K, int m, int n,
                                                        int64_t rows_per_chunk, float *__restrict__ colsum_part)
{
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int wm = w >> 1, wn = w & 1;
    const int m0 = blockIdx.y * (2 * WM * 32) + wm * WM * 32, n0 = blockIdx.z * (2 * WN * 32) + wn * WN * 32;
    const int64_t k_begin = (int64_t)blockIdx.x * rows_per_chunk, k_end = min(K, k_begin + rows_per_chunk);
    bool am[WM], bn[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) am[i] = m0 + 32 * i + lo < m;
#pragma unroll
    for (int j = 0; j < WN; ++j) bn[j] = n0 + 32 * j + lo < n;
    floatx16 acc[WM][WN];
    float cs[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        cs[j] = 0.f;
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    }
    for (int64_t k0 = k_begin; k0 < k_end; k0 += 2 * KU) {
        float a[KU][WM], b[KU][WN];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const int64_t row = k0 + 2 * u + hi;
            const bool ok = row < k_end;
#pragma unroll
            for (int i = 0; i < WM; ++i) a[u][i] = (ok && am[i]) ? A[row * m + m0 + 32 * i + lo] : 0.f;
#pragma unroll
            for (int j = 0; j < WN; ++j) b[u][j] = (ok && bn[j]) ? B[row * n + n0 + 32 * j + lo] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) {
#pragma unroll
            for (int j = 0; j < WN; ++j) cs[j] += b[u][j];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][i], b[u][j], acc[i][j], 0, 0, 0);
        }
    }
    if (colsum_part != nullptr && blockIdx.y == 0 && wm == 0) {
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const float t = cs[j] + __shfl_xor(cs[j], 32);
            if (hi == 0 && bn[j]) colsum_part[(size_t)blockIdx.x * n + n0 + 32 * j + lo] = t;
        }
    }
    float *out = part + (size_t)blockIdx.x * m * n;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            if (!bn[j]) continue;
            const int col = n0 + 32 * j + lo;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + 32 * i + 8 * (r >> 2) + 4 * hi + (r & 3);
                if (row < m) out[(size_t)row * n + col] = acc[i][j][r];
            }
        }
}

__global__ __launch_bounds__(kWG) void k_sum_partials(int nchunks, int per_group, int64_t count,
                                                      const float *__restrict__ part, float *__restrict__ C)
{
    // 32 outputs per work-group, 8 slices of the partials per output, combined through LDS in a
    // fixed order (bitwise reproducible).  blockIdx.y selects a group of `per_group` partials whose
    // sum goes to C[group][count] (one group = the plain case).
    __shared__ float red[kWG];
    const int64_t i = (int64_t)blockIdx.x * 32 + (threadIdx.x & 31);
    const int slice = threadIdx.x >> 5;
    const int q0 = blockIdx.y * per_group, q1 = min(nchunks, q0 + per_group);
    const float s = (i < count) ? sum_strided(part + i, (size_t)count, q0 + slice, q1, 8) : 0.f;
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x < 32 && i < count) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += red[k * 32 + threadIdx.x];
        C[(size_t)blockIdx.y * count + i] = t;
    }
}

constexpr int kSumGroup = 128;     // partials per first-stage group when there are many K-splits

// C[count] = sum of nchunks partials; with many partials in two stages (scratch2: ceil(nchunks /
// kSumGroup) * count floats) so that the first stage fills the chip
void sum_partials(int nchunks, int64_t count, const float *part, float *C, float *scratch2, hipStream_t st)
{
    const unsigned gx = (unsigned)((count + 31) / 32);
    if (nchunks <= kMaxChunks || !scratch2) {
        hipLaunchKernelGGL(k_sum_partials, dim3(gx), dim3(kWG), 0, st, nchunks, nchunks, count, part, C);
        return;
    }
    const int groups = (nchunks + kSumGroup - 1) / kSumGroup;
    hipLaunchKernelGGL(k_sum_partials, dim3(gx, groups), dim3(kWG), 0, st, nchunks, kSumGroup, count, part, scratch2);
    hipLaunchKernelGGL(k_sum_partials, dim3(gx), dim3(kWG), 0, st, groups, groups, count, scratch2, C);
}

// ------------------------------------------------------------------------------------------
// C[N x n] = epilogue(A[N x k] W[k x n])
// ------------------------------------------------------------------------------------------
enum { EPI_NONE = 0, EPI_BIAS_RELU = 1, EPI_RELU_MASK = 2 };
// kNK = k columns of A / rows of W staged per step: 16 for the wide tile (register budget), 64 for
// the narrow one (bandwidth-bound shape: whole 256-byte row pieces, fewer barriers)
template <int WAVES_M, int WAVES_N, int WM, int WN, int EPI, int kNK>
__global__ __launch_bounds__(kWG, 2) void k_gemm_nn(const float *__restrict__ A, const float *__restrict__ W,
                                                 float *__restrict__ C, int64_t N, int k, int n,
                                                 const float *__restrict__ aux)
{
    constexpr int TM = WAVES_M * WM * 32, TN = WAVES_N * WN * 32;
    constexpr int LDA = kNK + 1;                                        // padded: conflict-free operand reads
    constexpr int NA = TM * kNK / 4, NW = kNK * TN / 4;
    constexpr int UA = (NA + kWG - 1) / kWG, UW = (NW + kWG - 1) / kWG;
    __shared__ float sA[TM * LDA];
    __shared__ float sW[kNK][TN];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int wm = w / WAVES_N, wn = w % WAVES_N;
    const int64_t r0 = (int64_t)blockIdx.x * TM;
    const int n0 = blockIdx.y * TN;
    const bool va = (k % 4 == 0), vw = (n % 4 == 0);

    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[UA], rw[UW];
    const bool interior = va && vw && r0 + TM <= N && n0 + TN <= n;
    auto fetch_fast = [&](int k0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (kNK / 4), c = (idx % (kNK / 4)) * 4;
            if (idx < NA) ra[u] = *reinterpret_cast<const float4 *>(A + (r0 + r) * k + k0 + c);
        }
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NW) rw[u] = *reinterpret_cast<const float4 *>(W + (size_t)(k0 + r) * n + n0 + c);
        }
    };
    auto fetch_safe = [&](int k0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (kNK / 4), c = (idx % (kNK / 4)) * 4;
            if (idx < NA) ra[u] = guarded_load4(A, r0 + r, N, k0 + c, k, va);
        }
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NW) rw[u] = guarded_load4(W, k0 + r, k, n0 + c, n, vw);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (kNK / 4), c = (idx % (kNK / 4)) * 4;
            if (idx < NA) {
                float *d = &sA[r * LDA + c];
                d[0] = ra[u].x; d[1] = ra[u].y; d[2] = ra[u].z; d[3] = ra[u].w;
            }
        }
#pragma unroll
        for (int u = 0; u < UW; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NW) *reinterpret_cast<float4 *>(&sW[r][c]) = rw[u];
        }
    };

    auto fetch = [&](int k0) {
        if (interior && k0 + kNK <= k) fetch_fast(k0);
        else fetch_safe(k0);
    };
    fetch(0);
    for (int k0 = 0; k0 < k; k0 += kNK) {
        __syncthreads();                       // everyone is done reading the previous tiles
        stash();
        __syncthreads();
        if (k0 + kNK < k) fetch(k0 + kNK);
#pragma unroll
        for (int s = 0; s < kNK / 2; ++s) {
            float a[WM], b[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) a[i] = sA[((wm * WM + i) * 32 + lo) * LDA + 2 * s + hi];
#pragma unroll
            for (int j = 0; j < WN; ++j) b[j] = sW[2 * s + hi][(wn * WN + j) * 32 + lo];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
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

// out[c][r] = in[r][c] for a small rows x cols matrix
__global__ __launch_bounds__(kWG) void k_transpose_small(int rows, int cols, const float *__restrict__ in,
                                                         float *__restrict__ out)
{
    const int i = blockIdx.x * kWG + threadIdx.x;
    if (i >= rows * cols) return;
    const int r = i / cols, c = i % cols;
    out[(size_t)c * rows + r] = in[i];
}

// Small inner dimension (k <= KMAX): a bandwidth-bound outer-product update on the vector ALUs.
// A thread owns 4 consecutive output columns; its slice of W lives in registers and is reused
// for ROWS consecutive rows per work-group pass.
template <int KMAX, int EPI>
__global__ __launch_bounds__(kWG) void k_gemm_nn_smallk(const float *__restrict__ A, const float *__restrict__ W,
                                                        float *__restrict__ C, int64_t N, int k, int n,
                                                        const float *__restrict__ aux, int rows_per_wg)
{
    const int tpr = (n + 3) / 4;                         // threads per row, <= kWG
    const int rows_at_once = kWG / tpr;
    const int sub = threadIdx.x / tpr, c = (threadIdx.x % tpr) * 4;
    if (sub >= rows_at_once) return;
    float4 wreg[KMAX];
#pragma unroll
    for (int q = 0; q < KMAX; ++q) wreg[q] = guarded_load4(W, q, k, c, n, (n % 4) == 0);
    float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
    if constexpr (EPI == EPI_BIAS_RELU) bias = guarded_load4(aux, 0, 1, c, n, (n % 4) == 0);
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t re = min(N, rb + rows_per_wg);
    const bool vec = (n % 4 == 0), va = (k % 4 == 0);
    constexpr int RU = 2;                                // rows in flight per thread
    for (int64_t row0 = rb + sub; row0 < re; row0 += (int64_t)RU * rows_at_once) {
        float4 a[RU][KMAX / 4], mk[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int64_t row = row0 + (int64_t)u * rows_at_once;
#pragma unroll
            for (int q4 = 0; q4 < KMAX; q4 += 4) a[u][q4 / 4] = guarded_load4(A, row, re, q4, k, va);
            mk[u] = make_float4(1.f, 1.f, 1.f, 1.f);
            if constexpr (EPI == EPI_RELU_MASK) mk[u] = guarded_load4(aux, row, re, c, n, vec);
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int64_t row = row0 + (int64_t)u * rows_at_once;
            if (row >= re) break;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int q4 = 0; q4 < KMAX; q4 += 4) {
                const float av[4] = {a[u][q4 / 4].x, a[u][q4 / 4].y, a[u][q4 / 4].z, a[u][q4 / 4].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc.x = fmaf(av[j], wreg[q4 + j].x, acc.x);
                    acc.y = fmaf(av[j], wreg[q4 + j].y, acc.y);
                    acc.z = fmaf(av[j], wreg[q4 + j].z, acc.z);
                    acc.w = fmaf(av[j], wreg[q4 + j].w, acc.w);
                }
            }
            if constexpr (EPI == EPI_BIAS_RELU) {
                acc.x = fmaxf(acc.x + bias.x, 0.f); acc.y = fmaxf(acc.y + bias.y, 0.f);
                acc.z = fmaxf(acc.z + bias.z, 0.f); acc.w = fmaxf(acc.w + bias.w, 0.f);
            }
            if constexpr (EPI == EPI_RELU_MASK) {
                acc.x = mk[u].x > 0.f ? acc.x : 0.f; acc.y = mk[u].y > 0.f ? acc.y : 0.f;
                acc.z = mk[u].z > 0.f ? acc.z : 0.f; acc.w = mk[u].w > 0.f ? acc.w : 0.f;
            }
            float *o = C + row * n + c;
            if (vec && c + 3 < n) {
                *reinterpret_cast<float4 *>(o) = acc;
            } else {
                const float ov[4] = {acc.x, acc.y, acc.z, acc.w};
                for (int j = 0; j < 4 && c + j < n; ++j) o[j] = ov[j];
            }
        }
    }
}

// Backward through the second GCN layer's transform in one pass over H1 and dQ (both are read
// once): dPre = (dQ W2^T) * (H1 > 0) is written, and the weight gradient dW2 = H1^T dQ is
// accumulated on the way.  A thread owns 4 hidden columns; its slice of W2^T and its 4 x KMAX
// piece of dW2 live in registers; one wavefront's rows are reduced by a second kernel from
// per-wavefront partials (fixed order).  Bandwidth bound, vector ALUs only.
template <int KMAX>
__global__ __launch_bounds__(kWG) void k_hidden_backward(const float *__restrict__ dQ,
                                                         const float *__restrict__ W2T,
                                                         const float *__restrict__ H1, float *__restrict__ dPre,
                                                         float *__restrict__ part, int64_t N, int c, int hd,
                                                         int rows_per_wg)
{
    const int tpr = hd / 4;                              // threads per row (hd % 4 == 0, tpr <= kWG)
    const int rows_at_once = kWG / tpr;
    const int sub = threadIdx.x / tpr, col = (threadIdx.x % tpr) * 4;
    const bool active = sub < rows_at_once;              // left-over threads only take part in the barrier
    float4 wreg[KMAX], gw[KMAX];                         // W2^T slice; dW2[col..col+3][q] accumulators
#pragma unroll
    for (int q = 0; q < KMAX; ++q) {
        wreg[q] = (q < c) ? *reinterpret_cast<const float4 *>(W2T + (size_t)q * hd + col) : make_float4(0.f, 0.f, 0.f, 0.f);
        gw[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg, re = active ? min(N, rb + rows_per_wg) : rb;
    const bool vq = (c % 4 == 0);
    // software pipeline: the loads of the next row are in flight while the current row is computed
    float4 h_n = make_float4(0.f, 0.f, 0.f, 0.f), a_n[KMAX / 4];
    auto fetch = [&](int64_t row) {
        if (row < re) h_n = *reinterpret_cast<const float4 *>(H1 + row * hd + col);
#pragma unroll
        for (int q4 = 0; q4 < KMAX; q4 += 4) a_n[q4 / 4] = guarded_load4(dQ, row, re, q4, c, vq);
    };
    fetch(rb + sub);
    for (int64_t row = rb + sub; row < re; row += rows_at_once) {
        const float4 h = h_n;
        float a[KMAX];
#pragma unroll
        for (int q4 = 0; q4 < KMAX; q4 += 4) {
            a[q4] = a_n[q4 / 4].x; a[q4 + 1] = a_n[q4 / 4].y; a[q4 + 2] = a_n[q4 / 4].z; a[q4 + 3] = a_n[q4 / 4].w;
        }
        fetch(row + rows_at_once);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int q = 0; q < KMAX; ++q) {
            acc.x = fmaf(a[q], wreg[q].x, acc.x); acc.y = fmaf(a[q], wreg[q].y, acc.y);
            acc.z = fmaf(a[q], wreg[q].z, acc.z); acc.w = fmaf(a[q], wreg[q].w, acc.w);
            gw[q].x = fmaf(h.x, a[q], gw[q].x); gw[q].y = fmaf(h.y, a[q], gw[q].y);
            gw[q].z = fmaf(h.z, a[q], gw[q].z); gw[q].w = fmaf(h.w, a[q], gw[q].w);
        }
        acc.x = h.x > 0.f ? acc.x : 0.f; acc.y = h.y > 0.f ? acc.y : 0.f;
        acc.z = h.z > 0.f ? acc.z : 0.f; acc.w = h.w > 0.f ? acc.w : 0.f;
        *reinterpret_cast<float4 *>(dPre + row * hd + col) = acc;
    }
    // the row groups of the work-group are combined through LDS (fixed order), then one partial
    // dW2 per work-group goes out: part[wg][hd][c]
    extern __shared__ float red[];                        // (rows_at_once - 1) x hd x KMAX floats
    if (active && sub > 0) {
        float *r = red + ((size_t)(sub - 1) * hd + col) * KMAX;
#pragma unroll
        for (int q = 0; q < KMAX; ++q) {
            r[0 * KMAX + q] = gw[q].x; r[1 * KMAX + q] = gw[q].y;
            r[2 * KMAX + q] = gw[q].z; r[3 * KMAX + q] = gw[q].w;
        }
    }
    __syncthreads();
    if (sub == 0) {
        for (int g = 1; g < rows_at_once; ++g) {
            const float *r = red + ((size_t)(g - 1) * hd + col) * KMAX;
#pragma unroll
            for (int q = 0; q < KMAX; ++q) {
                gw[q].x += r[0 * KMAX + q]; gw[q].y += r[1 * KMAX + q];
                gw[q].z += r[2 * KMAX + q]; gw[q].w += r[3 * KMAX + q];
            }
        }
        float *o = part + (size_t)blockIdx.x * hd * c;
#pragma unroll
        for (int q = 0; q < KMAX; ++q)
            if (q < c) {
                o[(size_t)(col + 0) * c + q] = gw[q].x;
                o[(size_t)(col + 1) * c + q] = gw[q].y;
                o[(size_t)(col + 2) * c + q] = gw[q].z;
                o[(size_t)(col + 3) * c + q] = gw[q].w;
            }
    }
}

// The same backward step on the fp32 matrix instruction, for hd in {64, 128, 256} and c <= 16, without
// LDS.  A wavefront owns a slice of 64 hidden columns and walks blocks of 32 rows:
//   part 1  dPre tile = dQ[32 x 16] . W2T[16 x 64]: the A operand (a row of dQ per lane) comes
//           straight from global memory, the B operand (the wave's slice of W2T) stays in registers;
//   the H1 values of the block are loaded once, in the result layout of the instruction (register r
//           of lane l holds row 8 (r / 4) + 4 (l >> 5) + (r & 3), column l & 31): they mask the dPre
//           tile, and the very same registers are the A operand of
//   part 2  dW2 slice += H1^T . dQ, whose k index may run over the block's rows in any order: step s
//           uses the row that result register s holds, so no data has to move between lanes.
// With fewer than four column slices the spare wavefronts take the next row blocks.  Every
// wavefront ends with its own partial of dW2; a second kernel adds them in a fixed order.
__global__ __launch_bounds__(kWG) void k_hidden_backward_mfma(const float *__restrict__ dQ,
                                                              const float *__restrict__ W2T,
                                                              const float *__restrict__ H1, float *__restrict__ dPre,
                                                              float *__restrict__ part, int64_t N, int c, int hd,
                                                              int rows_per_wg)
{
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    // a wavefront owns 32 hidden columns; the work-group's 4 wavefronts cover 128 columns of one
    // 32-row block (hd = 128: one pass; hd = 256: blockIdx.y picks the half; hd = 64: two row blocks)
    const int CS = min(hd / 32, 4), RS = 4 / CS;         // column slices per work-group; row sub-blocks per pass
    const int slice = w % CS, rsub = w / CS;
    const int col0 = blockIdx.y * 128 + slice * 32;
    float bw[8];                                         // B operand of part 1: W2T[2 s + hi][col0 + lo]
#pragma unroll
    for (int s = 0; s < 8; ++s) bw[s] = (2 * s + hi < c) ? W2T[(size_t)(2 * s + hi) * hd + col0 + lo] : 0.f;
    floatx16 acc2;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[r] = 0.f;
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg, re = min(N, rb + rows_per_wg);
    const bool c16 = (c == 16);
    for (int64_t R0 = rb + 32 * rsub; R0 < re; R0 += 32 * RS) {
        // the lane's row of dQ (A operand of part 1), the dQ values in B-operand layout for part 2,
        // and the H1 values of the block: all loads first
        float q[16], b2[16], h[16];
        if (c16 && R0 + lo < re) {
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                const float4 v = *reinterpret_cast<const float4 *>(dQ + (R0 + lo) * 16 + 4 * j4);
                q[4 * j4] = v.x; q[4 * j4 + 1] = v.y; q[4 * j4 + 2] = v.z; q[4 * j4 + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) q[j] = (R0 + lo < re && j < c) ? dQ[(R0 + lo) * c + j] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = R0 + 8 * (r >> 2) + 4 * hi + (r & 3);
            h[r] = row < re ? H1[row * hd + col0 + lo] : 0.f;
            b2[r] = (row < re && lo < c) ? dQ[row * c + lo] : 0.f;
        }
        floatx16 d;
#pragma unroll
        for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) d = __builtin_amdgcn_mfma_f32_32x32x2f32(hi ? q[2 * s + 1] : q[2 * s], bw[s], d, 0, 0, 0);
        // part 2: step s takes the row held by result register s
#pragma unroll
        for (int s = 0; s < 16; ++s) acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(h[s], b2[s], acc2, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = R0 + 8 * (r >> 2) + 4 * hi + (r & 3);
            if (row < re) dPre[row * hd + col0 + lo] = h[r] > 0.f ? d[r] : 0.f;
        }
    }
    // partial (blockIdx.x, rsub) is filled by the wavefronts (and, for hd = 256, the two work-groups)
    // that share these rows: each writes its own 32 columns
    float *o = part + ((size_t)blockIdx.x * RS + rsub) * hd * c;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = col0 + 8 * (r >> 2) + 4 * hi + (r & 3);
        if (lo < c) o[(size_t)m * c + lo] = acc2[r];
    }
}

// The whole backward pass through the two dense transforms of a two-layer GCN in ONE pass over
// P, H1 and dQ, without ever writing dPre (N x hd) to memory:
//     dPre = (dQ W2^T) * (H1 > 0)       stays in registers
//     dW2 += H1^T dQ,   dW1 += P^T dPre,   db1 += column sums of dPre
// Same decomposition as k_hidden_backward_mfma (a wavefront owns 32 hidden columns and walks blocks
// of 32 rows; the dPre tile comes out in the result layout of the fp32 matrix instruction).  That
// tile is at once the B operand of the dW1 product: its k index runs over the block's rows in the
// order the result registers hold them (step s: row 8 (s / 4) + 4 (l >> 5) + (s & 3)), and the A
// operands P^T of that step are one contiguous load of P[that row][FI32 (l & 31) ...] per lane.
// With B3 the dW1 product runs on the bf16 instruction at fp32 accuracy: the eight values a lane
// holds for eight k-steps are cut into three bf16 pieces each and are, as they stand, its operand.
// FI32 = f_in / 32 row tiles of dW1 per wavefront.  Every wavefront ends with its partial of
// dW1[:, 32 columns], dW2[32 rows, :] and db1[32 columns]; fixed-order sums follow.
template <int FI32>
struct FusedBlock {                                  // everything one wavefront reads of a block of 32 rows
    float q[16];                                     // the lane's row of dQ (A operand of the dPre product)
    float b2[16];                                    // dQ in B-operand layout for the dW2 product
    float h[16];                                     // H1 in the result layout of the instruction
    float a[16][FI32];                               // P^T operands of the 16 k-steps of the dW1 product
};

template <int FI32, bool B3>
__global__ __launch_bounds__(kWG, 1) void k_gcn_backward_fused(const float *__restrict__ dQ, const float *__restrict__ W2T,
                                                            const float *__restrict__ H1, const float *__restrict__ P,
                                                            float *__restrict__ part_w1, float *__restrict__ part_w2,
                                                            float *__restrict__ part_b1, int64_t N, int c, int hd,
                                                            int rows_per_wg)
{
    constexpr int fi = FI32 * 32;
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int CS = min(hd / 32, 4), RS = 4 / CS;         // column slices per work-group; row sub-blocks per pass
    const int slice = w % CS, rsub = w / CS;
    const int col0 = blockIdx.y * 128 + slice * 32;
    float bw[8];                                         // B operand of the dPre product: W2T[2 s + hi][col0 + lo]
#pragma unroll
    for (int s = 0; s < 8; ++s) bw[s] = (2 * s + hi < c) ? W2T[(size_t)(2 * s + hi) * hd + col0 + lo] : 0.f;
    floatx16 acc2, acc1[FI32];
    float cs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[r] = 0.f;
#pragma unroll
    for (int i = 0; i < FI32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[i][r] = 0.f;
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg, re = min(N, rb + rows_per_wg);
    const bool c16 = (c == 16);
    // Loads are unconditional (addresses clamped into the arrays, values selected afterwards): a
    // load under a branch would force the following wait to drain ALL outstanding loads, the next
    // block's included.  Row tile i of dW1 takes the features FI32 * lane + i, so the P^T operands
    // of all FI32 tiles of one k-step are ONE contiguous load of FI32 floats per lane.
    const int qc = min(lo, c - 1);
    auto load = [&](FusedBlock<FI32> &B, int64_t R0) {
        {
            const int64_t row = min(R0 + lo, N - 1);
            if (c16) {
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const float4 v = *reinterpret_cast<const float4 *>(dQ + row * 16 + 4 * j4);
                    B.q[4 * j4] = v.x; B.q[4 * j4 + 1] = v.y; B.q[4 * j4 + 2] = v.z; B.q[4 * j4 + 3] = v.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) B.q[j] = dQ[row * c + min(j, c - 1)];
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = min(R0 + 8 * (r >> 2) + 4 * hi + (r & 3), N - 1);
            B.h[r] = H1[row * hd + col0 + lo];
            B.b2[r] = dQ[row * c + qc];
            load_vec<FI32 == 3 ? 1 : FI32>(P + row * fi + FI32 * lo, reinterpret_cast<float (&)[FI32 == 3 ? 1 : FI32]>(B.a[r][0]));
            if constexpr (FI32 == 3) { B.a[r][1] = P[row * fi + 3 * lo + 1]; B.a[r][2] = P[row * fi + 3 * lo + 2]; }
        }
    };
    // values of rows beyond the end of the work-group's range, and of classes beyond c, count as 0
    auto mask = [&](FusedBlock<FI32> &B, int64_t R0) {
        const bool rq = R0 + lo < re;
#pragma unroll
        for (int j = 0; j < 16; ++j) B.q[j] = (rq && j < c) ? B.q[j] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = R0 + 8 * (r >> 2) + 4 * hi + (r & 3) < re;
            B.h[r] = ok ? B.h[r] : 0.f;
            B.b2[r] = (ok && lo < c) ? B.b2[r] : 0.f;
#pragma unroll
            for (int i = 0; i < FI32; ++i) B.a[r][i] = ok ? B.a[r][i] : 0.f;
        }
    };
    auto compute = [&](const FusedBlock<FI32> &B) {
        floatx16 d;
#pragma unroll
        for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) d = __builtin_amdgcn_mfma_f32_32x32x2f32(hi ? B.q[2 * s + 1] : B.q[2 * s], bw[s], d, 0, 0, 0);
#pragma unroll
        for (int s = 0; s < 16; ++s) acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(B.h[s], B.b2[s], acc2, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {                   // ReLU mask; rows beyond the end hold h = 0
            d[r] = B.h[r] > 0.f ? d[r] : 0.f;
            cs += d[r];
        }
        // dW1[rows of tile i][col0 .. col0 + 31] += P^T dPre: k-step s takes the row that register s holds
        if constexpr (B3) {
            // on the bf16 instruction at fp32 accuracy: sixteen k-steps are two instructions of eight, the
            // eight values a lane holds for one of them are exactly its operand (cut into three pieces)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                float dv[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) dv[t] = d[8 * half + t];
                u32x4 pd[3];
                cut3x8(dv, pd);
#pragma unroll
                for (int i = 0; i < FI32; ++i) {
                    float av[8];
#pragma unroll
                    for (int t = 0; t < 8; ++t) av[t] = B.a[8 * half + t][i];
                    u32x4 pa[3];
                    cut3x8(av, pa);
                    acc1[i] = mfma16_b3(pa, pd, acc1[i]);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 16; ++s)
#pragma unroll
                for (int i = 0; i < FI32; ++i)
                    acc1[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(B.a[s][i], d[s], acc1[i], 0, 0, 0);
        }
    };
    {
        // One wavefront per SIMD with two register sets: all loads of the next block are in flight
        // while the 24 + 16 FI32 matrix instructions of the current block run.  The next block is
        // always requested, also behind the last one (clamped addresses make that harmless): no
        // branch may sit between a block's loads and the work on the block before it.
        FusedBlock<FI32> A, B;
        const int64_t step = 32 * RS;
        int64_t R0 = rb + 32 * rsub;
        if (R0 < re) {                                   // uniform over the wavefront
            load(A, R0);
            for (;;) {
                load(B, R0 + step);
                mask(A, R0);
                compute(A);
                R0 += step;
                if (R0 >= re) break;
                load(A, R0 + step);
                mask(B, R0);
                compute(B);
                R0 += step;
                if (R0 >= re) break;
            }
        }
    }
    const size_t pidx = (size_t)blockIdx.x * RS + rsub;  // partial shared by the wavefronts (and the work-groups
                                                         // of the other column halves) that walked these rows
    float *o2 = part_w2 + pidx * hd * c;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = col0 + 8 * (r >> 2) + 4 * hi + (r & 3);
        if (lo < c) o2[(size_t)m * c + lo] = acc2[r];
    }
    float *o1 = part_w1 + pidx * fi * hd;
#pragma unroll
    for (int i = 0; i < FI32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = FI32 * (8 * (r >> 2) + 4 * hi + (r & 3)) + i;    // the feature that row of tile i stands for
            o1[(size_t)m * hd + col0 + lo] = acc1[i][r];
        }
    const float t = cs + __shfl_xor(cs, 32);
    if (hi == 0) part_b1[pidx * hd + col0 + lo] = t;
}

// The same fused backward with the operands of the dW1 product staged through LDS: for hidden
// widths of 128 and 256 a work-group of NW = hd / 32 wavefronts covers ALL hidden columns of a
// block of 32 rows, so the block of P is read and cut into bf16 pieces once per work-group (8
// values per thread) instead of once per wavefront, and the wavefronts fetch their P^T operands
// with two 8-byte LDS reads per piece.  LDS layout of a block: sP[piece][feature][row] in bf16, a
// feature's 32 rows taking 64 bytes of a 72-byte line (lanes of a read phase on distinct banks); the row order inside a line is the natural one, and the operand
// of k-slot (hi, t) of instruction `half` is row 16 half + 8 (t / 4) + 4 hi + (t & 3): two runs of
// four consecutive rows.  dQ goes through LDS as well, cut into pieces, in both orientations (all
// three products run on the bf16 instruction); H1 comes straight from
// global memory in the result layout of the instruction, one block ahead.  Two LDS buffers, one
// barrier per block: the next block's global loads are issued before the work on the current
// one and written to the other buffer behind it.  All loads are unconditional (clamped rows).
template <int FI32, int NW>
__global__ __launch_bounds__(64 * NW, 1) void k_gcn_backward_lds(const float *__restrict__ dQ, const float *__restrict__ W2T,
                                                                 const float *__restrict__ H1, const float *__restrict__ P,
                                                                 float *__restrict__ part_w1, float *__restrict__ part_w2,
                                                                 float *__restrict__ part_b1, int64_t N, int c, int rows_per_wg)
{
    constexpr int fi = FI32 * 32, hd = NW * 32, T = 64 * NW;
    // bytes per (piece, feature) line: 32 rows x 2 + 8.  The 8-byte reads of the lanes (feature lo,
    // hi = const) then start 18 banks apart: sixteen consecutive lanes cover 32 distinct banks
    // (with 80-byte lines lanes lo and lo + 8 met in one bank and every read took two turns)
    constexpr int kLine = 72;
    constexpr int PV = 32 * fi / T;                        // values of the P block per thread
    static_assert(PV == 8 || PV == 16 || PV == 4, "a thread stages whole groups of rows of one feature");
    static_assert(T % fi == 0 || fi % T == 0, "threads map to (feature, row group)");
    __shared__ __attribute__((aligned(16))) unsigned char sP[2][3 * fi * kLine];
    // dQ in pieces, twice: row-major (32-byte lines: the operand of the dPre product) and
    // class-major (80-byte lines like sP: the operand of the dW2 product)
    __shared__ __attribute__((aligned(16))) unsigned char sQr[2][3 * 32 * 32];
    __shared__ __attribute__((aligned(16))) unsigned char sQc[2][3 * 16 * kLine];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lo = l & 31, hi = l >> 5;
    const int col0 = w * 32;
    const int64_t rb = (int64_t)blockIdx.x * rows_per_wg, re = min(N, rb + rows_per_wg);
    u32x4 w2b[3];                                          // operand of the dPre product: W2T[8 hi + t][col0 + lo], in pieces
    {
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = (8 * hi + t < c) ? W2T[(size_t)(8 * hi + t) * hd + col0 + lo] : 0.f;
        cut3x8(v, w2b);
    }
    floatx16 acc2, acc1[FI32];
    float cs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[r] = 0.f;
#pragma unroll
    for (int i = 0; i < FI32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[i][r] = 0.f;

    // staging roles: thread -> feature sf, rows sr0 .. sr0 + PV - 1 of the block (PV consecutive rows)
    constexpr int GROUPS = 32 / PV;                        // row groups per feature
    const int sf = tid % fi, sg = tid / fi;                // sg < GROUPS whenever T == fi * GROUPS
    static_assert(T == fi * GROUPS, "every (feature, row group) has exactly one thread");
    const int sr0 = sg * PV;
    const int qrow = tid >> 2, qc4 = (tid & 3) * 4;        // dQ: the first 128 threads take one float4 each (c == 16)

    float pv[PV], hn[16];
    float4 qv = make_float4(0.f, 0.f, 0.f, 0.f);
    auto fetch = [&](int64_t R0) {                         // global loads of block R0 into registers
#pragma unroll
        for (int j = 0; j < PV; ++j) {
            const int64_t row = min(R0 + sr0 + j, N - 1);
            pv[j] = P[row * fi + sf];
        }
        if (tid < 128) {
            const int64_t row = min(R0 + qrow, N - 1);
            if (c == 16) {
                qv = *reinterpret_cast<const float4 *>(dQ + row * 16 + qc4);
            } else {
                qv.x = dQ[row * c + min(qc4, c - 1)];
                qv.y = dQ[row * c + min(qc4 + 1, c - 1)];
                qv.z = dQ[row * c + min(qc4 + 2, c - 1)];
                qv.w = dQ[row * c + min(qc4 + 3, c - 1)];
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = min(R0 + 8 * (r >> 2) + 4 * hi + (r & 3), N - 1);
            hn[r] = H1[row * hd + col0 + lo];
        }
    };
    auto stash = [&](int buf, int64_t R0) {                // registers -> LDS buffer, rows beyond `re` as zeros
#pragma unroll
        for (int j0 = 0; j0 < PV; j0 += 8) {
            float v8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v8[j] = (R0 + sr0 + j0 + j < re) ? pv[j0 + j] : 0.f;
            u32x4 pc[3];
            cut3x8(v8, pc);
#pragma unroll
            for (int s = 0; s < 3; ++s)
            {                                          // lines are 8-byte aligned: two 8-byte writes
                unsigned char *d = &sP[buf][(s * fi + sf) * kLine + (sr0 + j0) * 2];
                *reinterpret_cast<uint2 *>(d) = make_uint2(pc[s][0], pc[s][1]);
                *reinterpret_cast<uint2 *>(d + 8) = make_uint2(pc[s][2], pc[s][3]);
            }
        }
        if (tid < 128) {
            const bool ok = R0 + qrow < re;
            uint32_t q0[3], q1[3], q2[3], q3[3];
            cut3((ok && qc4 < c) ? qv.x : 0.f, q0);
            cut3((ok && qc4 + 1 < c) ? qv.y : 0.f, q1);
            cut3((ok && qc4 + 2 < c) ? qv.z : 0.f, q2);
            cut3((ok && qc4 + 3 < c) ? qv.w : 0.f, q3);
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                *reinterpret_cast<uint2 *>(&sQr[buf][(s * 32 + qrow) * 32 + qc4 * 2]) =
                    make_uint2((q0[s] >> 16) | q1[s], (q2[s] >> 16) | q3[s]);
                unsigned char *col = &sQc[buf][(s * 16 + qc4) * kLine + qrow * 2];
                *reinterpret_cast<uint16_t *>(col) = (uint16_t)(q0[s] >> 16);
                *reinterpret_cast<uint16_t *>(col + kLine) = (uint16_t)(q1[s] >> 16);
                *reinterpret_cast<uint16_t *>(col + 2 * kLine) = (uint16_t)(q2[s] >> 16);
                *reinterpret_cast<uint16_t *>(col + 3 * kLine) = (uint16_t)(q3[s] >> 16);
            }
        }
    };

    float h[16];
    int buf = 0;
    if (rb < re) {                                         // uniform over the work-group
        fetch(rb);
        stash(0, rb);
#pragma unroll
        for (int r = 0; r < 16; ++r) h[r] = (rb + 8 * (r >> 2) + 4 * hi + (r & 3) < re) ? hn[r] : 0.f;
    }
    for (int64_t R0 = rb; R0 < re; R0 += 32, buf ^= 1) {
        __syncthreads();                                   // buffer `buf` is complete; the other one is free
        fetch(R0 + 32);                                    // always (clamped): no branch between loads and work
        floatx16 d;
#pragma unroll
        for (int r = 0; r < 16; ++r) d[r] = 0.f;
        {
            u32x4 qa[3];                                   // dQ[R0 + lo][8 hi + 0..7]
#pragma unroll
            for (int s = 0; s < 3; ++s) qa[s] = *reinterpret_cast<const u32x4 *>(&sQr[buf][(s * 32 + lo) * 32 + 16 * hi]);
            d = mfma16_b3(qa, w2b, d);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {             // dW2 += H1^T dQ, the block's rows in the k-slot order of the dW1 product
            float hv[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) hv[t] = h[8 * half + t];
            u32x4 ph[3], qb[3];
            cut3x8(hv, ph);
#pragma unroll
            for (int s = 0; s < 3; ++s) {                  // columns >= 16 of the result are not stored
                const unsigned char *line = &sQc[buf][(s * 16 + (lo & 15)) * kLine + (16 * half + 4 * hi) * 2];
                const uint2 x = *reinterpret_cast<const uint2 *>(line);
                const uint2 y = *reinterpret_cast<const uint2 *>(line + 16);
                qb[s] = u32x4{x.x, x.y, y.x, y.y};
            }
            acc2 = mfma16_b3(ph, qb, acc2);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            d[r] = h[r] > 0.f ? d[r] : 0.f;
            cs += d[r];
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float dv[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) dv[t] = d[8 * half + t];
            u32x4 pd[3];
            cut3x8(dv, pd);
#pragma unroll
            for (int i = 0; i < FI32; ++i) {
                u32x4 pa[3];
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const unsigned char *line = &sP[buf][(s * fi + 32 * i + lo) * kLine + (16 * half + 4 * hi) * 2];
                    const uint2 x = *reinterpret_cast<const uint2 *>(line);            // rows 16 half + 4 hi + 0..3
                    const uint2 y = *reinterpret_cast<const uint2 *>(line + 16);       // rows 16 half + 8 + 4 hi + 0..3
                    pa[s] = u32x4{x.x, x.y, y.x, y.y};
                }
                acc1[i] = mfma16_b3(pa, pd, acc1[i]);
            }
        }
        stash(buf ^ 1, R0 + 32);
#pragma unroll
        for (int r = 0; r < 16; ++r) h[r] = (R0 + 32 + 8 * (r >> 2) + 4 * hi + (r & 3) < re) ? hn[r] : 0.f;
    }
    const size_t pidx = blockIdx.x;
    float *o2 = part_w2 + pidx * hd * c;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = col0 + 8 * (r >> 2) + 4 * hi + (r & 3);
        if (lo < c) o2[(size_t)m * c + lo] = acc2[r];
    }
    float *o1 = part_w1 + pidx * fi * hd;
#pragma unroll
    for (int i = 0; i < FI32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = 32 * i + 8 * (r >> 2) + 4 * hi + (r & 3);
            o1[(size_t)m * hd + col0 + lo] = acc1[i][r];
        }
    const float t = cs + __shfl_xor(cs, 32);
    if (hi == 0) part_b1[pidx * hd + col0 + lo] = t;
}

inline bool hidden_backward_on_mfma(int32_t hd, int32_t c) { return (hd == 64 || hd == 128 || hd == 256) && c >= 1 && c <= 16; }

constexpr int kHiddenRowsPerWg = 1024;

template <int EPI>
void run_nn(int64_t N, int k, int n, const float *A, const float *W, float *C, const float *aux, hipStream_t st)
{
    if (k <= 16 && n <= 4 * kWG) {
        const int rows_per_wg = 512;                    // amortises the per-thread load of its W slice
        hipLaunchKernelGGL((k_gemm_nn_smallk<16, EPI>), dim3((unsigned)((N + rows_per_wg - 1) / rows_per_wg)),
                           dim3(kWG), 0, st, A, W, C, N, k, n, aux, rows_per_wg);
        return;
    }
    if (n > 64) {
        dim3 grid((unsigned)((N + 127) / 128), (n + 255) / 256);
        hipLaunchKernelGGL((k_gemm_nn<2, 2, 2, 4, EPI, 16>), grid, dim3(kWG), 0, st, A, W, C, N, k, n, aux);
    } else if (n > 32) {
        // 128 x 64 tile: a wave owns 32 rows across the whole width (bandwidth-bound shape)
        dim3 grid((unsigned)((N + 127) / 128), 1);
        hipLaunchKernelGGL((k_gemm_nn<4, 1, 1, 2, EPI, 32>), grid, dim3(kWG), 0, st, A, W, C, N, k, n, aux);
    } else {
        dim3 grid((unsigned)((N + 127) / 128), 1);
        hipLaunchKernelGGL((k_gemm_nn<4, 1, 1, 1, EPI, 64>), grid, dim3(kWG), 0, st, A, W, C, N, k, n, aux);
    }
}

}  // namespace

size_t gemm_tn_scratch_floats(int32_t m, int32_t n)
{
    const size_t chunks = (size_t)tn_max_chunks(m, n);
    const size_t stage2 = chunks > (size_t)kMaxChunks ? (chunks + kSumGroup - 1) / kSumGroup : 0;
    return (chunks + stage2) * ((size_t)m + 1) * n;
}

// C[m x n] = A^T B, A [K x m], B [K x n]; scratch holds gemm_tn_scratch_floats(m, n) floats.
// colsum (optional, n floats) receives the column sums of B.
int launch_gemm_tn(int64_t K, int32_t m, int32_t n, const float *A, const float *B, float *C,
                   float *colsum, float *scratch, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (m <= 0 || n <= 0) return AG_OK;
    if (K <= 0) {
        if (colsum) { int rc = launch_fill_zero(n, colsum, stream); if (rc) return rc; }
        return launch_fill_zero((int64_t)m * n, C, stream);
    }
    const int max_chunks = tn_max_chunks(m, n);
    float *cs_part = colsum ? scratch + (size_t)max_chunks * m * n : nullptr;
    const int kKS = kKSdef;
    int64_t steps = (K + kKS - 1) / kKS;
    int nchunks = (int)std::max<int64_t>(1, std::min<int64_t>(max_chunks, steps));
    int64_t rows_per_chunk = ((steps + nchunks - 1) / nchunks) * kKS;
    nchunks = (int)std::max<int64_t>(1, (K + rows_per_chunk - 1) / rows_per_chunk);
    if (tn_small_tile(m, n)) {
        // both widths small: a 64 x 64 tile, one 32 x 32 piece per wave
        dim3 grid(nchunks, (m + 63) / 64, 1);
        hipLaunchKernelGGL((k_gemm_tn<2, 2, 1, 1, kKSdef>), grid, dim3(kWG), 0, st, A, B, scratch, K, m, n, rows_per_chunk, cs_part);
    } else if (n > 32) {
        // wide outputs: operands straight from global memory, no LDS (0.69 ms against 0.76 ms for the
        // LDS-staged tile on the 1 M x 128 x 256 weight gradient; 8 k-steps of loads in flight beat 4 and 16)
        dim3 grid(nchunks, (m + 127) / 128, (n + 255) / 256);
        hipLaunchKernelGGL((k_gemm_tn_direct<2, 4, 8>), grid, dim3(kWG), 0, st, A, B, scratch, K, m, n, rows_per_chunk, cs_part);
    } else {
        dim3 grid(nchunks, (m + 255) / 256, 1);
        hipLaunchKernelGGL((k_gemm_tn<4, 1, 2, 1, kKSdef>), grid, dim3(kWG), 0, st, A, B, scratch, K, m, n, rows_per_chunk, cs_part);
    }
    const int64_t count = (int64_t)m * n;
    float *stage2 = max_chunks > kMaxChunks ? scratch + (size_t)max_chunks * ((size_t)m + 1) * n : nullptr;
    sum_partials(nchunks, count, scratch, C, stage2, st);
    if (colsum) sum_partials(nchunks, (int64_t)n, cs_part, colsum, stage2 ? stage2 + (size_t)((max_chunks + kSumGroup - 1) / kSumGroup) * count : nullptr, st);
    return hip_fail((int)hipGetLastError(), "gemm_tn launch");
}

// C[N x n] = A[N x k] W[k x n]; epilogue 0: none, 1: relu(. + aux[n]), 2: masked by aux[N x n] > 0
int launch_gemm_nn(int64_t N, int32_t k, int32_t n, const float *A, const float *W, float *C, int epilogue,
                   const float *aux, void *stream)
{
    if (N <= 0 || n <= 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    if (epilogue == EPI_BIAS_RELU) run_nn<EPI_BIAS_RELU>(N, k, n, A, W, C, aux, st);
    else if (epilogue == EPI_RELU_MASK) run_nn<EPI_RELU_MASK>(N, k, n, A, W, C, aux, st);
    else run_nn<EPI_NONE>(N, k, n, A, W, C, aux, st);
    return hip_fail((int)hipGetLastError(), "gemm_nn launch");
}

// Fused dPre = (dQ W2T) * (H1 > 0) and dW2 = H1^T dQ for c <= 16 classes and hd % 4 == 0 (<= 1024);
// returns AG_ERR_UNSUPPORTED for other shapes (the caller then uses the separate kernels).
size_t hidden_backward_scratch_floats(int64_t N, int32_t hd, int32_t c)
{
    if (hd < 4 || hd % 4 || hd / 4 > kWG || c > 16) return 0;
    const int64_t wgs = (N + kHiddenRowsPerWg - 1) / kHiddenRowsPerWg;
    if (hidden_backward_on_mfma(hd, c)) return (size_t)wgs * (hd == 64 ? 2 : 1) * hd * c;
    return (size_t)wgs * hd * c;
}

int launch_hidden_backward(int64_t N, int32_t hd, int32_t c, const float *dQ, const float *W2T, const float *H1,
                           float *dPre, float *dW2, float *scratch, void *stream)
{
    if (hd < 4 || hd % 4 || hd / 4 > kWG || c > 16 || c < 1) return AG_ERR_UNSUPPORTED;
    if (N <= 0) return launch_fill_zero((int64_t)hd * c, dW2, stream);
    hipStream_t st = (hipStream_t)stream;
    const int wgs = (int)((N + kHiddenRowsPerWg - 1) / kHiddenRowsPerWg);
    if (hidden_backward_on_mfma(hd, c)) {
        const int parts = wgs * (hd == 64 ? 2 : 1);
        hipLaunchKernelGGL(k_hidden_backward_mfma, dim3(wgs, hd == 256 ? 2 : 1), dim3(kWG), 0, st, dQ, W2T, H1, dPre, scratch, N, c, hd,
                           kHiddenRowsPerWg);
        const int64_t cnt = (int64_t)hd * c;
        hipLaunchKernelGGL(k_sum_partials, dim3((unsigned)((cnt + 31) / 32)), dim3(kWG), 0, st, parts, parts, cnt,
                           scratch, dW2);
        return hip_fail((int)hipGetLastError(), "hidden_backward launch");
    }
    if ((size_t)(kWG / (hd / 4) - 1) * hd * 16 * sizeof(float) > 65536) return AG_ERR_UNSUPPORTED;   // LDS for the in-group sum
    const int groups = kWG / (hd / 4);
    const size_t lds = (size_t)(groups - 1) * hd * 16 * sizeof(float);
    hipLaunchKernelGGL((k_hidden_backward<16>), dim3(wgs), dim3(kWG), lds, st, dQ, W2T, H1, dPre, scratch, N, c, hd,
                       kHiddenRowsPerWg);
    const int64_t count = (int64_t)hd * c;
    hipLaunchKernelGGL(k_sum_partials, dim3((unsigned)((count + 31) / 32)), dim3(kWG), 0, st, wgs, wgs, count,
                       scratch, dW2);
    return hip_fail((int)hipGetLastError(), "hidden_backward launch");
}

// Fused backward through both transforms of a two-layer GCN: dW2 = H1^T dQ, dW1 = P^T dPre and
// db1 = column sums of dPre with dPre = (dQ W2T) * (H1 > 0) kept in registers.  Shapes served:
// hidden width 64, 128 or 256, at most 16 classes, f_in in {32, 64, 96, 128}; AG_ERR_UNSUPPORTED
// otherwise (the caller then runs the separate kernels).
constexpr int kFusedRowsPerWg = 4096;

inline bool gcn_backward_fused_ok(int32_t fi, int32_t hd, int32_t c)
{
    return hidden_backward_on_mfma(hd, c) && fi >= 32 && fi <= 128 && fi % 32 == 0;
}

size_t gcn_backward_fused_scratch_floats(int64_t N, int32_t fi, int32_t hd, int32_t c)
{
    if (!gcn_backward_fused_ok(fi, hd, c)) return 0;
    const size_t parts = (size_t)((N + kFusedRowsPerWg - 1) / kFusedRowsPerWg) * (hd == 64 ? 2 : 1);
    const size_t stage2 = parts > (size_t)kMaxChunks ? (parts + kSumGroup - 1) / kSumGroup : 0;
    return parts * ((size_t)fi * hd + (size_t)hd * c + hd) + stage2 * (size_t)fi * hd + 64;
}

int launch_gcn_backward_fused(int64_t N, int32_t fi, int32_t hd, int32_t c, const float *dQ, const float *W2T,
                              const float *H1, const float *P, float *dW1, float *db1, float *dW2, float *scratch,
                              void *stream)
{
    if (!gcn_backward_fused_ok(fi, hd, c)) return AG_ERR_UNSUPPORTED;
    if (N <= 0) return AG_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const int wgs = (int)((N + kFusedRowsPerWg - 1) / kFusedRowsPerWg);
    const int parts = wgs * (hd == 64 ? 2 : 1);
    float *p1 = scratch, *p2 = p1 + (size_t)parts * fi * hd, *pb = p2 + (size_t)parts * hd * c;
    float *stage2 = parts > kMaxChunks ? pb + (size_t)parts * hd : nullptr;
    const dim3 grid(wgs, hd == 256 ? 2 : 1);
    if (fi == 128 && (hd == 128 || hd == 256)) {
        // all hidden columns in one work-group: the P block goes through LDS, cut once
        if (hd == 256)
            hipLaunchKernelGGL((k_gcn_backward_lds<4, 8>), dim3(wgs), dim3(512), 0, st, dQ, W2T, H1, P, p1, p2, pb, N, c, kFusedRowsPerWg);
        else
            hipLaunchKernelGGL((k_gcn_backward_lds<4, 4>), dim3(wgs), dim3(256), 0, st, dQ, W2T, H1, P, p1, p2, pb, N, c, kFusedRowsPerWg);
        sum_partials(parts, (int64_t)fi * hd, p1, dW1, stage2, st);
        sum_partials(parts, (int64_t)hd * c, p2, dW2, stage2, st);
        sum_partials(parts, (int64_t)hd, pb, db1, stage2, st);
        return hip_fail((int)hipGetLastError(), "gcn_backward_lds launch");
    }
#define AG_FUSED(t) hipLaunchKernelGGL((k_gcn_backward_fused<t, true>), grid, dim3(kWG), 0, st, dQ, W2T, H1, P, p1, p2, pb, N, c, hd, kFusedRowsPerWg)
    switch (fi / 32) {
    case 1: AG_FUSED(1); break;
    case 2: AG_FUSED(2); break;
    case 3: AG_FUSED(3); break;
    default: AG_FUSED(4); break;
    }
#undef AG_FUSED
    sum_partials(parts, (int64_t)fi * hd, p1, dW1, stage2, st);
    sum_partials(parts, (int64_t)hd * c, p2, dW2, stage2, st);
    sum_partials(parts, (int64_t)hd, pb, db1, stage2, st);
    return hip_fail((int)hipGetLastError(), "gcn_backward_fused launch");
}

int launch_transpose_small(int32_t rows, int32_t cols, const float *in, float *out, void *stream)
{
    if (rows <= 0 || cols <= 0) return AG_OK;
    hipLaunchKernelGGL(k_transpose_small, dim3((rows * cols + kWG - 1) / kWG), dim3(kWG), 0, (hipStream_t)stream,
                       rows, cols, in, out);
    return hip_fail((int)hipGetLastError(), "transpose launch");
}

}  // namespace ag
