// fp32 MFMA GEMMs for the dense Update part of the GCN step (paper Sec. 2.1 "Update", Sec. 5).
//
// gemm_tn:  C[m x n] = A^T B  with A [K x m], B [K x n] row-major and K = number of vertices
//           (the weight gradients dW = X^T dY).  K is split across work-groups; each writes a
//           partial m x n tile and a second kernel adds the partials in a fixed order.
//           Both MFMA operands are rows of A and B, so they are read coalesced and staged in LDS
//           without any transposition.
#include "kernels_common.h"

namespace ag {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kKS = 16;            // K rows staged per step
constexpr int kMaxChunks = 512;    // K-splits (partials) per output tile

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
template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ __launch_bounds__(kWG) void k_gemm_tn(const float *__restrict__ A, const float *__restrict__ B,
                                                 float *__restrict__ part, int64_t K, int m, int n,
                                                 int64_t rows_per_chunk)
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

    float4 ra[UA], rb[UB];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int idx = tid + u * kWG, r = idx / (TM / 4), c = (idx % (TM / 4)) * 4;
            if (idx < NA) ra[u] = guarded_load4(A, k0 + r, k_end, m0 + c, m, va);
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int idx = tid + u * kWG, r = idx / (TN / 4), c = (idx % (TN / 4)) * 4;
            if (idx < NB) rb[u] = guarded_load4(B, k0 + r, k_end, n0 + c, n, vb);
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

__global__ __launch_bounds__(kWG) void k_sum_partials(int nchunks, int64_t count,
                                                      const float *__restrict__ part, float *__restrict__ C)
{
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i >= count) return;
    float s = 0.f;
    for (int q = 0; q < nchunks; ++q) s += part[(size_t)q * count + i];
    C[i] = s;
}

}  // namespace

size_t gemm_tn_scratch_floats(int32_t m, int32_t n) { return (size_t)kMaxChunks * m * n; }

// C[m x n] = A^T B, A [K x m], B [K x n]; scratch holds gemm_tn_scratch_floats(m, n) floats.
int launch_gemm_tn(int64_t K, int32_t m, int32_t n, const float *A, const float *B, float *C,
                   float *scratch, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (m <= 0 || n <= 0) return AG_OK;
    if (K <= 0) return launch_fill_zero((int64_t)m * n, C, stream);
    int64_t steps = (K + kKS - 1) / kKS;
    int nchunks = (int)std::max<int64_t>(1, std::min<int64_t>(kMaxChunks, steps));
    int64_t rows_per_chunk = ((steps + nchunks - 1) / nchunks) * kKS;
    nchunks = (int)std::max<int64_t>(1, (K + rows_per_chunk - 1) / rows_per_chunk);
    if (n > 32) {
        dim3 grid(nchunks, (m + 127) / 128, (n + 255) / 256);
        hipLaunchKernelGGL((k_gemm_tn<2, 2, 2, 4>), grid, dim3(kWG), 0, st, A, B, scratch, K, m, n, rows_per_chunk);
    } else {
        dim3 grid(nchunks, (m + 255) / 256, 1);
        hipLaunchKernelGGL((k_gemm_tn<4, 1, 2, 1>), grid, dim3(kWG), 0, st, A, B, scratch, K, m, n, rows_per_chunk);
    }
    const int64_t count = (int64_t)m * n;
    hipLaunchKernelGGL(k_sum_partials, dim3((unsigned)((count + kWG - 1) / kWG)), dim3(kWG), 0, st, nchunks,
                       count, scratch, C);
    return hip_fail((int)hipGetLastError(), "gemm_tn launch");
}

}  // namespace ag
