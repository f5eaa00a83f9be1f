// Small element-wise / reduction kernels around the aggregation: row permutation between the
// caller's vertex order and the plan order, and the dense-layer glue of the GCN / GIN steps
// (paper Sec. 2.1 "Update", Sec. 5 "Benchmarks").  All bandwidth-bound, one pass each.
#include "kernels_common.h"

namespace ag {
namespace {

constexpr int kSumChunks = 1024;   // partial rows produced by the first stage of col_sum

// dst[r] = src[perm[r]]  (inverse: dst[perm[r]] = src[r]); one float4 (or float) per thread
template <int VEC>
__global__ __launch_bounds__(kWG) void k_permute(const int32_t *__restrict__ perm, int64_t n, int F,
                                                 const float *__restrict__ src, float *__restrict__ dst,
                                                 int inverse)
{
    const int per_row = F / VEC;
    const int64_t idx = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (idx >= n * per_row) return;
    const int64_t r = idx / per_row;
    const int c = (int)(idx % per_row) * VEC;
    const int64_t p = perm[r];
    float h[VEC];
    if (inverse) {
        load_vec<VEC>(src + r * F + c, h);
        store_vec<VEC>(dst + p * F + c, h);
    } else {
        load_vec<VEC>(src + p * F + c, h);
        store_vec<VEC>(dst + r * F + c, h);
    }
}

__global__ __launch_bounds__(kWG) void k_axpy(int64_t count, float a, const float *__restrict__ x,
                                              float *__restrict__ y)
{
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i < count) y[i] = fmaf(a, x[i], y[i]);
}

__global__ __launch_bounds__(kWG) void k_fill_zero(int64_t count, float *__restrict__ p)
{
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// One thread per vertex: z = Zin + bias; row loss = logsumexp(z) - z[label] (max-subtracted);
// dZ = (softmax(z) - onehot) / n.  Zout (optional) receives z.  CMAX > 0: the row (c <= CMAX,
// c % 4 == 0) is held in registers and moved with 16-byte loads and stores.
template <int CMAX>
__global__ __launch_bounds__(kWG) void k_softmax_xent(int64_t n, int c, const float *__restrict__ Zin,
                                                      const float *__restrict__ bias,
                                                      const int32_t *__restrict__ labels,
                                                      float *__restrict__ Zout, float *__restrict__ dZ,
                                                      float *__restrict__ rowloss)
{
    const int64_t r = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (r >= n) return;
    const int y = labels[r];
    const float invn = 1.f / (float)n;
    if constexpr (CMAX > 0) {
        float z[CMAX];
#pragma unroll
        for (int j = 0; j < CMAX; j += 4) {
            if (j < c) {
                const float4 t = *reinterpret_cast<const float4 *>(Zin + r * c + j);
                const float4 bb = *reinterpret_cast<const float4 *>(bias + j);
                z[j] = t.x + bb.x; z[j + 1] = t.y + bb.y; z[j + 2] = t.z + bb.z; z[j + 3] = t.w + bb.w;
            }
        }
        float m = -INFINITY, zy = 0.f;
#pragma unroll
        for (int j = 0; j < CMAX; ++j)
            if (j < c) { m = fmaxf(m, z[j]); zy = (j == y) ? z[j] : zy; }
        float s = 0.f, e[CMAX];
#pragma unroll
        for (int j = 0; j < CMAX; ++j)
            if (j < c) { e[j] = expf(z[j] - m); s += e[j]; }
        const float inv = 1.f / s;
#pragma unroll
        for (int j = 0; j < CMAX; j += 4) {
            if (j < c) {
                float4 d;
                d.x = (e[j] * inv - (j == y ? 1.f : 0.f)) * invn;
                d.y = (e[j + 1] * inv - (j + 1 == y ? 1.f : 0.f)) * invn;
                d.z = (e[j + 2] * inv - (j + 2 == y ? 1.f : 0.f)) * invn;
                d.w = (e[j + 3] * inv - (j + 3 == y ? 1.f : 0.f)) * invn;
                *reinterpret_cast<float4 *>(dZ + r * c + j) = d;
                if (Zout) *reinterpret_cast<float4 *>(Zout + r * c + j) = make_float4(z[j], z[j + 1], z[j + 2], z[j + 3]);
            }
        }
        rowloss[r] = (logf(s) + m - zy) * invn;
    } else {
        const float *z = Zin + r * c;
        float m = -INFINITY;
        for (int j = 0; j < c; ++j) m = fmaxf(m, z[j] + bias[j]);
        float s = 0.f;
        for (int j = 0; j < c; ++j) s += expf(z[j] + bias[j] - m);
        const float inv = 1.f / s;
        for (int j = 0; j < c; ++j) {
            const float zj = z[j] + bias[j];
            const float p = expf(zj - m) * inv;
            dZ[r * c + j] = (p - (j == y ? 1.f : 0.f)) * invn;
            if (Zout) Zout[r * c + j] = zj;
        }
        const float zy = (y >= 0 && y < c) ? z[y] + bias[y] : 0.f;      // a label outside [0,c) reads nothing
        rowloss[r] = (logf(s) + m - zy) * invn;
    }
}

// stage 1: chunk q sums rows [q*rows_per, ...) column-wise into part[q][f]
__global__ __launch_bounds__(kWG) void k_col_sum_stage1(int64_t n, int f, int64_t rows_per,
                                                        const float *__restrict__ M,
                                                        float *__restrict__ part)
{
    __shared__ float red[kWG];
    const int q = blockIdx.x;
    const int64_t rb = q * rows_per, re = min(n, rb + rows_per);
    // thread t owns column t % fw of every (kWG / fw)-th row, fw = columns handled per pass
    for (int c0 = 0; c0 < f; c0 += kWG) {
        const int fw = min(f - c0, kWG);
        const int lanes_per_col = kWG / fw;            // >= 1
        const int col = threadIdx.x % fw, sub = threadIdx.x / fw;
        float acc = 0.f;
        if (sub < lanes_per_col)
            for (int64_t r = rb + sub; r < re; r += lanes_per_col) acc += M[r * f + c0 + col];
        red[threadIdx.x] = (sub < lanes_per_col) ? acc : 0.f;
        __syncthreads();
        if (threadIdx.x < fw) {
            float s = 0.f;
            for (int k = 0; k < lanes_per_col; ++k) s += red[k * fw + threadIdx.x];
            part[(size_t)q * f + c0 + threadIdx.x] = s;
        }
        __syncthreads();
    }
}

// stage 2: out[c] = sum_q part[q][c]; 32 columns per work-group, 8 slices of the partial rows
// per column, combined through LDS in a fixed order
__global__ __launch_bounds__(kWG) void k_col_sum_stage2(int nq, int f, const float *__restrict__ part,
                                                        float *__restrict__ out)
{
    __shared__ float red[kWG];
    const int c = blockIdx.x * 32 + (threadIdx.x & 31), slice = threadIdx.x >> 5;
    const float s = (c < f) ? sum_strided(part + c, (size_t)f, slice, nq, 8) : 0.f;
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x < 32 && c < f) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += red[k * 32 + threadIdx.x];
        out[c] = t;
    }
}

inline dim3 grid1(int64_t count) { return dim3((unsigned)((count + kWG - 1) / kWG)); }

}  // namespace

int launch_permute_rows(const int32_t *perm, int64_t n, int32_t F, const float *src, float *dst,
                        bool inverse, void *stream)
{
    if (n == 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    if (F % 4 == 0)
        hipLaunchKernelGGL((k_permute<4>), grid1(n * (F / 4)), dim3(kWG), 0, st, perm, n, F, src, dst, inverse ? 1 : 0);
    else if (F % 2 == 0)
        hipLaunchKernelGGL((k_permute<2>), grid1(n * (F / 2)), dim3(kWG), 0, st, perm, n, F, src, dst, inverse ? 1 : 0);
    else
        hipLaunchKernelGGL((k_permute<1>), grid1(n * F), dim3(kWG), 0, st, perm, n, F, src, dst, inverse ? 1 : 0);
    return hip_fail((int)hipGetLastError(), "permute launch");
}

int launch_axpy(int64_t count, float a, const float *x, float *y, void *stream)
{
    if (count == 0) return AG_OK;
    hipLaunchKernelGGL(k_axpy, grid1(count), dim3(kWG), 0, (hipStream_t)stream, count, a, x, y);
    return hip_fail((int)hipGetLastError(), "axpy launch");
}

int launch_fill_zero(int64_t count, float *p, void *stream)
{
    if (count == 0) return AG_OK;
    hipLaunchKernelGGL(k_fill_zero, grid1(count), dim3(kWG), 0, (hipStream_t)stream, count, p);
    return hip_fail((int)hipGetLastError(), "fill launch");
}

int launch_softmax_xent(int64_t n, int32_t c, const float *Zin, const float *bias,
                        const int32_t *labels, float *Zout, float *dZ, float *rowloss, void *stream)
{
    if (n == 0) return AG_OK;
    if (c % 4 == 0 && c <= 16)
        hipLaunchKernelGGL((k_softmax_xent<16>), grid1(n), dim3(kWG), 0, (hipStream_t)stream, n, c, Zin, bias,
                           labels, Zout, dZ, rowloss);
    else if (c % 4 == 0 && c <= 64)
        hipLaunchKernelGGL((k_softmax_xent<64>), grid1(n), dim3(kWG), 0, (hipStream_t)stream, n, c, Zin, bias,
                           labels, Zout, dZ, rowloss);
    else
        hipLaunchKernelGGL((k_softmax_xent<0>), grid1(n), dim3(kWG), 0, (hipStream_t)stream, n, c, Zin, bias,
                           labels, Zout, dZ, rowloss);
    return hip_fail((int)hipGetLastError(), "softmax_xent launch");
}

size_t col_sum_scratch_floats(int32_t f) { return (size_t)kSumChunks * f; }

int launch_col_sum(int64_t n, int32_t f, const float *M, float *out, float *scratch, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    int nq = (int)std::min<int64_t>(kSumChunks, std::max<int64_t>(1, (n + 255) / 256));
    const int64_t rows_per = (n + nq - 1) / nq;
    nq = (int)((n + rows_per - 1) / std::max<int64_t>(1, rows_per));
    if (n == 0) { nq = 0; }
    if (nq > 0)
        hipLaunchKernelGGL(k_col_sum_stage1, dim3(nq), dim3(kWG), 0, st, n, f, rows_per, M, scratch);
    hipLaunchKernelGGL(k_col_sum_stage2, dim3((f + 31) / 32), dim3(kWG), 0, st, nq, f, scratch, out);
    return hip_fail((int)hipGetLastError(), "col_sum launch");
}

}  // namespace ag
