// CSR-based kernel for low, irregular density (paper Sec. 3.2 "CSR-based kernel", the
// inter-community case): rows are mapped to lane teams, every lane walks source neighbours
// and gathers their feature rows straight from global memory.  Differences from the paper's
// CUDA mapping: the topology of a row is fetched once by the team and passed between lanes
// with wave shuffles instead of through shared memory; one row is served by a group of lanes
// that covers the feature width with 16-byte loads (one or several groups per row); rows
// above a degree threshold are cut into segments, one wavefront each, whose partial sums are
// combined by a second kernel in a fixed order (no atomics, bitwise reproducible).
#include "kernels_common.h"

namespace ag {
namespace {

template <int G, int W, int NV, int VEC>
__global__ __launch_bounds__(kWG) void k_csr_rows(CsrDev A, const float *__restrict__ H,
                                                  float *__restrict__ Y, int F, int row_begin,
                                                  int row_end, int acc_below)
{
    constexpr int TEAMS = kWG / W, FT = G * VEC * NV;
    const int tid = threadIdx.x;
    const int team = tid / W, tl = tid % W, gl = tl % G;
    const int wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int row = row_begin + wg * TEAMS + team;
    if (row >= row_end) return;                       // the whole team leaves together
    const int beg = A.rowptr[row], end = A.rowptr[row + 1];
    if (end - beg > kLongThresh) return;              // served by the segment kernels
    if (beg == end && row < acc_below) return;        // nothing to add to a row that is already written
    const int f = blockIdx.y * FT + gl * VEC;
    bool fok[NV];
    float acc[NV][VEC];
#pragma unroll
    for (int q = 0; q < NV; ++q) {
        fok[q] = f + q * G * VEC < F;
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[q][j] = 0.f;
    }
    team_row_gather<G, W, NV, VEC>(A.col, A.val, beg, end, H, F, f, fok, tl, acc);
    team_reduce<G, W, NV, VEC>(acc);
    if (tl < G) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            if (!fok[q]) continue;
            float *y = Y + (size_t)row * F + f + q * G * VEC;
            if (row < acc_below) {
                float old[VEC];
                load_vec<VEC>(y, old);
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[q][j] += old[j];
            }
            // a row that is written here for the first time is final: non-temporal store
            // (2.5 % faster for the one-CSR compositions at configs[2] and configs[3])
            if (row < acc_below) store_vec<VEC>(y, acc[q]);
            else store_vec_nt<VEC>(y, acc[q]);
        }
    }
}

// one wavefront per segment of a long row; result goes to partial[segment][F]
template <int G, int VEC>
__global__ __launch_bounds__(kWG) void k_csr_segments(CsrDev A, const float *__restrict__ H,
                                                      float *__restrict__ partial, int F)
{
    constexpr int W = 64;
    const int tid = threadIdx.x;
    // each XCD walks one contiguous part of the segment list: the long rows of one community,
    // which share most of their sources, meet in one L2
    const int seg = xcd_contiguous(blockIdx.x, gridDim.x) * (kWG / W) + tid / W;
    if (seg >= A.nseg) return;
    const int tl = tid % W, gl = tl % G;
    const int f = blockIdx.y * (G * VEC) + gl * VEC;
    const bool fok[1] = {f < F};
    float acc[1][VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[0][j] = 0.f;
    team_row_gather<G, W, 1, VEC>(A.col, A.val, A.seg_beg[seg], A.seg_end[seg], H, F, f, fok, tl, acc);
    team_reduce<G, W, 1, VEC>(acc);
    if (tl < G && fok[0]) store_vec<VEC>(partial + (size_t)seg * F + f, acc[0]);
}

// one lane group per long row: Y[row] (+)= sum of its segments' partials, in segment order
template <int G, int VEC>
__global__ __launch_bounds__(kWG) void k_csr_segment_sum(CsrDev A, const float *__restrict__ partial,
                                                         float *__restrict__ Y, int F, int acc_below)
{
    const int tid = threadIdx.x;
    const int lr = blockIdx.x * (kWG / G) + tid / G;
    if (lr >= A.nlr) return;
    const int f = blockIdx.y * (G * VEC) + (tid % G) * VEC;
    if (f >= F) return;
    const int row = A.lr_row[lr];
    float acc[VEC];
    float *y = Y + (size_t)row * F + f;
    if (row < acc_below) {
        load_vec<VEC>(y, acc);
    } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
    }
    for (int s = A.lr_seg0[lr]; s < A.lr_seg0[lr + 1]; ++s) {
        float p[VEC];
        load_vec<VEC>(partial + (size_t)s * F + f, p);
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] += p[j];
    }
    store_vec<VEC>(y, acc);
}

struct Shape { int G, W, NV, VEC; };

// Lane layout for a feature width.  variant AG_K_CSR_WIDE: four lane groups per row; anything
// else (narrow): one lane group per row.  (Two vectors per lane, NV = 2, was measured and never
// beat NV = 1 for these kernels, so only NV = 1 is instantiated.)
Shape pick_shape(int F, int variant)
{
    Shape s;
    s.VEC = vec_width(F);
    s.NV = 1;
    const int need = (F + s.VEC - 1) / s.VEC, cap = (s.VEC == 4) ? 32 : 64;
    s.G = 4;
    while (s.G < need && s.G < cap) s.G <<= 1;
    s.W = s.G;
    if (variant == 1 && s.VEC == 4) s.W = (s.G >= 16) ? 64 : s.G * 4;
    return s;
}

template <int G, int W, int NV, int VEC>
void run_rows(const CsrDev &A, const float *H, float *Y, int F, int rb, int re, int acc_below,
              hipStream_t st)
{
    const int rows = re - rb, teams = kWG / W;
    dim3 grid((rows + teams - 1) / teams, (F + G * VEC * NV - 1) / (G * VEC * NV));
    hipLaunchKernelGGL((k_csr_rows<G, W, NV, VEC>), grid, dim3(kWG), 0, st, A, H, Y, F, rb, re, acc_below);
}

template <int G, int VEC>
void run_long(const CsrDev &A, const float *H, float *Y, int F, float *partial, int acc_below,
              hipStream_t st)
{
    const int ty = (F + G * VEC - 1) / (G * VEC);
    hipLaunchKernelGGL((k_csr_segments<G, VEC>), dim3((A.nseg + 3) / 4, ty), dim3(kWG), 0, st, A, H,
                       partial, F);
    const int teams = kWG / G;
    hipLaunchKernelGGL((k_csr_segment_sum<G, VEC>), dim3((A.nlr + teams - 1) / teams, ty), dim3(kWG),
                       0, st, A, partial, Y, F, acc_below);
}

}  // namespace

int launch_csr_rows(const CsrDev &A, const float *H, float *Y, int32_t F, int32_t row_begin,
                    int32_t row_end, int32_t acc_below, int variant, void *stream)
{
    if (row_end <= row_begin) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    const Shape s = pick_shape(F, variant);
#define AG_CASE(g, w, nv, v) \
    if (s.G == g && s.W == w && s.NV == nv && s.VEC == v) { run_rows<g, w, nv, v>(A, H, Y, F, row_begin, row_end, acc_below, st); return hip_fail((int)hipGetLastError(), "csr_rows launch"); }
    AG_CASE(4, 4, 1, 4) AG_CASE(4, 16, 1, 4) AG_CASE(8, 8, 1, 4) AG_CASE(8, 32, 1, 4)
    AG_CASE(16, 16, 1, 4) AG_CASE(16, 64, 1, 4) AG_CASE(32, 32, 1, 4) AG_CASE(32, 64, 1, 4)
    AG_CASE(4, 4, 1, 2) AG_CASE(8, 8, 1, 2) AG_CASE(16, 16, 1, 2) AG_CASE(32, 32, 1, 2) AG_CASE(64, 64, 1, 2)
    AG_CASE(4, 4, 1, 1) AG_CASE(8, 8, 1, 1) AG_CASE(16, 16, 1, 1) AG_CASE(32, 32, 1, 1) AG_CASE(64, 64, 1, 1)
#undef AG_CASE
    set_error("csr_rows: no kernel shape for this feature width");
    return AG_ERR_UNSUPPORTED;
}

int launch_csr_long(const CsrDev &A, const float *H, float *Y, int32_t F, float *partial,
                    int32_t acc_below, void *stream)
{
    if (A.nseg == 0) return AG_OK;
    hipStream_t st = (hipStream_t)stream;
    const Shape s = pick_shape(F, 0);
#define AG_CASE(g, v) \
    if (s.G == g && s.VEC == v) { run_long<g, v>(A, H, Y, F, partial, acc_below, st); return hip_fail((int)hipGetLastError(), "csr_long launch"); }
    AG_CASE(4, 4) AG_CASE(8, 4) AG_CASE(16, 4) AG_CASE(32, 4)
    AG_CASE(4, 2) AG_CASE(8, 2) AG_CASE(16, 2) AG_CASE(32, 2) AG_CASE(64, 2)
    AG_CASE(4, 1) AG_CASE(8, 1) AG_CASE(16, 1) AG_CASE(32, 1) AG_CASE(64, 1)
#undef AG_CASE
    set_error("csr_long: no kernel shape for this feature width");
    return AG_ERR_UNSUPPORTED;
}

}  // namespace ag
