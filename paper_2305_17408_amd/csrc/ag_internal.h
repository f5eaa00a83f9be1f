// Internal declarations shared by the translation units of libadaptgear.
#pragma once
#include <cstdint>
#include <exception>
#include <memory>
#include <string>
#include <algorithm>
#include <thread>
#include <vector>

#include "adaptgear.h"

namespace ag {

constexpr int kMaxBlock   = 128;   // rows of a diagonal block the dense kernels take; unit of the LDS tiles
constexpr int kMaxBlockWide = 256; // largest diagonal block (one-byte block-local columns), block-sparse kernel only
constexpr int kLongThresh = 96;    // remainder rows above this many entries are split ...
constexpr int kSegLen     = 384;   // ... into segments of this many entries, one wavefront each

// ----------------------------------------------------------------------------------------
// host-side matrices
// ----------------------------------------------------------------------------------------
struct HostCsr {
    int64_t n = 0;
    std::vector<int32_t> rowptr;   // n + 1
    std::vector<int32_t> col;
    std::vector<float>   val;      // empty when unit weights
    int64_t nnz() const { return rowptr.empty() ? 0 : rowptr.back(); }
};

// Integer-weighted undirected graph used by the multilevel reordering.
struct WGraph {
    int32_t n = 0;
    std::vector<int64_t> xadj;
    std::vector<int32_t> adj, ew, nw;
};

struct ReorderResult {
    std::vector<int32_t> perm, iperm, blk_ptr, comm;
    int32_t n_blocks = 0;
};

// run fn(t, begin, end) over [0,n) on a few host threads (t = thread index); returns the thread
// count.  An exception thrown by fn on a worker (an allocation failure, say) is re-thrown on the caller.
template <class Fn>
int parallel_ranges(int64_t n, Fn fn, int64_t min_per_thread = 4096)
{
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<int64_t>(std::max(1u, std::min(hw, 16u)), std::max<int64_t>(1, n / min_per_thread));
    if (nt <= 1) { fn(0, (int64_t)0, n); return 1; }
    std::vector<std::thread> th;
    std::vector<std::exception_ptr> err(nt);
    th.reserve(nt);
    std::exception_ptr spawn_err;
    for (int t = 0; t < nt; ++t) {
        try {
            th.emplace_back([=, &err] {
                try { fn(t, n * t / nt, n * (t + 1) / nt); } catch (...) { err[t] = std::current_exception(); }
            });
        } catch (...) {                                  // no more threads: finish this range here
            try { fn(t, n * t / nt, n * (t + 1) / nt); } catch (...) { spawn_err = std::current_exception(); }
        }
    }
    for (auto &x : th) x.join();
    if (spawn_err) std::rethrow_exception(spawn_err);
    for (auto &e : err) if (e) std::rethrow_exception(e);
    return nt;
}

// reorder.cpp
void build_pattern_graph(const HostCsr &A, const HostCsr &At, WGraph &g);
void community_reorder(const WGraph &g0, int32_t method, int32_t cap, int32_t min_block, int32_t sweeps,
                       int32_t max_levels, int32_t order_levels, ReorderResult &out);

// decompose.cpp
int  ingest_csr(const ag_csr *in, HostCsr &out, std::string &err);       // validate + sort rows
void transpose_csr(const HostCsr &A, HostCsr &At);
bool bitwise_equal(const HostCsr &A, const HostCsr &B);
void permute_and_split(const HostCsr &A, const ReorderResult &r, HostCsr &full, HostCsr &intra,
                       HostCsr &inter);

// One direction (forward = A, backward = A^T) of the decomposed matrix, in plan numbering.
struct HostDir {
    HostCsr full, intra, inter;
    // long-row segmentation of a CSR part: rows with more than kLongThresh entries
    struct Segs {
        std::vector<int32_t> seg_row, seg_beg, seg_end;   // one entry per segment
        std::vector<int32_t> lr_row, lr_seg0;             // per long row: row id, first segment (nlr+1)
    } segs_full, segs_inter;
    std::vector<uint8_t>  intra_col8;      // block-local column of every intra entry
    std::vector<uint32_t> bitmap;          // per dense-class block: 128 rows x 4 words
    std::vector<float>    tiles;           // per dense-class block: 4 x 64 x 64 floats (weighted only)
};

void build_segments(const HostCsr &A, HostDir::Segs &s);
void build_block_formats(const ReorderResult &r, const std::vector<int32_t> &dense_blocks,
                         bool unit, HostDir &d);

// ----------------------------------------------------------------------------------------
// device-side views (plain pointers, passed to kernels by value)
// ----------------------------------------------------------------------------------------
struct CsrDev {
    const int32_t *rowptr = nullptr, *col = nullptr;
    const float   *val = nullptr;          // nullptr = unit weights
    const int32_t *row = nullptr;          // row of every entry (COO form), only where the COO kernel may run
    int32_t n = 0, nnz = 0;
    const int32_t *seg_row = nullptr, *seg_beg = nullptr, *seg_end = nullptr;
    int32_t nseg = 0;
    const int32_t *lr_row = nullptr, *lr_seg0 = nullptr;
    int32_t nlr = 0;
};

struct BlocksDev {
    const int32_t *blk_ptr = nullptr;      // nb + 1
    int32_t nb = 0, n_block_rows = 0, max_block_rows = 0;
    const int32_t *i_rowptr = nullptr;     // n_block_rows + 1 (intra entries of block rows)
    const uint8_t *i_col8 = nullptr;
    const float   *i_val = nullptr;        // nullptr = unit weights
    const int32_t *list_dense = nullptr, *list_sparse = nullptr, *list_all = nullptr;
    int32_t n_dense = 0, n_sparse = 0;
    const uint32_t *bitmap = nullptr;      // n_dense x 128 x 4
    const float    *tiles = nullptr;       // n_dense x 16384, nullptr = unit weights
    // factored values: feature rows are multiplied by in_scale[row] when staged, a row's sum over its
    // block entries by out_scale[row] (plan numbering; nullptr = 1)
    const float *in_scale = nullptr, *out_scale = nullptr;
};

struct DevDir {
    CsrDev full, inter;
    BlocksDev blk;
};

// kernels_csr.hip
// Rows [row_begin,row_end) of `A`: rows below `acc_below` add to Y, the others overwrite it.
// `variant` is the remainder kernel id (AG_K_CSR_WIDE; anything else = narrow).
// Long rows are left to launch_csr_long.
int launch_csr_rows(const CsrDev &A, const float *H, float *Y, int32_t F, int32_t row_begin,
                    int32_t row_end, int32_t acc_below, int variant, void *stream);
// All long rows of `A`: segments -> partial[nseg][F] -> Y (rows below acc_below accumulate).
int launch_csr_long(const CsrDev &A, const float *H, float *Y, int32_t F, float *partial,
                    int32_t acc_below, void *stream);
// kernels_coo.hip
// Edge-parallel accumulation of all entries of `A` (needs A.row) onto Y with fp32 atomics; rows
// from zero_from on are cleared first (the rows nobody wrote before).
int launch_coo(const CsrDev &A, const float *H, float *Y, int32_t F, int32_t zero_from, void *stream);
// kernels_block.hip
int launch_block_sparse(const BlocksDev &B, const int32_t *list, int32_t nlist, const CsrDev *fused_rem,
                        const float *H, float *Y, int32_t F, void *stream);
// kernels_dense.hip
// fused_rem != null: the rows' remainder entries are added in the same kernel (one store per row)
int launch_block_dense(const BlocksDev &B, const CsrDev *fused_rem, const float *H, float *Y, int32_t F,
                       int variant, void *stream);
// kernels_max.hip
int launch_csr_max(const CsrDev &A, const float *H, float *Y, int32_t *arg, int32_t F, void *stream);
int launch_csr_max_t(const CsrDev &At, const float *G, const int32_t *arg, float *dH, int32_t F, void *stream);
// kernels_misc.hip
int launch_permute_rows(const int32_t *perm, int64_t n, int32_t F, const float *src, float *dst,
                        bool inverse, void *stream);
int launch_axpy(int64_t count, float a, const float *x, float *y, void *stream);
int launch_softmax_xent(int64_t n, int32_t c, const float *Zin, const float *bias,
                        const int32_t *labels, float *Zout, float *dZ, float *rowloss, void *stream);
size_t col_sum_scratch_floats(int32_t f);
int launch_col_sum(int64_t n, int32_t f, const float *M, float *out, float *scratch, void *stream);
int launch_fill_zero(int64_t count, float *p, void *stream);
// kernels_gemm.hip
size_t gemm_tn_scratch_floats(int32_t m, int32_t n);
int launch_gemm_tn(int64_t K, int32_t m, int32_t n, const float *A, const float *B, float *C,
                   float *colsum, float *scratch, void *stream);
int launch_gemm_nn(int64_t N, int32_t k, int32_t n, const float *A, const float *W, float *C, int epilogue,
                   const float *aux, void *stream);
// kernels_gemm_b3.hip
size_t gemm_nn_b3_scratch_floats(int32_t k, int32_t n);
int launch_gemm_nn_b3(int64_t N, int32_t k, int32_t n, const float *A, const float *W, float *C, int epilogue,
                      const float *aux, float *wsplit, void *stream);
int launch_gemm_chain_b3(int64_t N, int32_t k, int32_t n, int32_t c, const float *A, const float *W, const float *bias,
                         const float *W2, float *H, float *Q, float *wsplit, void *stream);
int launch_gemm_nn_auto(int64_t N, int32_t k, int32_t n, const float *A, const float *W, float *C, int epilogue,
                        const float *aux, float *wsplit, void *stream);
size_t hidden_backward_scratch_floats(int64_t N, int32_t hd, int32_t c);
int launch_hidden_backward(int64_t N, int32_t hd, int32_t c, const float *dQ, const float *W2T, const float *H1,
                           float *dPre, float *dW2, float *scratch, void *stream);
size_t gcn_backward_fused_scratch_floats(int64_t N, int32_t fi, int32_t hd, int32_t c);
int launch_gcn_backward_fused(int64_t N, int32_t fi, int32_t hd, int32_t c, const float *dQ, const float *W2T,
                              const float *H1, const float *P, float *dW1, float *db1, float *dW2, float *scratch,
                              void *stream);
int launch_transpose_small(int32_t rows, int32_t cols, const float *in, float *out, void *stream);

// api.cpp
// ag_aggregate with the settled kernel choice and `partial` (partial_bytes of device memory) in
// place of the plan's own long-row scratch; allocates nothing, refuses calls that need a trial.
int aggregate_settled(ag_plan *p, const float *X, float *Y, float *partial, size_t partial_bytes, void *stream);

void set_error(const std::string &msg);
int  hip_fail(int hip_error_code, const char *what);

}  // namespace ag
