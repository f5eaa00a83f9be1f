// Two-layer GCN training step (paper Sec. 5 "Benchmarks": GCN with its default two layers),
// forward + backward.  The three aggregations run through the plans' adaptive kernels; the
// dense Update GEMMs (Sec. 2.1) are plain library SGEMMs from rocBLAS, loaded on first use.
#include <dlfcn.h>
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>

#include <algorithm>
#include <mutex>

#include "ag_internal.h"

namespace ag {
int64_t plan_n(const ag_plan *p);
int32_t plan_f(const ag_plan *p);
int32_t plan_layout(const ag_plan *p);
bool plan_same_topology(const ag_plan *a, const ag_plan *b);
bool plan_host_only(const ag_plan *p);
}  // namespace ag

using namespace ag;

namespace {

struct Blas {
    void *lib = nullptr;
    rocblas_handle handle = nullptr;
    decltype(&rocblas_create_handle) create = nullptr;
    decltype(&rocblas_set_stream) set_stream = nullptr;
    decltype(&rocblas_sgemm) sgemm = nullptr;
    bool ok = false;
};

Blas &blas()
{
    static Blas b;
    static std::once_flag once;
    std::call_once(once, [] {
        b.lib = dlopen("librocblas.so", RTLD_NOW | RTLD_LOCAL);
        if (!b.lib) b.lib = dlopen("librocblas.so.5", RTLD_NOW | RTLD_LOCAL);
        if (!b.lib) return;
        b.create = (decltype(b.create))dlsym(b.lib, "rocblas_create_handle");
        b.set_stream = (decltype(b.set_stream))dlsym(b.lib, "rocblas_set_stream");
        b.sgemm = (decltype(b.sgemm))dlsym(b.lib, "rocblas_sgemm");
        if (!b.create || !b.set_stream || !b.sgemm) return;
        if (b.create(&b.handle) != rocblas_status_success) return;
        b.ok = true;
    });
    return b;
}

// row-major C[m x n] = op(A) op(B); A is m x k (or k x m when ta), B is k x n (or n x k when tb)
int gemm_rm(Blas &b, bool ta, bool tb, int64_t m, int64_t n, int64_t k, const float *A, const float *B,
            float *C)
{
    const float one = 1.f, zero = 0.f;
    // column-major view: C^T[n x m] = op(B)^T op(A)^T
    const rocblas_operation opB = tb ? rocblas_operation_transpose : rocblas_operation_none;
    const rocblas_operation opA = ta ? rocblas_operation_transpose : rocblas_operation_none;
    const int64_t ldb = tb ? k : n, lda = ta ? m : k;
    rocblas_status s = b.sgemm(b.handle, opB, opA, (rocblas_int)n, (rocblas_int)m, (rocblas_int)k, &one, B,
                               (rocblas_int)ldb, A, (rocblas_int)lda, &zero, C, (rocblas_int)n);
    if (s != rocblas_status_success) {
        set_error("rocblas_sgemm failed with status " + std::to_string((int)s));
        return AG_ERR_HIP;
    }
    return AG_OK;
}

struct Ws {
    float *P, *H1, *Q, *Z, *dZ, *dQ, *dH1, *rowloss, *scratch;
};

size_t ws_floats(int64_t n, int32_t fi, int32_t hd, int32_t c)
{
    return (size_t)n * ((size_t)fi + 2 * (size_t)hd + 4 * (size_t)c + 1) +
           std::max(col_sum_scratch_floats(std::max(hd, c)),
                    std::max(gemm_tn_scratch_floats(fi, hd), gemm_tn_scratch_floats(hd, c))) + 64;
}

}  // namespace

extern "C" {

size_t ag_gcn_workspace_bytes(int64_t n, int32_t f_in, int32_t hidden, int32_t n_class)
{
    if (n < 0 || f_in < 1 || hidden < 1 || n_class < 1) return 0;
    return ws_floats(n, f_in, hidden, n_class) * sizeof(float);
}

int ag_gcn_step(ag_plan *p_in, ag_plan *p_out, const ag_gcn_io *io, const float *X,
                const int32_t *labels, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!p_in || !p_out || !io || !X || !labels || !workspace) { set_error("null argument"); return AG_ERR_INVALID; }
    if (plan_host_only(p_in)) { set_error("host-only plan"); return AG_ERR_UNSUPPORTED; }
    const int64_t n = plan_n(p_in);
    const int32_t fi = io->f_in, hd = io->hidden, c = io->n_class;
    if (fi < 1 || hd < 1 || c < 1 || plan_f(p_in) != fi || plan_f(p_out) != c || !plan_same_topology(p_in, p_out)) {
        set_error("plans do not match the layer widths (need clones of one topology with F = f_in and F = n_class)");
        return AG_ERR_INVALID;
    }
    if (plan_layout(p_in) != AG_LAYOUT_REORDERED || plan_layout(p_out) != AG_LAYOUT_REORDERED) {
        set_error("ag_gcn_step needs AG_LAYOUT_REORDERED plans");
        return AG_ERR_UNSUPPORTED;
    }
    if (!io->W1 || !io->b1 || !io->W2 || !io->b2 || !io->dW1 || !io->db1 || !io->dW2 || !io->db2 || !io->loss) {
        set_error("null parameter or gradient pointer");
        return AG_ERR_INVALID;
    }
    if (workspace_bytes < ag_gcn_workspace_bytes(n, fi, hd, c)) { set_error("workspace too small"); return AG_ERR_INVALID; }
    Blas &b = blas();
    if (!b.ok) { set_error("rocBLAS could not be loaded"); return AG_ERR_UNSUPPORTED; }
    if (b.set_stream(b.handle, (hipStream_t)stream) != rocblas_status_success) {
        set_error("rocblas_set_stream failed");
        return AG_ERR_HIP;
    }
    Ws w;
    float *q = (float *)workspace;
    w.P = q; q += (size_t)n * fi;
    w.H1 = q; q += (size_t)n * hd;
    w.dH1 = q; q += (size_t)n * hd;
    w.Q = q; q += (size_t)n * c;
    w.Z = q; q += (size_t)n * c;
    w.dZ = q; q += (size_t)n * c;
    w.dQ = q; q += (size_t)n * c;
    w.rowloss = q; q += (size_t)n;
    w.scratch = q;
    int rc;
    // forward
    if ((rc = ag_aggregate(p_in, X, w.P, stream))) return rc;                       // P = A X
    if ((rc = gemm_rm(b, false, false, n, hd, fi, w.P, io->W1, w.H1))) return rc;   // P W1
    if ((rc = launch_bias_relu(n, hd, io->b1, w.H1, stream))) return rc;            // H1 = relu(. + b1)
    if ((rc = gemm_rm(b, false, false, n, c, hd, w.H1, io->W2, w.Q))) return rc;    // Q = H1 W2
    if ((rc = ag_aggregate(p_out, w.Q, w.Z, stream))) return rc;                    // Z = A Q (+ b2 below)
    if ((rc = launch_softmax_xent(n, c, w.Z, io->b2, labels, io->logits, w.dZ, w.rowloss, stream))) return rc;
    if ((rc = launch_col_sum(n, 1, w.rowloss, io->loss, w.scratch, stream))) return rc;
    // backward
    if ((rc = launch_col_sum(n, c, w.dZ, io->db2, w.scratch, stream))) return rc;
    if ((rc = ag_aggregate_t(p_out, w.dZ, w.dQ, stream))) return rc;                // dQ = A^T dZ
    if ((rc = launch_gemm_tn(n, hd, c, w.H1, w.dQ, io->dW2, w.scratch, stream))) return rc;   // dW2 = H1^T dQ
    if ((rc = gemm_rm(b, false, true, n, hd, c, w.dQ, io->W2, w.dH1))) return rc;   // dH1 = dQ W2^T
    if ((rc = launch_relu_grad(n * (int64_t)hd, w.H1, w.dH1, stream))) return rc;   // through the ReLU
    if ((rc = launch_gemm_tn(n, fi, hd, w.P, w.dH1, io->dW1, w.scratch, stream))) return rc;  // dW1 = P^T dPre
    if ((rc = launch_col_sum(n, hd, w.dH1, io->db1, w.scratch, stream))) return rc;
    return AG_OK;
}

}  // extern "C"
