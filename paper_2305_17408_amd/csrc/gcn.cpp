// Two-layer GCN training step (paper Sec. 5 "Benchmarks": GCN with its default two layers),
// forward + backward.  The three aggregations run through the plans' adaptive kernels; the
// dense Update GEMMs (Sec. 2.1) are the library's own fp32 MFMA kernels with the bias / ReLU /
// ReLU-backward / bias-gradient work fused into them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

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

struct Ws {
    float *P, *H1, *Q, *Z, *dZ, *dQ, *dH1, *rowloss, *W2T, *wsplit, *scratch;
};

// every sub-buffer starts on a 16-byte boundary (the kernels use 16-byte loads where widths allow)
size_t pad4(size_t floats) { return (floats + 3) & ~(size_t)3; }

// scratch for the split (bf16 pieces) copy of a weight matrix, largest over the transforms of the step
size_t wsplit_floats(int32_t fi, int32_t hd, int32_t c)
{
    return std::max(std::max(gemm_nn_b3_scratch_floats(fi, hd), gemm_nn_b3_scratch_floats(hd, c)),
                    gemm_nn_b3_scratch_floats(c, hd));
}

size_t ws_floats(int64_t n, int32_t fi, int32_t hd, int32_t c)
{
    return pad4((size_t)n * fi) + 2 * pad4((size_t)n * hd) + 4 * pad4((size_t)n * c) + pad4((size_t)n) +
           pad4((size_t)hd * c) + pad4(wsplit_floats(fi, hd, c)) +
           std::max(std::max(std::max(col_sum_scratch_floats(std::max(hd, c)), hidden_backward_scratch_floats(n, hd, c)),
                             std::max(gemm_tn_scratch_floats(fi, hd), gemm_tn_scratch_floats(hd, c))),
                    gcn_backward_fused_scratch_floats(n, fi, hd, c)) + 64;
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
    const uintptr_t align_all = (uintptr_t)X | (uintptr_t)workspace | (uintptr_t)io->W1 | (uintptr_t)io->b1 |
                                (uintptr_t)io->W2 | (uintptr_t)io->b2 | (uintptr_t)io->dW1 | (uintptr_t)io->dW2 |
                                (uintptr_t)io->logits;
    if (align_all & 15) { set_error("device pointers must be 16-byte aligned"); return AG_ERR_INVALID; }
    Ws w;
    float *q = (float *)workspace;
    w.P = q; q += pad4((size_t)n * fi);
    w.H1 = q; q += pad4((size_t)n * hd);
    w.dH1 = q; q += pad4((size_t)n * hd);
    w.Q = q; q += pad4((size_t)n * c);
    w.Z = q; q += pad4((size_t)n * c);
    w.dZ = q; q += pad4((size_t)n * c);
    w.dQ = q; q += pad4((size_t)n * c);
    w.rowloss = q; q += pad4((size_t)n);
    w.W2T = q; q += pad4((size_t)hd * c);
    w.wsplit = q; q += pad4(wsplit_floats(fi, hd, c));
    w.scratch = q;
    int rc;
    // forward
    if ((rc = ag_aggregate(p_in, X, w.P, stream))) return rc;                                  // P = A X
    // H1 = relu(P W1 + b1) and Q = H1 W2: in one pass where the shape allows it
    rc = launch_gemm_chain_b3(n, fi, hd, c, w.P, io->W1, io->b1, io->W2, w.H1, w.Q, w.wsplit, stream);
    if (rc == AG_ERR_UNSUPPORTED) {
        if ((rc = launch_gemm_nn_auto(n, fi, hd, w.P, io->W1, w.H1, 1, io->b1, w.wsplit, stream))) return rc;
        rc = launch_gemm_nn_auto(n, hd, c, w.H1, io->W2, w.Q, 0, nullptr, w.wsplit, stream);
    }
    if (rc) return rc;
    if ((rc = ag_aggregate(p_out, w.Q, w.Z, stream))) return rc;                               // Z = A Q (+ b2 below)
    if ((rc = launch_softmax_xent(n, c, w.Z, io->b2, labels, io->logits, w.dZ, w.rowloss, stream))) return rc;
    if ((rc = launch_col_sum(n, 1, w.rowloss, io->loss, w.scratch, stream))) return rc;
    // backward
    if ((rc = launch_col_sum(n, c, w.dZ, io->db2, w.scratch, stream))) return rc;
    if ((rc = ag_aggregate_t(p_out, w.dZ, w.dQ, stream))) return rc;                           // dQ = A^T dZ
    if ((rc = launch_transpose_small(hd, c, io->W2, w.W2T, stream))) return rc;
    // dW2, dW1 and db1 in one pass over P, H1 and dQ, dPre never leaving the registers, where the shape allows it
    rc = launch_gcn_backward_fused(n, fi, hd, c, w.dQ, w.W2T, w.H1, w.P, io->dW1, io->db1, io->dW2, w.scratch, stream);
    if (rc != AG_ERR_UNSUPPORTED) return rc;
    // otherwise dW2 = H1^T dQ and dPre = (dQ W2^T) * (H1 > 0) in one fused pass where the shape allows that
    rc = launch_hidden_backward(n, hd, c, w.dQ, w.W2T, w.H1, w.dH1, io->dW2, w.scratch, stream);
    if (rc == AG_ERR_UNSUPPORTED) {
        if ((rc = launch_gemm_tn(n, hd, c, w.H1, w.dQ, io->dW2, nullptr, w.scratch, stream))) return rc;
        rc = launch_gemm_nn_auto(n, c, hd, w.dQ, w.W2T, w.dH1, 2, w.H1, w.wsplit, stream);
    }
    if (rc) return rc;
    if ((rc = launch_gemm_tn(n, fi, hd, w.P, w.dH1, io->dW1, io->db1, w.scratch, stream))) return rc;  // dW1 = P^T dPre, db1
    return AG_OK;
}

}  // extern "C"
