// L-layer GIN training step (paper Sec. 5 "Benchmarks": GIN; Sec. 2.1: aggregate-sum followed by
// a dense Update), forward + backward.  Every aggregation runs through the plans' adaptive
// kernels; the Update GEMMs, bias / ReLU / ReLU-backward / bias-gradient work are the library's
// own fused fp32 MFMA kernels.
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

size_t pad4(size_t floats) { return (floats + 3) & ~(size_t)3; }   // sub-buffers stay 16-byte aligned

bool widths_ok(const ag_gin_io *io)
{
    if (!io || io->n_layers < 1 || io->n_layers > AG_GIN_MAX_LAYERS) return false;
    for (int l = 0; l <= io->n_layers; ++l)
        if (io->width[l] < 1) return false;
    return true;
}

// the last layer transforms first when that makes its aggregation narrower
bool last_transforms_first(const ag_gin_io *io)
{
    const int L = io->n_layers;
    return io->width[L - 1] > io->width[L];
}

struct Layout {
    size_t A[AG_GIN_MAX_LAYERS], H[AG_GIN_MAX_LAYERS + 1];   // offsets (floats); H[0] unused
    size_t Q, Z, dZ, T, dP[2], rowloss, WT, wsplit, scratch, total;
};

Layout carve(int64_t n, const ag_gin_io *io)
{
    Layout y{};
    const int L = io->n_layers;
    const bool tf = last_transforms_first(io);
    size_t at = 0;
    auto take = [&](size_t floats) { size_t o = at; at += pad4(floats); return o; };
    int32_t wmax_out = 1, whid = 1;
    size_t wt = 1, sc = col_sum_scratch_floats(1), wsp = 0;
    for (int l = 0; l < L; ++l) {
        const int32_t wi = io->width[l], wo = io->width[l + 1];
        if (!(tf && l == L - 1)) y.A[l] = take((size_t)n * wi);
        if (l < L - 1) { y.H[l + 1] = take((size_t)n * wo); whid = std::max(whid, wo); }
        wmax_out = std::max(wmax_out, wo);
        wt = std::max(wt, (size_t)wi * wo);
        wsp = std::max(wsp, std::max(gemm_nn_b3_scratch_floats(wi, wo), gemm_nn_b3_scratch_floats(wo, wi)));
        sc = std::max(sc, gemm_tn_scratch_floats(wi, wo));
        sc = std::max(sc, col_sum_scratch_floats(std::max(wi, wo)));
        sc = std::max(sc, hidden_backward_scratch_floats(n, wi, wo));
    }
    const int32_t c = io->width[L];
    y.Q = take((size_t)n * c);
    y.Z = take((size_t)n * c);
    y.dZ = take((size_t)n * c);
    y.T = take((size_t)n * wmax_out);
    y.dP[0] = take((size_t)n * whid);
    y.dP[1] = take((size_t)n * whid);
    y.rowloss = take((size_t)n);
    y.WT = take(wt);
    y.wsplit = take(wsp + 4);
    y.scratch = take(sc + 64);
    y.total = at;
    return y;
}

}  // namespace

extern "C" {

size_t ag_gin_workspace_bytes(int64_t n, const ag_gin_io *io)
{
    if (n < 0 || !widths_ok(io)) return 0;
    return carve(n, io).total * sizeof(float);
}

int ag_gin_step(ag_plan *const *plans, const ag_gin_io *io, const float *X, const int32_t *labels,
                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!plans || !io || !X || !labels || !workspace) { set_error("null argument"); return AG_ERR_INVALID; }
    if (!widths_ok(io)) { set_error("bad layer count or width"); return AG_ERR_INVALID; }
    const int L = io->n_layers;
    uintptr_t align_all = (uintptr_t)X | (uintptr_t)workspace | (uintptr_t)io->logits;
    for (int l = 0; l <= L; ++l) {
        if (!plans[l]) { set_error("null plan"); return AG_ERR_INVALID; }
        if (plan_host_only(plans[l])) { set_error("host-only plan"); return AG_ERR_UNSUPPORTED; }
        if (plan_layout(plans[l]) != AG_LAYOUT_REORDERED) {
            set_error("ag_gin_step needs AG_LAYOUT_REORDERED plans");
            return AG_ERR_UNSUPPORTED;
        }
        if (plan_f(plans[l]) != io->width[l] || !plan_same_topology(plans[0], plans[l])) {
            set_error("plans do not match the layer widths (need clones of one topology with F = width[l])");
            return AG_ERR_INVALID;
        }
    }
    for (int l = 0; l < L; ++l) {
        if (!io->W[l] || !io->b[l] || !io->dW[l] || !io->db[l]) {
            set_error("null parameter or gradient pointer");
            return AG_ERR_INVALID;
        }
        align_all |= (uintptr_t)io->W[l] | (uintptr_t)io->dW[l];
    }
    if (!io->loss) { set_error("null loss pointer"); return AG_ERR_INVALID; }
    if (align_all & 15) { set_error("device pointers must be 16-byte aligned"); return AG_ERR_INVALID; }
    const int64_t n = plan_n(plans[0]);
    const Layout y = carve(n, io);
    if (workspace_bytes < y.total * sizeof(float)) { set_error("workspace too small"); return AG_ERR_INVALID; }
    float *ws = (float *)workspace;
    const bool tf = last_transforms_first(io);
    const int32_t c = io->width[L];
    const float eps = io->eps;
    float *wsplit = ws + y.wsplit;
    int rc;

    // ---- forward -------------------------------------------------------------------------------
    const float *Hl[AG_GIN_MAX_LAYERS + 1];
    Hl[0] = X;
    for (int l = 0; l < L; ++l) {
        const int32_t wi = io->width[l], wo = io->width[l + 1];
        if (l < L - 1) {
            float *A = ws + y.A[l], *Hn = ws + y.H[l + 1];
            if ((rc = ag_gin_layer(plans[l], eps, Hl[l], A, stream))) return rc;                       // A_l
            if ((rc = launch_gemm_nn_auto(n, wi, wo, A, io->W[l], Hn, 1, io->b[l], wsplit, stream))) return rc;    // relu(A W + b)
            Hl[l + 1] = Hn;
        } else if (tf) {
            if ((rc = launch_gemm_nn_auto(n, wi, c, Hl[l], io->W[l], ws + y.Q, 0, nullptr, wsplit, stream))) return rc;   // Q = H W
            if ((rc = ag_gin_layer(plans[L], eps, ws + y.Q, ws + y.Z, stream))) return rc;                   // A.Q (+ b below)
        } else {
            float *A = ws + y.A[l];
            if ((rc = ag_gin_layer(plans[l], eps, Hl[l], A, stream))) return rc;
            if ((rc = launch_gemm_nn_auto(n, wi, c, A, io->W[l], ws + y.Z, 0, nullptr, wsplit, stream))) return rc;
        }
    }
    float *dZ = ws + y.dZ, *scratch = ws + y.scratch, *T = ws + y.T, *WT = ws + y.WT;
    if ((rc = launch_softmax_xent(n, c, ws + y.Z, io->b[L - 1], labels, io->logits, dZ, ws + y.rowloss, stream))) return rc;
    if ((rc = launch_col_sum(n, 1, ws + y.rowloss, io->loss, scratch, stream))) return rc;

    // ---- backward ------------------------------------------------------------------------------
    const float *dPre = dZ;                    // gradient w.r.t. the pre-activation of layer l, N x width[l+1]
    for (int l = L - 1; l >= 0; --l) {
        const int32_t wi = io->width[l], wo = io->width[l + 1];
        float *dPrev = ws + y.dP[l & 1];       // N x width[l]: gradient of layer l-1's pre-activation
        const bool layer_tf = tf && l == L - 1;
        if (layer_tf) {
            if ((rc = launch_col_sum(n, wo, dPre, io->db[l], scratch, stream))) return rc;
            if ((rc = ag_gin_layer_t(plans[L], eps, dPre, T, stream))) return rc;                     // T = A^T dZ
            if (l == 0) {
                if ((rc = launch_gemm_tn(n, wi, wo, X, T, io->dW[l], nullptr, scratch, stream))) return rc;
                break;
            }
            if ((rc = launch_transpose_small(wi, wo, io->W[l], WT, stream))) return rc;
            rc = launch_hidden_backward(n, wi, wo, T, WT, Hl[l], dPrev, io->dW[l], scratch, stream);
            if (rc == AG_ERR_UNSUPPORTED) {
                if ((rc = launch_gemm_tn(n, wi, wo, Hl[l], T, io->dW[l], nullptr, scratch, stream))) return rc;
                rc = launch_gemm_nn_auto(n, wo, wi, T, WT, dPrev, 2, Hl[l], wsplit, stream);
            }
            if (rc) return rc;
        } else {
            // dW_l = A_l^T dPre, db_l = column sums of dPre
            if ((rc = launch_gemm_tn(n, wi, wo, ws + y.A[l], dPre, io->dW[l], io->db[l], scratch, stream))) return rc;
            if (l == 0) break;
            if ((rc = ag_gin_layer_t(plans[l + 1], eps, dPre, T, stream))) return rc;                 // T = A^T dPre
            if ((rc = launch_transpose_small(wi, wo, io->W[l], WT, stream))) return rc;
            // dPre_{l-1} = (T W_l^T) masked by H_l > 0
            if ((rc = launch_gemm_nn_auto(n, wo, wi, T, WT, dPrev, 2, Hl[l], wsplit, stream))) return rc;
        }
        dPre = dPrev;
    }
    return AG_OK;
}

}  // extern "C"
