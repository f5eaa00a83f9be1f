// Plan life cycle, kernel composition and the adaptive selector (paper Sec. 3.1, Sec. 3.3).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstring>

#include "ag_internal.h"
#include "selector.h"

namespace ag {

static thread_local std::string g_err;
void set_error(const std::string &msg)
{
    try { g_err = msg; } catch (...) { }                 // out of memory: the code still reaches the caller
}
int hip_fail(int code, const char *what)
{
    if (code == (int)hipSuccess) return AG_OK;
    try { g_err = std::string(what) + ": " + hipGetErrorString((hipError_t)code); } catch (...) { }
    return AG_ERR_HIP;
}

namespace {

double now_sec()
{
    using namespace std::chrono;
    return duration<double>(steady_clock::now().time_since_epoch()).count();
}

void *default_alloc(size_t bytes, void *)
{
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
    return p;
}
void default_free(void *p, void *) { (void)hipFree(p); }

}  // namespace

// Everything that depends only on the matrix: shared by a plan and its width clones.
struct Topology {
    ag_options opt{};
    int64_t n = 0, nnz = 0;
    bool unit = false, symmetric = false, host_only = false;
    bool factored = false;              // intra-community values are row_scale[i] * col_scale[j]: blocks run value-free
    std::vector<float> rs_plan, cs_plan;   // the factors in plan numbering (empty = all ones)
    const float *rs_dev = nullptr, *cs_dev = nullptr;
    ReorderResult r;
    HostDir h[2];                       // h[1] is filled only for non-symmetric matrices
    std::vector<int32_t> dense_blocks, sparse_blocks, all_blocks;
    DevDir d[2];
    const int32_t *perm_dev = nullptr;
    std::vector<void *> owned;          // device allocations
    int64_t device_bytes = 0;
    double sec_reorder = 0, sec_split = 0, sec_build = 0, sec_upload = 0;
    int64_t max_segments = 0;

    ~Topology()
    {
        for (void *p : owned) opt.dev_free(p, opt.user);
    }

    void *dalloc(size_t bytes)
    {
        void *p = opt.dev_alloc(bytes ? bytes : 16, opt.user);
        if (p) {
            owned.push_back(p);
            device_bytes += (int64_t)bytes;
        }
        return p;
    }

    template <class T>
    int upload(const std::vector<T> &v, const T *&out)
    {
        out = nullptr;
        void *p = dalloc(v.size() * sizeof(T));
        if (!p) { set_error("device allocation failed"); return AG_ERR_NOMEM; }
        if (!v.empty()) {
            int rc = hip_fail((int)hipMemcpy(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice), "upload");
            if (rc) return rc;
        }
        out = (const T *)p;
        return AG_OK;
    }

    int upload_csr(const HostCsr &A, const HostDir::Segs &s, CsrDev &D, bool with_rows)
    {
        int rc;
        D.n = (int32_t)A.n;
        D.nnz = (int32_t)A.nnz();
        if (with_rows) {                                  // COO form: the row of every entry
            std::vector<int32_t> rows((size_t)A.nnz());
            for (int64_t i = 0; i < A.n; ++i)
                std::fill(rows.begin() + A.rowptr[i], rows.begin() + A.rowptr[i + 1], (int32_t)i);
            if ((rc = upload(rows, D.row))) return rc;
        }
        if ((rc = upload(A.rowptr, D.rowptr))) return rc;
        if ((rc = upload(A.col, D.col))) return rc;
        if (!A.val.empty()) { if ((rc = upload(A.val, D.val))) return rc; }
        if ((rc = upload(s.seg_row, D.seg_row))) return rc;
        if ((rc = upload(s.seg_beg, D.seg_beg))) return rc;
        if ((rc = upload(s.seg_end, D.seg_end))) return rc;
        if ((rc = upload(s.lr_row, D.lr_row))) return rc;
        if ((rc = upload(s.lr_seg0, D.lr_seg0))) return rc;
        D.nseg = (int32_t)s.seg_row.size();
        D.nlr = (int32_t)s.lr_row.size();
        max_segments = std::max<int64_t>(max_segments, D.nseg);
        return AG_OK;
    }

    int upload_dir(int k, const int32_t *blk_ptr_dev, const int32_t *ld, const int32_t *ls, const int32_t *la)
    {
        HostDir &H = h[k];
        DevDir &D = d[k];
        int rc;
        if ((rc = upload_csr(H.full, H.segs_full, D.full, false))) return rc;
        if ((rc = upload_csr(H.inter, H.segs_inter, D.inter, true))) return rc;
        BlocksDev &B = D.blk;
        B.blk_ptr = blk_ptr_dev;
        B.nb = r.n_blocks;
        B.n_block_rows = r.blk_ptr.back();
        B.max_block_rows = 0;
        for (int32_t b = 0; b < r.n_blocks; ++b) B.max_block_rows = std::max(B.max_block_rows, r.blk_ptr[b + 1] - r.blk_ptr[b]);
        std::vector<int32_t> irp(H.intra.rowptr.begin(), H.intra.rowptr.begin() + B.n_block_rows + 1);
        if ((rc = upload(irp, B.i_rowptr))) return rc;
        if ((rc = upload(H.intra_col8, B.i_col8))) return rc;
        if (!H.intra.val.empty() && !factored) { if ((rc = upload(H.intra.val, B.i_val))) return rc; }
        B.list_dense = ld; B.list_sparse = ls; B.list_all = la;
        B.n_dense = (int32_t)dense_blocks.size();
        B.n_sparse = (int32_t)sparse_blocks.size();
        if ((rc = upload(H.bitmap, B.bitmap))) return rc;
        if (!unit && !factored && B.n_dense > 0) { if ((rc = upload(H.tiles, B.tiles))) return rc; }
        // A = diag(rs) P diag(cs): forward scales sources by cs and sums by rs; A^T the other way round
        B.in_scale = (k == 0) ? cs_dev : rs_dev;
        B.out_scale = (k == 0) ? rs_dev : cs_dev;
        return AG_OK;
    }
};

}  // namespace ag

using namespace ag;

struct ag_plan {
    std::shared_ptr<Topology> topo;
    int32_t F = 0, layout = 0, trials = 3;
    float *partial = nullptr;            // long-row partial sums: max_segments x F
    float *tmp_in = nullptr, *tmp_out = nullptr;   // AG_LAYOUT_ORIGINAL staging, n x F each
    Selector sel[2];
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    std::vector<void *> owned;
    // optional per-call kernel timing (ag_plan_set_profiling): a ring of event quadruples
    struct Pending { int dir; int slot; };
    bool profiling = false;
    std::vector<hipEvent_t> prof_ev;            // 4 * kProfRing events
    std::vector<Pending> prof_pending;
    int prof_next = 0;
    double prof_ms[2][3] = {{0, 0, 0}, {0, 0, 0}}, prof_total[2] = {0, 0};
    int64_t prof_calls[2] = {0, 0};

    ~ag_plan()
    {
        for (auto &e : ev) if (e) (void)hipEventDestroy(e);
        for (auto &e : prof_ev) if (e) (void)hipEventDestroy(e);
        if (topo) for (void *p : owned) topo->opt.dev_free(p, topo->opt.user);
    }
};

namespace {

void init_selector(ag_plan *p, int dir, bool keep_forced)
{
    Selector &s = p->sel[dir];
    s.reset(keep_forced);
    const Topology &t = *p->topo;
    s.ncand[AG_CLS_BLOCKS_DENSE] = t.dense_blocks.empty() ? 1 : ((t.unit || t.factored) ? 3 : 2);
    s.ncand[AG_CLS_BLOCKS_SPARSE] = 1;
    s.ncand[AG_CLS_REMAINDER] = 3;
    s.ncand[AG_CLS_COMPOSE] = 4;
}

int plan_device_buffers(ag_plan *p)
{
    Topology &t = *p->topo;
    if (t.host_only) return AG_OK;
    auto take = [&](size_t bytes) -> float * {
        void *q = t.opt.dev_alloc(bytes ? bytes : 16, t.opt.user);
        if (q) p->owned.push_back(q);
        return (float *)q;
    };
    p->partial = take((size_t)t.max_segments * p->F * sizeof(float));
    if (!p->partial) { set_error("device allocation failed (partials)"); return AG_ERR_NOMEM; }
    if (p->layout == AG_LAYOUT_ORIGINAL) {
        p->tmp_in = take((size_t)t.n * p->F * sizeof(float));
        p->tmp_out = take((size_t)t.n * p->F * sizeof(float));
        if (!p->tmp_in || !p->tmp_out) { set_error("device allocation failed (staging)"); return AG_ERR_NOMEM; }
    }
    return AG_OK;
}

// Enqueue one aggregation with a fixed kernel choice.  `ev` (4 events) may be null.
int run_choice(ag_plan *p, int dir_idx, const int *k, const float *H, float *Y, hipStream_t st,
               hipEvent_t *ev, float *partial)
{
    const Topology &t = *p->topo;
    const DevDir &D = t.d[dir_idx];
    const int32_t F = p->F, n = (int32_t)t.n, nbr = D.blk.n_block_rows;
    const int wide = k[AG_CLS_REMAINDER];                 // CSR kernel variant (COO falls back to narrow)
    const bool coo = k[AG_CLS_REMAINDER] == AG_K_COO;     // only the SPLIT composition has a COO form
    int rc = AG_OK;
    if (ev) (void)hipEventRecord(ev[0], st);
    switch (k[AG_CLS_COMPOSE]) {
    case AG_COMPOSE_FULL_CSR:
    case AG_COMPOSE_FULL_CSR_WIDE:
        if (ev) { (void)hipEventRecord(ev[1], st); (void)hipEventRecord(ev[2], st); }
        if ((rc = launch_csr_rows(D.full, H, Y, F, 0, n, 0,
                                  k[AG_CLS_COMPOSE] == AG_COMPOSE_FULL_CSR_WIDE ? AG_K_CSR_WIDE : AG_K_CSR_NARROW, st)))
            return rc;
        if ((rc = launch_csr_long(D.full, H, Y, F, partial, 0, st))) return rc;
        break;
    case AG_COMPOSE_FUSED:
        if (k[AG_CLS_BLOCKS_DENSE] != AG_K_BLOCK_SPARSE && D.blk.n_dense >= AG_MIN_BLOCKS_OWN_LAUNCH) {
            // the dense class keeps its own kernel, which then also adds its rows' remainder
            if ((rc = launch_block_dense(D.blk, &D.inter, H, Y, F, k[AG_CLS_BLOCKS_DENSE], st))) return rc;
            if (ev) (void)hipEventRecord(ev[1], st);
            if ((rc = launch_block_sparse(D.blk, D.blk.list_sparse, D.blk.n_sparse, &D.inter, H, Y, F, st))) return rc;
            if (ev) (void)hipEventRecord(ev[2], st);
        } else {
            if ((rc = launch_block_sparse(D.blk, D.blk.list_all, D.blk.nb, &D.inter, H, Y, F, st))) return rc;
            if (ev) { (void)hipEventRecord(ev[1], st); (void)hipEventRecord(ev[2], st); }
        }
        if ((rc = launch_csr_rows(D.inter, H, Y, F, nbr, n, 0, wide, st))) return rc;
        if ((rc = launch_csr_long(D.inter, H, Y, F, partial, nbr, st))) return rc;
        break;
    default:
        if (k[AG_CLS_BLOCKS_DENSE] != AG_K_BLOCK_SPARSE)
            rc = launch_block_dense(D.blk, nullptr, H, Y, F, k[AG_CLS_BLOCKS_DENSE], st);
        else
            rc = launch_block_sparse(D.blk, D.blk.list_dense, D.blk.n_dense, nullptr, H, Y, F, st);
        if (rc) return rc;
        if (ev) (void)hipEventRecord(ev[1], st);
        if ((rc = launch_block_sparse(D.blk, D.blk.list_sparse, D.blk.n_sparse, nullptr, H, Y, F, st))) return rc;
        if (ev) (void)hipEventRecord(ev[2], st);
        if (coo) {
            if ((rc = launch_coo(D.inter, H, Y, F, nbr, st))) return rc;
        } else {
            if ((rc = launch_csr_rows(D.inter, H, Y, F, 0, n, nbr, wide, st))) return rc;
            if ((rc = launch_csr_long(D.inter, H, Y, F, partial, nbr, st))) return rc;
        }
        break;
    }
    if (ev) (void)hipEventRecord(ev[3], st);
    return AG_OK;
}

// Read the events of a trial call and hand the four intervals to the selector.
void record_trial(ag_plan *p, Selector &s, const int *k, hipEvent_t *ev)
{
    float ms[4] = {0, 0, 0, 0};
    (void)hipEventSynchronize(ev[3]);
    (void)hipEventElapsedTime(&ms[0], ev[0], ev[1]);
    (void)hipEventElapsedTime(&ms[1], ev[1], ev[2]);
    (void)hipEventElapsedTime(&ms[2], ev[2], ev[3]);
    (void)hipEventElapsedTime(&ms[3], ev[0], ev[3]);
    selector_record(s, p->trials, k, ms);
}

constexpr int kProfRing = 64;

void prof_drain(ag_plan *p)
{
    for (const auto &q : p->prof_pending) {
        hipEvent_t *e = p->prof_ev.data() + 4 * q.slot;
        float a = 0, b = 0, c = 0, d = 0;
        (void)hipEventSynchronize(e[3]);
        (void)hipEventElapsedTime(&a, e[0], e[1]);
        (void)hipEventElapsedTime(&b, e[1], e[2]);
        (void)hipEventElapsedTime(&c, e[2], e[3]);
        (void)hipEventElapsedTime(&d, e[0], e[3]);
        p->prof_ms[q.dir][0] += a;
        p->prof_ms[q.dir][1] += b;
        p->prof_ms[q.dir][2] += c;
        p->prof_total[q.dir] += d;
        p->prof_calls[q.dir]++;
    }
    p->prof_pending.clear();
    p->prof_next = 0;
}

int check_call(const ag_plan *p, const float *X, const float *Y)
{
    if (!p) { set_error("null plan"); return AG_ERR_INVALID; }
    const Topology &t = *p->topo;
    if (t.host_only) { set_error("plan was created with AG_FLAG_HOST_ONLY"); return AG_ERR_UNSUPPORTED; }
    if (t.n == 0) return AG_OK;
    if (!X || !Y) { set_error("null argument"); return AG_ERR_INVALID; }
    if (X == Y) { set_error("input and output must not alias"); return AG_ERR_INVALID; }
    if ((((uintptr_t)X | (uintptr_t)Y) & 15)) {
        set_error("feature matrices must be 16-byte aligned");
        return AG_ERR_INVALID;
    }
    return AG_OK;
}

int aggregate_dir(ag_plan *p, int dir, const float *X, float *Y, void *stream)
{
    int rc0 = check_call(p, X, Y);
    if (rc0 || p->topo->n == 0) return rc0;
    Topology &t = *p->topo;
    hipStream_t st = (hipStream_t)stream;
    const int dir_idx = (dir == AG_DIR_BWD && !t.symmetric) ? 1 : 0;
    Selector &s = p->sel[dir];
    const float *in = X;
    float *out = Y;
    int rc;
    if (p->layout == AG_LAYOUT_ORIGINAL) {
        if ((rc = launch_permute_rows(t.perm_dev, t.n, p->F, X, p->tmp_in, false, st))) return rc;
        in = p->tmp_in;
        out = p->tmp_out;
    }
    int k[AG_NUM_CLS];
    ++s.calls;
    const bool trial = selector_next(s, k);
    if (trial && !p->ev[0])
        for (auto &e : p->ev)
            if ((rc = hip_fail((int)hipEventCreate(&e), "event create"))) return rc;
    hipEvent_t *evs = trial ? p->ev : nullptr;
    if (!trial && p->profiling) {
        if ((int)p->prof_pending.size() >= kProfRing) prof_drain(p);
        evs = p->prof_ev.data() + 4 * p->prof_next;
        p->prof_pending.push_back({dir, p->prof_next++});
    }
    if ((rc = run_choice(p, dir_idx, k, in, out, st, evs, p->partial))) return rc;
    if (trial) record_trial(p, s, k, p->ev);
    if (p->layout == AG_LAYOUT_ORIGINAL)
        if ((rc = launch_permute_rows(t.perm_dev, t.n, p->F, p->tmp_out, Y, true, st))) return rc;
    return AG_OK;
}

}  // namespace

namespace ag {

// Forward aggregation with the plan's settled kernel choice and caller-supplied memory for the
// partial sums of long rows.  Creates no event, grows no container and allocates no device or
// host memory: a call that would need a selector trial is refused instead.
int aggregate_settled(ag_plan *p, const float *X, float *Y, float *partial, size_t partial_bytes, void *stream)
{
    int rc = check_call(p, X, Y);
    if (rc || p->topo->n == 0) return rc;
    const Topology &t = *p->topo;
    Selector &s = p->sel[AG_DIR_FWD];
    int k[AG_NUM_CLS];
    bool all_forced = true;
    for (int c = 0; c < AG_NUM_CLS; ++c) all_forced = all_forced && s.forced[c] >= 0;
    if (all_forced) {
        for (int c = 0; c < AG_NUM_CLS; ++c) k[c] = s.forced[c];
    } else if (s.phase == 2) {
        for (int c = 0; c < AG_NUM_CLS; ++c) k[c] = s.choice[c];
    } else {
        set_error("the kernel choice is not settled yet: run ag_aggregate until the selector has frozen, "
                  "or pin all four classes with ag_plan_force_kernels");
        return AG_ERR_UNSUPPORTED;
    }
    const size_t need = (size_t)t.max_segments * (size_t)p->F * sizeof(float);
    if (need > partial_bytes) {
        try {
            set_error("long-row partial sums need " + std::to_string(need) + " bytes of scratch, more than the " +
                      std::to_string(partial_bytes) + " bytes of the static buffer");
        } catch (...) { }
        return AG_ERR_UNSUPPORTED;
    }
    hipStream_t st = (hipStream_t)stream;
    const float *in = X;
    float *out = Y;
    if (p->layout == AG_LAYOUT_ORIGINAL) {               // staging buffers exist since plan creation
        if ((rc = launch_permute_rows(t.perm_dev, t.n, p->F, X, p->tmp_in, false, st))) return rc;
        in = p->tmp_in;
        out = p->tmp_out;
    }
    if ((rc = run_choice(p, 0, k, in, out, st, nullptr, partial))) return rc;
    if (p->layout == AG_LAYOUT_ORIGINAL)
        if ((rc = launch_permute_rows(t.perm_dev, t.n, p->F, p->tmp_out, Y, true, st))) return rc;
    return AG_OK;
}

}  // namespace ag

namespace {

// A reordering handed in by the caller: checked completely (a permutation, ascending block
// pointers, block sizes the kernels accept) before anything is built on it.
bool adopt_reordering(int64_t n, const int32_t *perm, const int32_t *blk_ptr, int32_t n_blocks, ag::ReorderResult &r,
                      std::string &err)
{
    if (n_blocks < 0 || (n_blocks > 0 && !blk_ptr)) { err = "reuse_blk_ptr / reuse_n_blocks do not describe blocks"; return false; }
    r.perm.assign(perm, perm + n);
    r.iperm.assign((size_t)n, -1);
    for (int64_t q = 0; q < n; ++q) {
        const int32_t v = perm[q];
        if (v < 0 || v >= n || r.iperm[v] != -1) { err = "reuse_perm is not a permutation of 0..n-1"; return false; }
        r.iperm[v] = (int32_t)q;
    }
    r.blk_ptr.assign((size_t)n_blocks + 1, 0);
    for (int32_t b = 0; b <= n_blocks; ++b) r.blk_ptr[b] = n_blocks > 0 ? blk_ptr[b] : 0;
    if (r.blk_ptr[0] != 0 || r.blk_ptr[n_blocks] > n) { err = "reuse_blk_ptr must run from 0 to at most n"; return false; }
    for (int32_t b = 0; b < n_blocks; ++b) {
        const int64_t sz = (int64_t)r.blk_ptr[b + 1] - r.blk_ptr[b];
        if (sz < 1 || sz > ag::kMaxBlockWide) { err = "reuse_blk_ptr: every block needs 1..256 rows"; return false; }
    }
    r.n_blocks = n_blocks;
    r.comm.clear();
    return true;
}

}  // namespace

using namespace ag;

extern "C" {

const char *ag_last_error(void) { return g_err.c_str(); }

int ag_plan_create(const ag_csr *A, int64_t N, int32_t F, const ag_options *opt_in, ag_plan **out)
{
    if (!out) { set_error("out is null"); return AG_ERR_INVALID; }
    *out = nullptr;
    if (!A || A->n != N) { set_error("N does not match the matrix"); return AG_ERR_INVALID; }
    if (F < 1) { set_error("F must be at least 1"); return AG_ERR_INVALID; }
    ag_options o{};
    if (opt_in) o = *opt_in;
    if (o.num_communities < 0) { set_error("option out of range"); return AG_ERR_INVALID; }
    if (o.block_cap == 0 && o.num_communities > 0)
        o.block_cap = (int32_t)std::max<int64_t>(1, std::min<int64_t>(kMaxBlockWide, (N + o.num_communities - 1) / o.num_communities));
    if (o.block_cap == 0) o.block_cap = kMaxBlock;
    if (o.min_block == 0) o.min_block = std::min(16, o.block_cap);
    if (o.sweeps == 0) o.sweeps = 8;
    if (o.max_levels == 0) o.max_levels = 12;
    if (o.order_levels == 0) o.order_levels = 3;          // negative = keep the communities in id order
    if (o.trials == 0) o.trials = 3;
    if (o.block_cap < 1 || o.block_cap > kMaxBlockWide || o.min_block < 1 || o.sweeps < 1 || o.max_levels < 1 ||
        o.trials < 1 || o.trials > kMaxTrials || (o.method != AG_METHOD_LABEL_PROPAGATION && o.method != AG_METHOD_MODULARITY) || (o.layout != AG_LAYOUT_ORIGINAL && o.layout != AG_LAYOUT_REORDERED) ||
        (!o.dev_alloc) != (!o.dev_free)) {
        set_error("option out of range");
        return AG_ERR_INVALID;
    }
    if (!o.dev_alloc) { o.dev_alloc = default_alloc; o.dev_free = default_free; }
    try {
        auto t = std::make_shared<Topology>();
        t->opt = o;
        t->host_only = (o.flags & AG_FLAG_HOST_ONLY) != 0;
        HostCsr A0, At;
        std::string err;
        int rc = ingest_csr(A, A0, err);
        if (rc) { set_error(err); return rc; }
        t->n = A0.n;
        t->nnz = A0.nnz();
        t->unit = A0.val.empty();
        const bool want_factored = o.row_scale || o.col_scale;
        if (want_factored && t->unit) {
            set_error("row_scale / col_scale describe stored values: vals is required");
            return AG_ERR_INVALID;
        }
        // the value-free dense kernels (bit maps, bf16 form) overtake the block-sparse kernel at far lower densities
        if (o.dense_density == 0.f) o.dense_density = t->opt.dense_density = (t->unit || want_factored) ? 0.05f : 0.20f;
        double t0 = now_sec();
        transpose_csr(A0, At);
        t->symmetric = bitwise_equal(A0, At);
        if (o.reuse_perm) {
            if (!adopt_reordering(t->n, o.reuse_perm, o.reuse_blk_ptr, o.reuse_n_blocks, t->r, err)) {
                set_error(err);
                return AG_ERR_INVALID;
            }
        } else {
            WGraph g;
            build_pattern_graph(A0, At, g);
            community_reorder(g, o.method, o.block_cap, o.min_block, o.sweeps, o.max_levels,
                              o.order_levels < 0 ? 0 : o.order_levels, t->r);
        }
        double t1 = now_sec();
        t->sec_reorder = t1 - t0;
        permute_and_split(A0, t->r, t->h[0].full, t->h[0].intra, t->h[0].inter);
        if (!t->symmetric) permute_and_split(At, t->r, t->h[1].full, t->h[1].intra, t->h[1].inter);
        if (want_factored) {
            // factors in plan numbering; every intra-community value must be their product
            const int64_t n = t->n;
            if (o.row_scale) { t->rs_plan.resize(n); for (int64_t q = 0; q < n; ++q) t->rs_plan[q] = o.row_scale[t->r.perm[q]]; }
            if (o.col_scale) { t->cs_plan.resize(n); for (int64_t q = 0; q < n; ++q) t->cs_plan[q] = o.col_scale[t->r.perm[q]]; }
            const HostCsr &I0 = t->h[0].intra;
            for (int64_t i = 0; i < n; ++i)
                for (int32_t e = I0.rowptr[i]; e < I0.rowptr[i + 1]; ++e) {
                    const float prod = (o.row_scale ? t->rs_plan[i] : 1.f) * (o.col_scale ? t->cs_plan[I0.col[e]] : 1.f);
                    const float v = I0.val[e];
                    if (!(std::fabs(v - prod) <= 1e-6f * std::fabs(v))) {
                        set_error("a stored value is not row_scale[i] * col_scale[j]");
                        return AG_ERR_INVALID;
                    }
                }
            t->factored = true;
        }
        t->opt.row_scale = t->opt.col_scale = nullptr;        // borrowed pointers are not kept
        t->opt.reuse_perm = t->opt.reuse_blk_ptr = nullptr;
        double t2 = now_sec();
        t->sec_split = t2 - t1;
        // density classes (decided on the forward matrix; the transpose has the same counts)
        const HostCsr &I = t->h[0].intra;
        for (int32_t b = 0; b < t->r.n_blocks; ++b) {
            const int32_t r0 = t->r.blk_ptr[b], r1 = t->r.blk_ptr[b + 1];
            const double sz = r1 - r0, cnt = I.rowptr[r1] - I.rowptr[r0];
            t->all_blocks.push_back(b);
            // the dense kernels take blocks of 32 to 128 rows (four wavefronts of 32 rows, 128-bit row maps)
            if (cnt >= o.dense_density * sz * sz && sz >= 32 && sz <= kMaxBlock) t->dense_blocks.push_back(b);
            else t->sparse_blocks.push_back(b);
        }
        const int ndir = t->symmetric ? 1 : 2;
        for (int k = 0; k < ndir; ++k) {
            build_segments(t->h[k].full, t->h[k].segs_full);
            build_segments(t->h[k].inter, t->h[k].segs_inter);
            build_block_formats(t->r, t->dense_blocks, t->unit || t->factored, t->h[k]);
        }
        double t3 = now_sec();
        t->sec_build = t3 - t2;
        if (!t->host_only) {
            const int32_t *bp = nullptr, *ld = nullptr, *ls = nullptr, *la = nullptr;
            if ((rc = t->upload(t->r.blk_ptr, bp))) return rc;
            if ((rc = t->upload(t->dense_blocks, ld))) return rc;
            if ((rc = t->upload(t->sparse_blocks, ls))) return rc;
            if ((rc = t->upload(t->all_blocks, la))) return rc;
            if ((rc = t->upload(t->r.perm, t->perm_dev))) return rc;
            if (!t->rs_plan.empty()) { if ((rc = t->upload(t->rs_plan, t->rs_dev))) return rc; }
            if (!t->cs_plan.empty()) { if ((rc = t->upload(t->cs_plan, t->cs_dev))) return rc; }
            for (int k = 0; k < ndir; ++k)
                if ((rc = t->upload_dir(k, bp, ld, ls, la))) return rc;
            if ((rc = hip_fail((int)hipDeviceSynchronize(), "upload sync"))) return rc;
        }
        t->sec_upload = now_sec() - t3;
        auto *p = new ag_plan();
        p->topo = t;
        p->F = F;
        p->layout = o.layout;
        p->trials = o.trials;
        init_selector(p, 0, false);
        init_selector(p, 1, false);
        if ((rc = plan_device_buffers(p))) { delete p; return rc; }
        *out = p;
        return AG_OK;
    } catch (const std::bad_alloc &) {
        set_error("host allocation failed");
        return AG_ERR_NOMEM;
    } catch (const std::exception &e) {
        set_error(std::string("internal error: ") + e.what());
        return AG_ERR_INVALID;
    }
}

int ag_plan_clone_for_width(const ag_plan *p, int32_t F2, ag_plan **out)
{
    if (!p || !out || F2 < 1) { set_error("bad argument"); return AG_ERR_INVALID; }
    *out = nullptr;
    auto *q = new (std::nothrow) ag_plan();
    if (!q) { set_error("host allocation failed"); return AG_ERR_NOMEM; }
    try {
        q->topo = p->topo;
        q->F = F2;
        q->layout = p->layout;
        q->trials = p->trials;
        init_selector(q, 0, false);
        init_selector(q, 1, false);
        int rc = plan_device_buffers(q);
        if (rc) { delete q; return rc; }
    } catch (const std::bad_alloc &) {
        delete q;
        set_error("host allocation failed");
        return AG_ERR_NOMEM;
    }
    *out = q;
    return AG_OK;
}

void ag_plan_destroy(ag_plan *p) { delete p; }

int ag_aggregate(ag_plan *p, const float *H, float *Y, void *stream)
{
    return aggregate_dir(p, AG_DIR_FWD, H, Y, stream);
}

int ag_aggregate_t(ag_plan *p, const float *G, float *dH, void *stream)
{
    return aggregate_dir(p, AG_DIR_BWD, G, dH, stream);
}

int ag_permute_rows(const ag_plan *p, const float *src, float *dst, int32_t F, int32_t inverse, void *stream)
{
    if (!p || !src || !dst || F < 1 || src == dst) { set_error("bad argument"); return AG_ERR_INVALID; }
    if (p->topo->host_only) { set_error("host-only plan"); return AG_ERR_UNSUPPORTED; }
    if ((((uintptr_t)src | (uintptr_t)dst) & 15)) {
        set_error("feature matrices must be 16-byte aligned");
        return AG_ERR_INVALID;
    }
    return launch_permute_rows(p->topo->perm_dev, p->topo->n, F, src, dst, inverse != 0, stream);
}

int ag_plan_force_kernels(ag_plan *p, int32_t cls, int32_t dir, int32_t kernel_id)
{
    if (!p || cls < 0 || cls >= AG_NUM_CLS || (dir != AG_DIR_FWD && dir != AG_DIR_BWD)) {
        set_error("bad class or direction");
        return AG_ERR_INVALID;
    }
    static const int limit[AG_NUM_CLS] = {3, 1, 3, 4};
    if (kernel_id < -1 || kernel_id >= 4) { set_error("kernel id out of range"); return AG_ERR_INVALID; }
    if (kernel_id >= limit[cls]) { set_error("kernel id not available for this class"); return AG_ERR_UNSUPPORTED; }
    if (cls == AG_CLS_BLOCKS_DENSE && kernel_id == AG_K_BLOCK_DENSE_BF16X3 && !p->topo->unit && !p->topo->factored) {
        set_error("the bf16x3 dense kernel takes unit-weight or factored matrices only");
        return AG_ERR_UNSUPPORTED;
    }
    Selector &s = p->sel[dir];
    const int keep[AG_NUM_CLS] = {s.forced[0], s.forced[1], s.forced[2], s.forced[3]};
    init_selector(p, dir, false);
    for (int c = 0; c < AG_NUM_CLS; ++c) s.forced[c] = keep[c];
    s.forced[cls] = kernel_id;
    return AG_OK;
}

int ag_plan_selector_info(const ag_plan *p, int32_t dir, ag_selector_info *out)
{
    if (!p || !out || (dir != AG_DIR_FWD && dir != AG_DIR_BWD)) { set_error("bad argument"); return AG_ERR_INVALID; }
    const Selector &s = p->sel[dir];
    out->frozen = s.phase == 2;
    out->calls = s.calls;
    for (int c = 0; c < AG_NUM_CLS; ++c) {
        out->choice[c] = s.choice[c];
        for (int k = 0; k < 4; ++k) out->trial_ms[c][k] = s.median_ms[c][k];
    }
    out->total_trial_ms = s.total_trial_ms;
    return AG_OK;
}

int ag_plan_set_profiling(ag_plan *p, int32_t on)
{
    if (!p) { set_error("null plan"); return AG_ERR_INVALID; }
    if (p->topo->host_only) { set_error("host-only plan"); return AG_ERR_UNSUPPORTED; }
    prof_drain(p);
    for (int d = 0; d < 2; ++d) {
        p->prof_total[d] = 0;
        p->prof_calls[d] = 0;
        for (int c = 0; c < 3; ++c) p->prof_ms[d][c] = 0;
    }
    if (on && p->prof_ev.empty()) {
        try {
            p->prof_pending.reserve(kProfRing);           // later calls push without allocating
            p->prof_ev.assign(4 * kProfRing, nullptr);
        } catch (const std::bad_alloc &) {
            p->prof_ev.clear();
            set_error("host allocation failed");
            return AG_ERR_NOMEM;
        }
        for (auto &e : p->prof_ev) {
            int rc = hip_fail((int)hipEventCreate(&e), "event create");
            if (rc) return rc;
        }
    }
    p->profiling = on != 0;
    return AG_OK;
}

int ag_plan_profile(ag_plan *p, int32_t dir, ag_profile *out)
{
    if (!p || !out || (dir != AG_DIR_FWD && dir != AG_DIR_BWD)) { set_error("bad argument"); return AG_ERR_INVALID; }
    prof_drain(p);
    out->calls = p->prof_calls[dir];
    for (int c = 0; c < 3; ++c) out->class_ms[c] = p->prof_ms[dir][c];
    out->total_ms = p->prof_total[dir];
    out->compose = p->sel[dir].choice[AG_CLS_COMPOSE];
    return AG_OK;
}

int ag_plan_export(const ag_plan *p, ag_export *out)
{
    if (!p || !out) { set_error("bad argument"); return AG_ERR_INVALID; }
    const Topology &t = *p->topo;
    const HostDir &h = t.h[0];
    out->n = t.n;
    out->nnz_intra = h.intra.nnz();
    out->nnz_inter = h.inter.nnz();
    out->n_blocks = t.r.n_blocks;
    out->perm = t.r.perm.data();
    out->iperm = t.r.iperm.data();
    out->blk_ptr = t.r.blk_ptr.data();
    out->intra_rowptr = h.intra.rowptr.data();
    out->intra_col = h.intra.col.data();
    out->intra_val = t.unit ? nullptr : h.intra.val.data();
    out->inter_rowptr = h.inter.rowptr.data();
    out->inter_col = h.inter.col.data();
    out->inter_val = t.unit ? nullptr : h.inter.val.data();
    return AG_OK;
}

int ag_plan_stats(const ag_plan *p, ag_stats *out)
{
    if (!p || !out) { set_error("bad argument"); return AG_ERR_INVALID; }
    const Topology &t = *p->topo;
    std::memset(out, 0, sizeof(*out));
    out->n = t.n;
    out->nnz = t.nnz;
    out->nnz_intra = t.h[0].intra.nnz();
    out->nnz_inter = t.h[0].inter.nnz();
    out->F = p->F;
    out->n_blocks = t.r.n_blocks;
    out->n_block_rows = t.r.blk_ptr.back();
    out->n_dense_blocks = (int32_t)t.dense_blocks.size();
    out->symmetric = t.symmetric;
    out->unit_weights = t.unit;
    out->n_long_rows = (int64_t)t.h[0].segs_inter.lr_row.size();
    out->n_long_segments = (int64_t)t.h[0].segs_inter.seg_row.size();
    const double nn = (double)t.n * (double)t.n;
    double blk_area = 0;
    const HostCsr &I = t.h[0].intra;
    for (int32_t b = 0; b < t.r.n_blocks; ++b) {
        const int32_t r0 = t.r.blk_ptr[b], r1 = t.r.blk_ptr[b + 1];
        const double s = r1 - r0, d = (I.rowptr[r1] - I.rowptr[r0]) / (s * s);
        blk_area += s * s;
        out->block_density_hist[std::min(7, (int)(d * 8.0))]++;
    }
    const HostCsr &O = t.h[0].inter;
    for (int32_t b : t.dense_blocks) {
        const int32_t r0 = t.r.blk_ptr[b], r1 = t.r.blk_ptr[b + 1];
        out->dense_rows += r1 - r0;
        out->nnz_intra_dense += I.rowptr[r1] - I.rowptr[r0];
        out->nnz_inter_dense_rows += O.rowptr[r1] - O.rowptr[r0];
    }
    out->nnz_inter_block_rows = O.rowptr[out->n_block_rows];
    out->factored = t.factored;
    out->density_full = nn > 0 ? (double)t.nnz / nn : 0;
    out->density_intra = blk_area > 0 ? (double)out->nnz_intra / blk_area : 0;
    out->density_inter = nn - blk_area > 0 ? (double)out->nnz_inter / (nn - blk_area) : 0;
    out->sec_reorder = t.sec_reorder;
    out->sec_split = t.sec_split;
    out->sec_build = t.sec_build;
    out->sec_upload = t.sec_upload;
    out->device_bytes = t.device_bytes;
    return AG_OK;
}

namespace {
int max_checks(ag_plan *p, const void *a, const void *b, const void *c)
{
    if (!p) { set_error("null plan"); return AG_ERR_INVALID; }
    const Topology &t = *p->topo;
    if (t.host_only) { set_error("plan was created with AG_FLAG_HOST_ONLY"); return AG_ERR_UNSUPPORTED; }
    if (p->layout != AG_LAYOUT_REORDERED) {
        set_error("the max aggregator needs an AG_LAYOUT_REORDERED plan");
        return AG_ERR_UNSUPPORTED;
    }
    if (t.n == 0) return AG_OK;
    if (!a || !b) { set_error("null argument"); return AG_ERR_INVALID; }
    if (a == b) { set_error("input and output must not alias"); return AG_ERR_INVALID; }
    if ((((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 15)) {
        set_error("matrices must be 16-byte aligned");
        return AG_ERR_INVALID;
    }
    return AG_OK;
}
}  // namespace

int ag_aggregate_max(ag_plan *p, const float *H, float *Y, int32_t *arg, void *stream)
{
    int rc = max_checks(p, H, Y, arg);
    if (rc || p->topo->n == 0) return rc;
    return launch_csr_max(p->topo->d[0].full, H, Y, arg, p->F, stream);
}

int ag_aggregate_max_t(ag_plan *p, const float *G, const int32_t *arg, float *dH, void *stream)
{
    int rc = max_checks(p, G, dH, arg);
    if (rc || p->topo->n == 0) return rc;
    if (!arg) { set_error("null argument"); return AG_ERR_INVALID; }
    const Topology &t = *p->topo;
    return launch_csr_max_t(t.d[t.symmetric ? 0 : 1].full, G, arg, dH, p->F, stream);
}

int ag_gin_layer(ag_plan *p, float eps, const float *H, float *Y, void *stream)
{
    int rc = aggregate_dir(p, AG_DIR_FWD, H, Y, stream);
    if (rc || eps == 0.f) return rc;
    return launch_axpy(p->topo->n * (int64_t)p->F, eps, H, Y, stream);
}

int ag_gin_layer_t(ag_plan *p, float eps, const float *G, float *dH, void *stream)
{
    int rc = aggregate_dir(p, AG_DIR_BWD, G, dH, stream);
    if (rc || eps == 0.f) return rc;
    return launch_axpy(p->topo->n * (int64_t)p->F, eps, G, dH, stream);
}

}  // extern "C"

// accessors for gcn.cpp
namespace ag {
int64_t plan_n(const ag_plan *p) { return p->topo->n; }
int32_t plan_f(const ag_plan *p) { return p->F; }
int32_t plan_layout(const ag_plan *p) { return p->layout; }
bool plan_same_topology(const ag_plan *a, const ag_plan *b) { return a->topo == b->topo; }
bool plan_host_only(const ag_plan *p) { return p->topo->host_only; }
}  // namespace ag
