/*
 * adaptgear.h -- C ABI of the MI355X (gfx950) neighbour-aggregation library.
 *
 * The library implements the hot path of AdaptGear (arXiv 2305.17408): the
 * GNN aggregate-sum operator  Y = A.H  and its backward  dH = A^T.G  in fp32,
 * where A is an N x N sparse (normalised) adjacency matrix whose rows are
 * destination vertices and whose columns are source vertices (paper Sec. 2.1,
 * "Graph Format"), and H is a dense row-major N x F feature matrix.
 *
 * Following the paper's design (Sec. 3), a plan reorders the vertices by
 * communities once on the CPU, decomposes the matrix into an intra-community
 * subgraph (diagonal blocks) and an inter-community subgraph (the remainder),
 * runs each with a kernel suited to its density (Sec. 3.2), and picks the
 * kernel set by timing the candidates during the first calls (Sec. 3.3).
 *
 * Conventions
 *   - every function returns AG_OK (0) or a negative AG_ERR_* code and never
 *     aborts; ag_last_error() gives a thread-local message for the last error;
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the current device, fp32 row-major, 16-byte aligned;
 *   - a plan owns its device topology; feature matrices stay owned by the caller;
 *   - work is enqueued on the caller's HIP stream and the call returns without
 *     waiting, except during the selector's trial calls (which read events);
 *   - calls on one plan (and on its clones) must not overlap in time: they
 *     share scratch memory for partial sums of very long rows.
 */
#ifndef ADAPTGEAR_H
#define ADAPTGEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AG_OK               0
#define AG_ERR_INVALID     -1   /* bad argument or malformed matrix            */
#define AG_ERR_NOMEM       -2   /* host or device allocation failed            */
#define AG_ERR_HIP         -3   /* a HIP runtime call failed                   */
#define AG_ERR_UNSUPPORTED -4   /* valid request this build cannot serve       */

typedef struct ag_plan ag_plan;   /* opaque */

/* Sparse matrix in CSR form, HOST memory, borrowed only during ag_plan_create.
 * rowptr is monotone with rowptr[0] = 0 and rowptr[n] = nnz; column indices lie in
 * [0, n); rows may be unsorted (they are sorted); a repeated (row, col) pair is an
 * error.  vals == NULL means unit weights (the weight-free sum of Algorithm 1). */
typedef struct {
    int64_t        n;
    int64_t        nnz;
    const int32_t *rowptr;   /* n + 1 */
    const int32_t *colidx;   /* nnz, source vertex of each entry */
    const float   *vals;     /* nnz or NULL */
} ag_csr;

/* vertex order of the feature matrices passed to ag_aggregate* */
#define AG_LAYOUT_ORIGINAL  0   /* caller's numbering; the library permutes in and out   */
#define AG_LAYOUT_REORDERED 1   /* rows already in plan order (see ag_permute_rows)      */

/* community detection behind the reordering (Sec. 2.2, Sec. 4.2 stage 1) */
#define AG_METHOD_LABEL_PROPAGATION 0  /* multilevel size-constrained label propagation (default)  */
#define AG_METHOD_MODULARITY        1  /* one pass of size-constrained agglomeration, vertices in  *
                                        * ascending degree, each joining the neighbouring community *
                                        * with the largest integer modularity gain                  *
                                        * conn * 2m - deg_u * deg_v                                 */

#define AG_FLAG_HOST_ONLY   1   /* build the decomposition on the host only: no device   *
                                 * memory, ag_aggregate* return AG_ERR_UNSUPPORTED       */

/* All fields optional: zero selects the default. */
typedef struct {
    int32_t block_cap;      /* largest community / diagonal block, 1..256 (default 128; the   *
                             * paper used 16, Sec. 2.3).  Blocks of more than 128 rows always  *
                             * run the block-sparse kernel, with a larger LDS tile             */
    int32_t num_communities;/* alternative to block_cap (Sec. 4.2 lets the user give either the   *
                             * size or the number): if > 0 and block_cap == 0, the cap becomes     *
                             * min(256, ceil(n / num_communities))                                */
    int32_t min_block;      /* communities smaller than this go to the block-less tail (16, or   *
                             * the cap if that is smaller)                                        */
    int32_t sweeps;         /* label-propagation sweeps per level (8)                          */
    int32_t max_levels;     /* coarsening levels (12)                                          */
    int32_t order_levels;   /* extra levels that only order the communities so that connected   *
                             * ones are adjacent (3; negative = plain ascending-id order)         */
    int32_t trials;         /* timed runs per candidate in the selector (3; at most 15)        */
    int32_t layout;         /* AG_LAYOUT_*                                                     */
    int32_t flags;          /* AG_FLAG_*                                                       */
    float   dense_density;  /* blocks at least this dense may use the dense kernels (0.20;      *
                             * 0.05 for unit-weight matrices, which have the bf16 form)        */
    void *(*dev_alloc)(size_t bytes, void *user);   /* default hipMalloc                       */
    void  (*dev_free)(void *ptr, void *user);       /* default hipFree                         */
    void   *user;
    /* Factored values (optional, host arrays of n floats, borrowed during ag_plan_create): a     *
     * declaration that vals[i][j] = row_scale[i] * col_scale[j] up to fp32 rounding, a missing   *
     * array counting as all ones: D^-1/2 on both sides for the GCN normalisation, D^-1 as        *
     * row_scale for aggregate-mean (Sec. 2.1).  The diagonal blocks then run value-free: the     *
     * pattern kernels (the bit-map dense kernels of Sec. 3.2 included) with col_scale applied to  *
     * the feature rows on the way in and row_scale to the sums on the way out; the remainder     *
     * keeps the stored values.  Needs vals; AG_ERR_INVALID if an intra-community value departs   *
     * from the product by more than 1e-6 relative.                                               */
    const float *row_scale, *col_scale;
    int32_t method;         /* community detection of the reordering, AG_METHOD_* (Sec. 4.2: the        *
                             * partitioner is the user's choice; Sec. 6.1 compares two)                  */
    /* A reordering computed earlier (host arrays, borrowed during ag_plan_create): the perm and    *
     * blk_ptr of an ag_plan_export of a plan of the same matrix, or the output of a partitioner of  *
     * the caller's own (Sec. 4.2: the preprocessing is paid once per graph and reused across       *
     * trainings).  reuse_perm[new] = old is a permutation of 0..n-1; reuse_blk_ptr has              *
     * reuse_n_blocks + 1 ascending entries from 0 to at most n, every block of 1..256 rows; rows    *
     * from the last entry on are the block-less tail.  When reuse_perm is given the community      *
     * detection is skipped (block_cap, min_block, sweeps, max_levels, order_levels and method are   *
     * then unused); anything else about the arrays is AG_ERR_INVALID.                               */
    const int32_t *reuse_perm, *reuse_blk_ptr;
    int32_t reuse_n_blocks;
} ag_options;

/* ---- plan life cycle -------------------------------------------------------------------- */

/* Reorder (Sec. 2.2, Sec. 4.2 stage 1), decompose (Sec. 3.3, Sec. 4.2 stage 2), build the
 * per-kernel formats and upload them.  `N` must equal A->n; `F` (>= 1) is the feature width
 * the plan will be called with.  On success *out receives a new plan. */
int ag_plan_create(const ag_csr *A, int64_t N, int32_t F, const ag_options *opt, ag_plan **out);

/* A second plan for feature width F2 that shares the topology (host and device) of `p`: the
 * layers of a model have different widths but one graph (Sec. 4.1: the decomposed subgraphs are
 * passed to every layer), and the kernel choice depends on the width, so each width has its own
 * selector state (Sec. 3.3).  Destroy both; the topology goes with the last one. */
int ag_plan_clone_for_width(const ag_plan *p, int32_t F2, ag_plan **out);

void ag_plan_destroy(ag_plan *p);

/* ---- the hot path ----------------------------------------------------------------------- */

/* Y = A.H (aggregate-sum of Sec. 2.1 with an edge value).  H, Y: device, N x F, Y is
 * overwritten and must not alias H.
 * Finite inputs: the sparse kernels touch stored entries only (an Inf or NaN feature reaches
 * exactly the rows that reference it), but the dense kernels AG_K_BLOCK_DENSE* multiply the
 * non-neighbours of a block by zero, so one non-finite feature row turns every row of its
 * diagonal block into NaN.  Which kernel runs is the selector's timing decision: with non-finite
 * features pin AG_CLS_BLOCKS_DENSE to AG_K_BLOCK_SPARSE (ag_plan_force_kernels), or the result
 * for the rows of that block is unspecified. */
int ag_aggregate(ag_plan *p, const float *H_dev, float *Y_dev, void *hip_stream);

/* dH = A^T.G, the backward of ag_aggregate (training, Sec. 5 "Benchmarks"). */
int ag_aggregate_t(ag_plan *p, const float *G_dev, float *dH_dev, void *hip_stream);

/* ag_aggregate for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels and the same result, but the scratch
 * memory of the long-row kernels (partial sums of row segments) is a static device array of
 * AG_STATIC_SCRATCH_BYTES per GPU instead of plan-owned memory, and the call allocates nothing on
 * the host or the device and creates no events.
 *   - the kernel choice must be settled: the forward selector has frozen (ag_plan_selector_info),
 *     or all four classes are pinned with ag_plan_force_kernels; otherwise AG_ERR_UNSUPPORTED
 *     (a selector trial would need events);
 *   - the plan's long-row segments times F floats must fit the static array; otherwise
 *     AG_ERR_UNSUPPORTED with the sizes in ag_last_error();
 *   - all calls on one GPU share that GPU's array (whatever the plan): calls that overlap in time
 *     on one GPU race, also across streams and plans.  Nothing in it has to start at zero. */
#define AG_STATIC_SCRATCH_BYTES (32u << 20)
int ag_aggregate_static(ag_plan *p, const float *H_dev, float *Y_dev, void *hip_stream);

/* The paper reorders the data set once in preprocessing (Sec. 4.2, first stage): this applies the
 * plan's vertex order to a feature matrix.  dst[new] = src[perm[new]] (inverse == 0: caller order
 * -> plan order) or dst[perm[new]] = src[new] (inverse != 0).  N x F device matrices, no aliasing. */
int ag_permute_rows(const ag_plan *p, const float *src_dev, float *dst_dev, int32_t F,
                    int32_t inverse, void *hip_stream);

/* ---- kernel selection (Sec. 3.3 "Adaptive Selector") ------------------------------------ */

/* subgraph classes */
#define AG_CLS_BLOCKS_DENSE   0   /* diagonal blocks with density >= dense_density          */
#define AG_CLS_BLOCKS_SPARSE  1   /* all other diagonal blocks                               */
#define AG_CLS_REMAINDER      2   /* inter-community subgraph (+ tail rows)                  */
#define AG_CLS_COMPOSE        3   /* how the pieces are combined                             */
#define AG_NUM_CLS            4

/* kernels for the two block classes */
#define AG_K_BLOCK_SPARSE     0   /* block CSR with features staged in LDS (Sec. 3.2, CSR intra) */
#define AG_K_BLOCK_DENSE      1   /* dense tile on fp32 MFMA (Sec. 3.2, dense-based kernel);      *
                                   * finite features only, see ag_aggregate                        */
#define AG_K_BLOCK_DENSE_BF16X3 2 /* the same on bf16 MFMA at fp32 accuracy: features cut into     *
                                   * three bf16 pieces that sum to them exactly; unit-weight        *
                                   * or factored matrices only (AG_ERR_UNSUPPORTED otherwise)       */
/* kernels for the remainder: lanes cooperating on one row */
#define AG_K_CSR_NARROW       0   /* one feature-wide lane group per row (Sec. 3.2, CSR inter)    */
#define AG_K_CSR_WIDE         1   /* several lane groups per row, neighbours interleaved          */
#define AG_K_COO              2   /* edge-parallel with fp32 atomics (Algorithm 1 + edge value);  *
                                   * summation order varies between runs; used in AG_COMPOSE_SPLIT *
                                   * only (the other compositions fall back to AG_K_CSR_NARROW)    */
/* compositions */
#define AG_COMPOSE_SPLIT      0   /* block kernels write Y, the remainder kernel accumulates      */
#define AG_COMPOSE_FUSED      1   /* the block kernels also add their rows' remainder entries and *
                                   * store each row once.  The dense class runs its own (dense)   *
                                   * kernel here only if that kernel was chosen for it and the    *
                                   * class has at least AG_MIN_BLOCKS_OWN_LAUNCH blocks; otherwise *
                                   * all blocks go through the sparse-block kernel in one launch  */
#define AG_MIN_BLOCKS_OWN_LAUNCH 256
#define AG_COMPOSE_FULL_CSR   2   /* no decomposition at run time: one CSR over the whole matrix, *
                                   * one lane group per row                                       */
#define AG_COMPOSE_FULL_CSR_WIDE 3 /* the same with several lane groups per row                   */

#define AG_DIR_FWD 0
#define AG_DIR_BWD 1

/* Pin the kernel of class `cls` for direction `dir`; kernel_id = -1 returns the class to the
 * adaptive selector (and restarts its trials). */
int ag_plan_force_kernels(ag_plan *p, int32_t cls, int32_t dir, int32_t kernel_id);

typedef struct {
    int32_t frozen;                 /* 1 once the trials are over                              */
    int32_t calls;                  /* calls seen for this direction                           */
    int32_t choice[AG_NUM_CLS];     /* current kernel id per class                             */
    float   trial_ms[AG_NUM_CLS][4];/* median time of each candidate (ms), <0 = not measured   */
    float   total_trial_ms;         /* wall time spent inside trial calls                      */
} ag_selector_info;

int ag_plan_selector_info(const ag_plan *p, int32_t dir, ag_selector_info *out);

/* Per-kernel timing of ordinary (non-trial) calls, the "monitor" of Sec. 3.3 kept available
 * after the trials: while switched on, every call records HIP events on the caller's stream
 * around its subgraph kernels.  ag_plan_profile waits for the recorded events and returns the
 * sums since profiling was switched on.  With AG_COMPOSE_SPLIT class_ms[0..2] are the dense-
 * class block kernel, the sparse-class block kernel and the remainder kernels; with
 * AG_COMPOSE_FUSED class_ms[0] is the fused block kernel (all blocks, or the dense class when it
 * runs its own kernel, then class_ms[1] is the fused kernel of the sparse class) and class_ms[2]
 * the tail/long-row kernels; with the one-CSR compositions everything is in class_ms[2]. */
typedef struct {
    int64_t calls;
    double  class_ms[3];
    double  total_ms;
    int32_t compose;
} ag_profile;

int ag_plan_set_profiling(ag_plan *p, int32_t on);
int ag_plan_profile(ag_plan *p, int32_t dir, ag_profile *out);

/* ---- inspection (tests, reports) -------------------------------------------------------- */

/* Host views of the decomposition (Sec. 3.3 / Sec. 4.2: the reordering and the intra- and
 * inter-community subgraphs), owned by the plan, valid until it is destroyed.
 * perm[new] = old, iperm[old] = new; diagonal block b covers plan rows
 * [blk_ptr[b], blk_ptr[b+1]); rows from blk_ptr[n_blocks] on are the tail.  The two CSR
 * parts are in plan numbering, columns ascending, values carried over unchanged. */
typedef struct {
    int64_t n, nnz_intra, nnz_inter;
    int32_t n_blocks;
    const int32_t *perm, *iperm, *blk_ptr;
    const int32_t *intra_rowptr, *intra_col; const float *intra_val;   /* val NULL if unit */
    const int32_t *inter_rowptr, *inter_col; const float *inter_val;
} ag_export;

int ag_plan_export(const ag_plan *p, ag_export *out);

typedef struct {
    int64_t n, nnz, nnz_intra, nnz_inter;
    int32_t F, n_blocks, n_block_rows, n_dense_blocks, symmetric, unit_weights;
    int64_t n_long_rows, n_long_segments;      /* remainder rows split across wavefronts     */
    double  density_full, density_intra, density_inter;  /* cf. the paper's density figure   */
    double  sec_reorder, sec_split, sec_build, sec_upload;
    int64_t device_bytes;                      /* topology held on the device                */
    int32_t block_density_hist[8];             /* diagonal blocks with density in [k/8, (k+1)/8) */
    /* the dense class on its own (forward direction): its rows, its intra-community entries and *
     * the remainder entries of its rows; and the remainder entries of all block rows            */
    int64_t dense_rows, nnz_intra_dense, nnz_inter_dense_rows, nnz_inter_block_rows;
    int32_t factored;                          /* row_scale / col_scale in use (value-free blocks) */
} ag_stats;

int ag_plan_stats(const ag_plan *p, ag_stats *out);

const char *ag_last_error(void);

/* Aggregate-max (Sec. 2.1: sum, mean and max are the Aggregate choices; aggregate-mean is the sum
 * with row-normalised edge values).  Edge values are ignored.
 *   Y[i][k]   = max over the stored entries (i, j) of H[j][k]; rows without entries give 0
 *   arg[i][k] = the source j that attains it, in plan numbering (-1 for rows without entries;
 *               the smallest j among equal values); device int32 N x F, may be NULL
 *   dH[j][k]  = sum of G[i][k] over the rows i with arg[i][k] == j   (ag_aggregate_max_t)
 * AG_LAYOUT_REORDERED plans only (AG_ERR_UNSUPPORTED otherwise); matrices device row-major
 * N x F in plan order, 16-byte aligned; NaN inputs are not supported.  One kernel over the whole
 * reordered matrix; the selector plays no part.  Results are bitwise reproducible. */
int ag_aggregate_max  (ag_plan *p, const float *H_dev, float *Y_dev, int32_t *arg_dev, void *hip_stream);
int ag_aggregate_max_t(ag_plan *p, const float *G_dev, const int32_t *arg_dev, float *dH_dev, void *hip_stream);

/* ---- model-step drivers ----------------------------------------------------------------- */

/* GIN sum aggregation (Sec. 2.1 aggregate-sum, Sec. 5): Y = A.H + eps*H, where the stored
 * pattern already holds the unit diagonal ((1+eps) self term); ag_gin_layer_t is its backward. */
int ag_gin_layer  (ag_plan *p, float eps, const float *H_dev, float *Y_dev, void *hip_stream);
int ag_gin_layer_t(ag_plan *p, float eps, const float *G_dev, float *dH_dev, void *hip_stream);

/* Two-layer GCN training step (Sec. 5 "Benchmarks"), forward + backward, no optimiser update:
 *   P = A.X; H1 = relu(P W1 + b1); Q = H1 W2; Z = A.Q + b2; loss = mean softmax-CE(Z, labels)
 *   dZ; dQ = A^T dZ; dW2 = H1^T dQ; db2; dH1 = dQ W2^T; dPre = dH1 * (H1 > 0); dW1 = P^T dPre; db1
 * All matrices device fp32 row-major in PLAN order (AG_LAYOUT_REORDERED plans only).
 * p_in is a plan of width f_in, p_out one of width n_class (clones of one topology).
 * The workspace is caller-provided device memory of at least ag_gcn_workspace_bytes(). */
typedef struct {
    int32_t f_in, hidden, n_class;
    const float *W1, *b1, *W2, *b2;        /* device: f_in x hidden, hidden, hidden x n_class, n_class */
    float *dW1, *db1, *dW2, *db2;          /* device outputs, same shapes                              */
    float *loss;                           /* device, 1 float                                          */
    float *logits;                         /* device N x n_class output (Z), may be NULL               */
} ag_gcn_io;

size_t ag_gcn_workspace_bytes(int64_t n, int32_t f_in, int32_t hidden, int32_t n_class);
int ag_gcn_step(ag_plan *p_in, ag_plan *p_out, const ag_gcn_io *io, const float *X_dev,
                const int32_t *labels_dev, void *workspace_dev, size_t workspace_bytes,
                void *hip_stream);

/* L-layer GIN training step (Sec. 5 "Benchmarks": GIN; Sec. 2.1 aggregate-sum + Update), forward +
 * backward, no optimiser update.  With H_0 = X and width[0..L] the feature widths:
 *   A_l = A.H_l + eps*H_l                      (the stored pattern carries the unit diagonal)
 *   H_{l+1} = relu(A_l W_l + b_l)  for l < L-1;   Z = A_{L-1} W_{L-1} + b_{L-1}
 *   loss = mean softmax-CE(Z, labels);  gradients dW_l, db_l of every layer.
 * The last layer is evaluated as A.(H W) when that is the narrower aggregation; backward
 * aggregations run at the layer's output width ((A^T dPre) W^T = A^T (dPre W^T)).
 * plans[l], l = 0..L, are AG_LAYOUT_REORDERED plans of ONE topology (ag_plan_clone_for_width) with
 * F = width[l]; equal widths may share one plan.  All matrices are device fp32 row-major in plan
 * order, 16-byte aligned; W[l] is width[l] x width[l+1].  Returns AG_ERR_INVALID on mismatching
 * widths / plans / workspace size, AG_ERR_UNSUPPORTED for host-only or caller-order plans. */
#define AG_GIN_MAX_LAYERS 8
typedef struct {
    int32_t n_layers;                          /* L, 1..AG_GIN_MAX_LAYERS                          */
    int32_t width[AG_GIN_MAX_LAYERS + 1];      /* width[0] inputs ... width[L] classes             */
    float   eps;
    const float *W[AG_GIN_MAX_LAYERS], *b[AG_GIN_MAX_LAYERS];     /* device parameters             */
    float *dW[AG_GIN_MAX_LAYERS], *db[AG_GIN_MAX_LAYERS];         /* device outputs, same shapes   */
    float *loss;                               /* device, 1 float                                  */
    float *logits;                             /* device N x width[L] output (Z), may be NULL      */
} ag_gin_io;

size_t ag_gin_workspace_bytes(int64_t n, const ag_gin_io *io);
int ag_gin_step(ag_plan *const *plans, const ag_gin_io *io, const float *X_dev, const int32_t *labels_dev,
                void *workspace_dev, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ADAPTGEAR_H */
