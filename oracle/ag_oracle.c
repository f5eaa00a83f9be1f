/*
 * CPU oracle for the AdaptGear aggregation path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 reference code written from the paper.  Nothing in the
 * product (the HIP library or its Python binding) may include, link or call
 * this file; only the tests, the smoke check and the bench's CPU-baseline leg
 * use it.  It shares no code with the HIP path.
 *
 * What it defines
 *   orc_spmm        Y = A.H        aggregate-sum of neighbour features (paper
 *                                  Sec. 2.1, the Aggregate equation; CSR rows
 *                                  are destinations, columns are sources,
 *                                  Sec. 2.1 "Graph Format"), with an optional
 *                                  edge value a_ij, plus the abs-sum
 *                                  S = sum_j |a_ij h_jk| used by the tolerance.
 *   orc_spmm_t      dH = A^T.G     the adjoint, needed for training (Sec. 5
 *                                  "Benchmarks": end-to-end training).
 *   orc_coo_sum     Algorithm 1 (edge list, Y[dst] += X[src]) run serially.
 *   orc_spmax       aggregate-max (Sec. 2.1 lists sum, mean and max as the
 *                   Aggregate choices): Y[i][k] = max over the stored entries
 *                   (i, j) of H[j][k], with the smallest such j as the argmax;
 *                   rows without entries give 0 and argmax -1.
 *   orc_spmax_t     its adjoint for training: every G[i][k] goes to the source
 *                   vertex that attained the maximum.
 *   orc_reorder     community reordering (Sec. 2.2 / Sec. 4.2 first stage).
 *                   The paper delegates this to an external partitioner; the
 *                   reading used here is a multilevel, size-constrained label
 *                   propagation in pure integer arithmetic (spelled out at the
 *                   function).
 *   orc_reorder_method  the same with a choice of the community detection:
 *                   0 = the label propagation above, 1 = one pass of size-constrained
 *                   agglomeration by the integer modularity gain (spelled out at
 *                   agglomerate_by_gain); ordering levels and layout are shared.
 *   orc_split       decomposition into intra- / inter-community subgraphs
 *                   (Sec. 3.3 first paragraphs, Sec. 4.2 second stage).
 *
 * Parity status: every function here is pinned by tests that do not go through
 * this file (dense brute force, closed forms, scipy CSR product, adjoint
 * identity, hand-traced reorder examples, partition invariants).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef int32_t i32;
typedef int64_t i64;

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* Y[i][k] = sum_{e in row i} a_e * H[col_e][k]                               */
/* ------------------------------------------------------------------------ */
void orc_spmm(i64 n, const i32 *rowptr, const i32 *col, const float *vals, i32 F,
              const float *H, double *Y, double *S, i32 use_threads)
{
    i64 i;
#pragma omp parallel for schedule(dynamic, 256) if (use_threads)
    for (i = 0; i < n; ++i) {
        double *y = Y + i * F;
        double *s = S ? S + i * F : 0;
        for (i32 k = 0; k < F; ++k) y[k] = 0.0;
        if (s) for (i32 k = 0; k < F; ++k) s[k] = 0.0;
        for (i32 e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            double a = vals ? (double)vals[e] : 1.0;
            const float *h = H + (i64)col[e] * F;
            for (i32 k = 0; k < F; ++k) {
                double t = a * (double)h[k];
                y[k] += t;
                if (s) s[k] += fabs(t);
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* dH[j][k] = sum_{e=(i,j)} a_e * G[i][k]      (scatter along the columns)    */
/* Threads, when used, own disjoint feature ranges, so there is no race.      */
/* ------------------------------------------------------------------------ */
void orc_spmm_t(i64 n, const i32 *rowptr, const i32 *col, const float *vals, i32 F,
                const float *G, double *dH, double *S, i32 use_threads)
{
    memset(dH, 0, sizeof(double) * (size_t)n * F);
    if (S) memset(S, 0, sizeof(double) * (size_t)n * F);
    int nt = use_threads ? orc_num_threads() : 1;
    if (nt > F) nt = F;
    int t;
#pragma omp parallel for schedule(static, 1) num_threads(nt) if (nt > 1)
    for (t = 0; t < nt; ++t) {
        i32 k0 = (i32)((i64)F * t / nt), k1 = (i32)((i64)F * (t + 1) / nt);
        for (i64 i = 0; i < n; ++i) {
            const float *g = G + i * F;
            for (i32 e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double a = vals ? (double)vals[e] : 1.0;
                double *d = dH + (i64)col[e] * F;
                double *s = S ? S + (i64)col[e] * F : 0;
                for (i32 k = k0; k < k1; ++k) {
                    double v = a * (double)g[k];
                    d[k] += v;
                    if (s) s[k] += fabs(v);
                }
            }
        }
    }
}

/* Algorithm 1: for every edge and every feature, Y[dst] += X[src] (serial). */
void orc_coo_sum(i64 n, i64 E, const i32 *row, const i32 *colv, i32 F, const float *X, double *Y)
{
    memset(Y, 0, sizeof(double) * (size_t)n * F);
    for (i64 e = 0; e < E; ++e) {
        i64 dst = row[e], src = colv[e];
        for (i32 d = 0; d < F; ++d) Y[dst * F + d] += (double)X[src * F + d];
    }
}

/* ------------------------------------------------------------------------ */
/* Reordering                                                                */
/* ------------------------------------------------------------------------ */
/* ------------------------------------------------------------------------ */
/* Y[i][k] = max_{e in row i} H[col_e][k]; arg = smallest column attaining it */
/* ------------------------------------------------------------------------ */
void orc_spmax(i64 n, const i32 *rowptr, const i32 *col, i32 F, const float *H, double *Y, i32 *arg)
{
    for (i64 i = 0; i < n; ++i) {
        for (i32 k = 0; k < F; ++k) {
            double best = 0.0;
            i32 who = -1;
            for (i32 e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const double h = (double)H[(i64)col[e] * F + k];
                if (who < 0 || h > best || (h == best && col[e] < who)) {
                    best = h;
                    who = col[e];
                }
            }
            Y[i * F + k] = best;
            arg[i * F + k] = who;
        }
    }
}

/* dH[j][k] = sum over rows i with arg[i][k] == j of G[i][k]; S the same sum of |G| */
void orc_spmax_t(i64 n, i32 F, const i32 *arg, const float *G, double *D, double *S)
{
    for (i64 q = 0; q < n * F; ++q) { D[q] = 0.0; S[q] = 0.0; }
    for (i64 i = 0; i < n; ++i)
        for (i32 k = 0; k < F; ++k) {
            const i32 j = arg[i * F + k];
            if (j < 0) continue;
            const double g = (double)G[i * F + k];
            D[(i64)j * F + k] += g;
            S[(i64)j * F + k] += fabs(g);
        }
}

static int cmp_i32(const void *a, const void *b)
{
    i32 x = *(const i32 *)a, y = *(const i32 *)b;
    return (x > y) - (x < y);
}

typedef struct { i32 nbr; i32 w; } arc_t;
static int cmp_arc(const void *a, const void *b)
{
    i32 x = ((const arc_t *)a)->nbr, y = ((const arc_t *)b)->nbr;
    return (x > y) - (x < y);
}

/* A weighted undirected graph in adjacency-array form. */
typedef struct {
    i32 n;
    i64 *xadj;   /* n+1 */
    i32 *adj;    /* neighbours */
    i32 *ew;     /* integer edge weights */
    i32 *nw;     /* node weights */
} wgraph;

static void wgraph_free(wgraph *g)
{
    free(g->xadj); free(g->adj); free(g->ew); free(g->nw);
    memset(g, 0, sizeof(*g));
}

/* Level-0 graph: u ~ v  iff  (a_uv stored or a_vu stored) and u != v. */
static int build_pattern_graph(i64 n, const i32 *rowptr, const i32 *col, wgraph *g)
{
    i64 *cnt = (i64 *)calloc((size_t)n + 1, sizeof(i64));
    if (!cnt) return -1;
    for (i64 i = 0; i < n; ++i)
        for (i32 e = rowptr[i]; e < rowptr[i + 1]; ++e)
            if (col[e] != i) { cnt[i + 1]++; cnt[col[e] + 1]++; }
    for (i64 i = 0; i < n; ++i) cnt[i + 1] += cnt[i];
    i64 tot = cnt[n];
    i32 *tmp = (i32 *)malloc(sizeof(i32) * (size_t)(tot ? tot : 1));
    i64 *pos = (i64 *)malloc(sizeof(i64) * (size_t)(n + 1));
    if (!tmp || !pos) return -1;
    memcpy(pos, cnt, sizeof(i64) * (size_t)(n + 1));
    for (i64 i = 0; i < n; ++i)
        for (i32 e = rowptr[i]; e < rowptr[i + 1]; ++e)
            if (col[e] != i) { tmp[pos[i]++] = col[e]; tmp[pos[col[e]]++] = (i32)i; }
    /* sort every list and drop duplicates */
    g->n = (i32)n;
    g->xadj = (i64 *)calloc((size_t)n + 1, sizeof(i64));
    g->adj = (i32 *)malloc(sizeof(i32) * (size_t)(tot ? tot : 1));
    i64 out = 0;
    for (i64 i = 0; i < n; ++i) {
        i64 b = cnt[i], e = cnt[i + 1];
        qsort(tmp + b, (size_t)(e - b), sizeof(i32), cmp_i32);
        g->xadj[i] = out;
        for (i64 p = b; p < e; ++p)
            if (p == b || tmp[p] != tmp[p - 1]) g->adj[out++] = tmp[p];
    }
    g->xadj[n] = out;
    g->ew = (i32 *)malloc(sizeof(i32) * (size_t)(out ? out : 1));
    g->nw = (i32 *)malloc(sizeof(i32) * (size_t)(n ? n : 1));
    for (i64 p = 0; p < out; ++p) g->ew[p] = 1;
    for (i64 i = 0; i < n; ++i) g->nw[i] = 1;
    free(tmp); free(pos); free(cnt);
    return 0;
}

/*
 * One level of size-constrained label propagation.
 * Every node starts in its own label.  Nodes are visited in ascending id, up
 * to `sweeps` times; a node looks at the total edge weight conn[L] towards
 * every neighbouring label L and moves to the label with the largest conn
 * that still has room (size + own weight <= cap); ties go to the current
 * label first, then to the smallest label id.  A label must attract at least
 * `thr` weight to be joined (1 in the very first sweep of the finest level or
 * for nodes of total weight < 2, otherwise 2).  A node attached to its current
 * label by less than `thr` gives that attachment up: it accepts any admissible
 * neighbouring label, and if there is none it returns to its own label when
 * that is empty.  Sizes are updated immediately (asynchronous propagation).
 * Returns the number of clusters; cluster ids are dense, numbered by first
 * appearance when scanning the nodes in ascending id.
 */
static i32 propagate_level(const wgraph *g, i32 level, i32 cap, i32 sweeps, i32 *cluster)
{
    i32 n = g->n;
    i32 *label = (i32 *)malloc(sizeof(i32) * (size_t)(n ? n : 1));
    i32 *size = (i32 *)malloc(sizeof(i32) * (size_t)(n ? n : 1));
    i64 *conn = (i64 *)calloc((size_t)(n ? n : 1), sizeof(i64));
    i64 *tot = (i64 *)calloc((size_t)(n ? n : 1), sizeof(i64));
    i32 maxdeg = 0;
    for (i32 v = 0; v < n; ++v) {
        label[v] = v;
        size[v] = g->nw[v];
        for (i64 e = g->xadj[v]; e < g->xadj[v + 1]; ++e) tot[v] += g->ew[e];
        i64 d = g->xadj[v + 1] - g->xadj[v];
        if (d > maxdeg) maxdeg = (i32)d;
    }
    i32 *cand = (i32 *)malloc(sizeof(i32) * (size_t)(maxdeg ? maxdeg : 1));
    for (i32 s = 0; s < sweeps; ++s) {
        i64 moved = 0;
        for (i32 v = 0; v < n; ++v) {
            if (tot[v] == 0) continue;
            i32 nc = 0;
            for (i64 e = g->xadj[v]; e < g->xadj[v + 1]; ++e) {
                i32 L = label[g->adj[e]];
                if (conn[L] == 0) cand[nc++] = L;
                conn[L] += g->ew[e];
            }
            i64 thr = ((level == 0 && s == 0) || tot[v] < 2) ? 1 : 2;
            i32 cur = label[v];
            i64 bw = conn[cur];
            i32 best = cur;
            if (bw < thr) {
                bw = 0;
                if (size[cur] > g->nw[v] && size[v] == 0) best = v;
            }
            qsort(cand, (size_t)nc, sizeof(i32), cmp_i32);
            for (i32 c = 0; c < nc; ++c) {
                i32 L = cand[c];
                if (L == cur) continue;
                if (conn[L] >= thr && size[L] + g->nw[v] <= cap && conn[L] > bw) {
                    best = L;
                    bw = conn[L];
                }
            }
            for (i32 c = 0; c < nc; ++c) conn[cand[c]] = 0;
            if (best != cur) {
                size[cur] -= g->nw[v];
                size[best] += g->nw[v];
                label[v] = best;
                ++moved;
            }
        }
        if (moved == 0) break;
    }
    /* dense renumbering by first appearance */
    i32 *newid = size;                       /* reuse */
    for (i32 v = 0; v < n; ++v) newid[v] = -1;
    i32 k = 0;
    for (i32 v = 0; v < n; ++v) {
        if (newid[label[v]] < 0) newid[label[v]] = k++;
        cluster[v] = newid[label[v]];
    }
    free(label); free(size); free(conn); free(tot); free(cand);
    return k;
}

/* Contract clusters into nodes: weights add up, inner edges disappear. */
static int contract(const wgraph *g, const i32 *cluster, i32 k, wgraph *c)
{
    i32 n = g->n;
    c->n = k;
    c->nw = (i32 *)calloc((size_t)(k ? k : 1), sizeof(i32));
    i64 *cnt = (i64 *)calloc((size_t)k + 1, sizeof(i64));
    for (i32 v = 0; v < n; ++v) {
        c->nw[cluster[v]] += g->nw[v];
        for (i64 e = g->xadj[v]; e < g->xadj[v + 1]; ++e)
            if (cluster[g->adj[e]] != cluster[v]) cnt[cluster[v] + 1]++;
    }
    for (i32 q = 0; q < k; ++q) cnt[q + 1] += cnt[q];
    i64 tot = cnt[k];
    arc_t *arcs = (arc_t *)malloc(sizeof(arc_t) * (size_t)(tot ? tot : 1));
    i64 *pos = (i64 *)malloc(sizeof(i64) * ((size_t)k + 1));
    memcpy(pos, cnt, sizeof(i64) * ((size_t)k + 1));
    for (i32 v = 0; v < n; ++v)
        for (i64 e = g->xadj[v]; e < g->xadj[v + 1]; ++e) {
            i32 cu = cluster[g->adj[e]], cv = cluster[v];
            if (cu != cv) { arcs[pos[cv]].nbr = cu; arcs[pos[cv]].w = g->ew[e]; pos[cv]++; }
        }
    c->xadj = (i64 *)calloc((size_t)k + 1, sizeof(i64));
    c->adj = (i32 *)malloc(sizeof(i32) * (size_t)(tot ? tot : 1));
    c->ew = (i32 *)malloc(sizeof(i32) * (size_t)(tot ? tot : 1));
    i64 out = 0;
    for (i32 q = 0; q < k; ++q) {
        i64 b = cnt[q], e = cnt[q + 1];
        qsort(arcs + b, (size_t)(e - b), sizeof(arc_t), cmp_arc);
        c->xadj[q] = out;
        for (i64 p = b; p < e; ++p) {
            if (p > b && arcs[p].nbr == arcs[p - 1].nbr) c->ew[out - 1] += arcs[p].w;
            else { c->adj[out] = arcs[p].nbr; c->ew[out] = arcs[p].w; ++out; }
        }
    }
    c->xadj[k] = out;
    free(arcs); free(pos); free(cnt);
    return 0;
}

/*
 * Second community-detection method (Sec. 4.2 leaves the choice of the partitioner to the user and
 * Sec. 6.1 compares two of them): one pass of size-constrained agglomeration by the integer
 * modularity gain, in the spirit of incremental-aggregation orderings.
 *   Every vertex starts as a community of its own with degree deg = number of its neighbours;
 *   M2 = sum of all degrees (twice the edge count).  Vertices are visited once, in ascending
 *   degree (ties: ascending id); isolated vertices are skipped.  The visited vertex u stands for
 *   the community it is the root of (itself plus everything merged into it so far).  For every
 *   other community r that one of u's members touches, with conn = number of edges between the
 *   two, the gain of merging is  conn * M2 - deg[u] * deg[r]  (the modularity difference times a
 *   positive constant, so integers suffice).  Among the communities with a positive gain and
 *   size[u] + size[r] <= cap the largest gain wins (ties: smallest root id) and u's community is
 *   merged into it: sizes and degrees add up, r stays the root.  Without such a community u's
 *   community stays as it is (it can still receive others later).
 * Cluster ids are dense, numbered by first appearance when scanning the vertices in ascending id.
 */
typedef struct { i64 deg; i32 v; } degkey_t;
static int cmp_degkey(const void *a, const void *b)
{
    const degkey_t *x = (const degkey_t *)a, *y = (const degkey_t *)b;
    if (x->deg != y->deg) return (x->deg > y->deg) - (x->deg < y->deg);
    return (x->v > y->v) - (x->v < y->v);
}

static i32 agglomerate_by_gain(const wgraph *g, i32 cap, i32 *cluster)
{
    const i32 n = g->n;
    const size_t nn = (size_t)(n ? n : 1);
    i32 *root = (i32 *)malloc(sizeof(i32) * nn);      /* community (root vertex) of every vertex */
    i32 *next = (i32 *)malloc(sizeof(i32) * nn);      /* member lists: singly linked, head = root */
    i32 *last = (i32 *)malloc(sizeof(i32) * nn);
    i32 *size = (i32 *)malloc(sizeof(i32) * nn);
    i64 *deg = (i64 *)malloc(sizeof(i64) * nn);
    i64 *conn = (i64 *)calloc(nn, sizeof(i64));
    i32 *cand = (i32 *)malloc(sizeof(i32) * nn);
    degkey_t *order = (degkey_t *)malloc(sizeof(degkey_t) * nn);
    i64 M2 = 0;
    for (i32 v = 0; v < n; ++v) {
        root[v] = v; next[v] = -1; last[v] = v; size[v] = g->nw[v];
        deg[v] = 0;
        for (i64 e = g->xadj[v]; e < g->xadj[v + 1]; ++e) deg[v] += g->ew[e];
        M2 += deg[v];
        order[v].deg = deg[v];
        order[v].v = v;
    }
    qsort(order, (size_t)n, sizeof(degkey_t), cmp_degkey);
    for (i32 t = 0; t < n; ++t) {
        const i32 u = order[t].v;
        if (order[t].deg == 0) continue;
        i32 nc = 0;
        for (i32 x = u; x >= 0; x = next[x])
            for (i64 e = g->xadj[x]; e < g->xadj[x + 1]; ++e) {
                const i32 r = root[g->adj[e]];
                if (r == u) continue;
                if (conn[r] == 0) cand[nc++] = r;
                conn[r] += g->ew[e];
            }
        i32 best = -1;
        i64 best_gain = 0;
        for (i32 c = 0; c < nc; ++c) {
            const i32 r = cand[c];
            const i64 gain = conn[r] * M2 - deg[u] * deg[r];
            if (gain > 0 && size[u] + size[r] <= cap &&
                (gain > best_gain || (gain == best_gain && r < best))) {
                best = r;
                best_gain = gain;
            }
        }
        for (i32 c = 0; c < nc; ++c) conn[cand[c]] = 0;
        if (best >= 0) {
            for (i32 x = u; x >= 0; x = next[x]) root[x] = best;
            next[last[best]] = u;
            last[best] = last[u];
            size[best] += size[u];
            deg[best] += deg[u];
        }
    }
    i32 *newid = size;                        /* reuse */
    for (i32 v = 0; v < n; ++v) newid[v] = -1;
    i32 k = 0;
    for (i32 v = 0; v < n; ++v) {
        if (newid[root[v]] < 0) newid[root[v]] = k++;
        cluster[v] = newid[root[v]];
    }
    free(root); free(next); free(last); free(size); free(deg); free(conn); free(cand); free(order);
    return k;
}

/*
 * Community reordering.
 *   levels: run propagate_level, map every original vertex to its cluster,
 *   contract, and repeat on the coarse graph while a level still shrinks the
 *   node count by at least 5 % (20*k <= 19*n) and fewer than max_levels ran.
 *   layout: communities in the order described below (ascending id when no
 *   ordering level merges anything); those with at least min_block members
 *   become diagonal blocks (members in ascending original id); all remaining
 *   vertices follow as a block-less tail in ascending original id.
 * Outputs: perm[new] = old, iperm[old] = new, blk_ptr[0..nb], comm[old]
 * (final community id of every original vertex).  blk_ptr needs n+1 slots.
 */
typedef struct { i32 key[4]; i32 c; } ordkey_t;
static int cmp_ordkey(const void *a, const void *b)
{
    const ordkey_t *x = (const ordkey_t *)a, *y = (const ordkey_t *)b;
    for (int t = 0; t < 4; ++t)
        if (x->key[t] != y->key[t]) return (x->key[t] > y->key[t]) - (x->key[t] < y->key[t]);
    return (x->c > y->c) - (x->c < y->c);
}

int orc_reorder_method(i64 n, const i32 *rowptr, const i32 *col, i32 method, i32 cap, i32 min_block, i32 sweeps,
                       i32 max_levels, i32 order_levels, i32 *perm, i32 *iperm, i32 *blk_ptr, i32 *nb_out, i32 *comm)
{
    wgraph g;
    memset(&g, 0, sizeof(g));
    if (build_pattern_graph(n, rowptr, col, &g)) return -1;
    for (i64 v = 0; v < n; ++v) comm[v] = (i32)v;
    i32 ncomm = (i32)n;
    i32 level = 0;
    if (method == 1 && g.n > 0) {              /* agglomeration by modularity gain: one pass, one level */
        ncomm = agglomerate_by_gain(&g, cap, comm);
        wgraph_free(&g);
    }
    while (g.n > 0) {
        i32 *cluster = (i32 *)malloc(sizeof(i32) * (size_t)g.n);
        i32 k = propagate_level(&g, level, cap, sweeps, cluster);
        for (i64 v = 0; v < n; ++v) comm[v] = cluster[comm[v]];
        ncomm = k;
        ++level;
        int go_on = (k < g.n) && ((i64)20 * k <= (i64)19 * g.n) && (level < max_levels);
        if (go_on) {
            wgraph c;
            memset(&c, 0, sizeof(c));
            contract(&g, cluster, k, &c);
            wgraph_free(&g);
            g = c;
        }
        free(cluster);
        if (!go_on) break;
    }
    wgraph_free(&g);
    /*
     * Order of the communities.  Up to order_levels (<= 3) further propagation levels run on the
     * graph of communities with the cap multiplied by 8 each time (same rules, level index > 0).
     * They only decide the ORDER: communities are sorted by (cluster at the top level, ...,
     * cluster at the first ordering level, community id), so communities that are strongly
     * connected end up next to each other.  A level that merges nothing ends the sequence.
     */
    ordkey_t *ord = (ordkey_t *)malloc(sizeof(ordkey_t) * (size_t)(ncomm ? ncomm : 1));
    for (i32 c = 0; c < ncomm; ++c) { ord[c].c = c; for (int t = 0; t < 4; ++t) ord[c].key[t] = 0; }
    if (order_levels > 3) order_levels = 3;
    if (order_levels > 0 && ncomm > 1) {
        wgraph g0, cg;
        memset(&g0, 0, sizeof(g0));
        memset(&cg, 0, sizeof(cg));
        if (build_pattern_graph(n, rowptr, col, &g0)) return -1;
        contract(&g0, comm, ncomm, &cg);
        wgraph_free(&g0);
        i32 *at_node = (i32 *)malloc(sizeof(i32) * (size_t)ncomm);   /* coarse node of every community */
        for (i32 c = 0; c < ncomm; ++c) at_node[c] = c;
        i64 cap2 = cap;
        for (i32 ol = 0; ol < order_levels && cg.n > 1; ++ol) {
            cap2 *= 8;
            if (cap2 > 0x3fffffff) cap2 = 0x3fffffff;
            i32 *cluster = (i32 *)malloc(sizeof(i32) * (size_t)cg.n);
            i32 kk = propagate_level(&cg, 1 + ol, (i32)cap2, sweeps, cluster);
            if (kk == cg.n) { free(cluster); break; }
            for (i32 c = 0; c < ncomm; ++c) {
                at_node[c] = cluster[at_node[c]];
                ord[c].key[2 - ol] = at_node[c];             /* higher levels are more significant */
            }
            wgraph nx;
            memset(&nx, 0, sizeof(nx));
            contract(&cg, cluster, kk, &nx);
            wgraph_free(&cg);
            cg = nx;
            free(cluster);
        }
        wgraph_free(&cg);
        free(at_node);
        qsort(ord, (size_t)ncomm, sizeof(ordkey_t), cmp_ordkey);
    }
    /* layout */
    i32 *csize = (i32 *)calloc((size_t)(ncomm ? ncomm : 1), sizeof(i32));
    for (i64 v = 0; v < n; ++v) csize[comm[v]]++;
    i32 *cstart = (i32 *)malloc(sizeof(i32) * (size_t)(ncomm ? ncomm : 1));
    i32 nb = 0, at = 0;
    blk_ptr[0] = 0;
    for (i32 oc = 0; oc < ncomm; ++oc) {
        const i32 c = ord[oc].c;
        if (csize[c] >= min_block) {
            cstart[c] = at;
            at += csize[c];
            blk_ptr[++nb] = at;
        } else cstart[c] = -1;
    }
    i32 tail = at;
    for (i64 v = 0; v < n; ++v) {
        i32 c = comm[v];
        i32 p = (cstart[c] >= 0) ? cstart[c]++ : tail++;
        perm[p] = (i32)v;
        iperm[v] = p;
    }
    *nb_out = nb;
    free(csize); free(cstart); free(ord);
    return 0;
}

/* method 0: multilevel size-constrained label propagation (the default) */
int orc_reorder(i64 n, const i32 *rowptr, const i32 *col, i32 cap, i32 min_block, i32 sweeps,
                i32 max_levels, i32 order_levels, i32 *perm, i32 *iperm, i32 *blk_ptr, i32 *nb_out, i32 *comm)
{
    return orc_reorder_method(n, rowptr, col, 0, cap, min_block, sweeps, max_levels, order_levels, perm, iperm,
                              blk_ptr, nb_out, comm);
}

/* ------------------------------------------------------------------------ */
/* Decomposition: one pass over the reordered edges; an entry whose row and   */
/* column fall in the same diagonal block is intra, every other one is inter. */
/* Tail vertices belong to no block.  Rows come out with ascending columns.   */
/* ------------------------------------------------------------------------ */
typedef struct { i32 c; float v; } ent_t;
static int cmp_ent(const void *a, const void *b)
{
    i32 x = ((const ent_t *)a)->c, y = ((const ent_t *)b)->c;
    return (x > y) - (x < y);
}

int orc_split(i64 n, const i32 *rowptr, const i32 *col, const float *vals, const i32 *perm,
              const i32 *iperm, const i32 *blk_ptr, i32 nb,
              i32 *in_rowptr, i32 *in_col, float *in_val,
              i32 *out_rowptr, i32 *out_col, float *out_val)
{
    i32 *blk = (i32 *)malloc(sizeof(i32) * (size_t)(n ? n : 1));
    for (i64 r = 0; r < n; ++r) blk[r] = -1;
    for (i32 b = 0; b < nb; ++b)
        for (i32 r = blk_ptr[b]; r < blk_ptr[b + 1]; ++r) blk[r] = b;
    i32 maxd = 0;
    for (i64 i = 0; i < n; ++i)
        if (rowptr[i + 1] - rowptr[i] > maxd) maxd = rowptr[i + 1] - rowptr[i];
    ent_t *row = (ent_t *)malloc(sizeof(ent_t) * (size_t)(maxd ? maxd : 1));
    i32 ni = 0, no = 0;
    in_rowptr[0] = 0;
    out_rowptr[0] = 0;
    for (i64 r = 0; r < n; ++r) {
        i32 old = perm[r];
        i32 d = 0;
        for (i32 e = rowptr[old]; e < rowptr[old + 1]; ++e) {
            row[d].c = iperm[col[e]];
            row[d].v = vals ? vals[e] : 1.0f;
            ++d;
        }
        qsort(row, (size_t)d, sizeof(ent_t), cmp_ent);
        for (i32 t = 0; t < d; ++t) {
            int same = blk[r] >= 0 && blk[row[t].c] == blk[r];
            if (same) { in_col[ni] = row[t].c; if (in_val) in_val[ni] = row[t].v; ++ni; }
            else      { out_col[no] = row[t].c; if (out_val) out_val[no] = row[t].v; ++no; }
        }
        in_rowptr[r + 1] = ni;
        out_rowptr[r + 1] = no;
    }
    free(blk); free(row);
    return 0;
}
