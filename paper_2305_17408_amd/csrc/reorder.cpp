// Community-based vertex reordering (paper Sec. 2.2 and Sec. 4.2, first preprocessing stage).
//
// The paper hands this step to an external partitioner with "community size" as its
// parameter.  This library uses its own integer-only, deterministic methods: multilevel
// label propagation under a community-size cap (the default) or one pass of agglomeration
// by modularity gain under the same cap.  Vertices end up grouped by community;
// communities of at least `min_block` members become the diagonal blocks of the
// intra-community subgraph, everything else is placed behind them as a block-less tail.
#include <algorithm>
#include <array>
#include <numeric>

#include "ag_internal.h"

namespace ag {

// u ~ v  iff  a_uv or a_vu is stored and u != v: merge row v of A with row v of A^T.
void build_pattern_graph(const HostCsr &A, const HostCsr &At, WGraph &g)
{
    const int64_t n = A.n;
    g.n = (int32_t)n;
    g.xadj.assign(n + 1, 0);
    // merge of the two sorted rows without the diagonal; emit == nullptr only counts
    auto merge_row = [&](int64_t v, int32_t *emit) -> int64_t {
        int32_t a = A.rowptr[v], ae = A.rowptr[v + 1];
        int32_t b = At.rowptr[v], be = At.rowptr[v + 1];
        int64_t cnt = 0;
        while (a < ae || b < be) {
            int32_t x;
            if (b >= be || (a < ae && A.col[a] <= At.col[b])) {
                x = A.col[a];
                if (b < be && At.col[b] == x) ++b;
                ++a;
            } else {
                x = At.col[b++];
            }
            if (x != v) {
                if (emit) emit[cnt] = x;
                ++cnt;
            }
        }
        return cnt;
    };
    parallel_ranges(n, [&](int, int64_t lo, int64_t hi) {
        for (int64_t v = lo; v < hi; ++v) g.xadj[v + 1] = merge_row(v, nullptr);
    });
    for (int64_t v = 0; v < n; ++v) g.xadj[v + 1] += g.xadj[v];
    g.adj.resize((size_t)g.xadj[n]);
    parallel_ranges(n, [&](int, int64_t lo, int64_t hi) {
        for (int64_t v = lo; v < hi; ++v) merge_row(v, g.adj.data() + g.xadj[v]);
    });
    g.ew.assign(g.adj.size(), 1);
    g.nw.assign((size_t)n, 1);
}

namespace {

// One level of capped label propagation; returns the cluster count and fills `cluster`
// with dense ids numbered by first appearance in ascending node order.
int32_t propagate(const WGraph &g, int32_t level, int32_t cap, int32_t sweeps,
                  std::vector<int32_t> &cluster)
{
    const int32_t n = g.n;
    std::vector<int32_t> label(n), size(g.nw);
    std::vector<int64_t> tot(n, 0), conn(n, 0);
    std::iota(label.begin(), label.end(), 0);
    for (int32_t v = 0; v < n; ++v)
        for (int64_t e = g.xadj[v]; e < g.xadj[v + 1]; ++e) tot[v] += g.ew[e];
    std::vector<int32_t> touched;
    // A node is evaluated only if its outcome can differ from "stay": `dirty` = it or a neighbour
    // moved since its last evaluation (its connection weights or its own label changed), `sens` =
    // its last evaluation depended on label sizes (a stronger neighbouring label was full, or it
    // was weakly attached).  Otherwise the same weights and the same current label give the same
    // "stay", whatever happened to the sizes: skipping it changes nothing in the result.
    std::vector<uint8_t> dirty(n, 1), sens(n, 0);
    for (int32_t s = 0; s < sweeps; ++s) {
        int64_t moved = 0;
        const bool all = (level == 0 && s == 1);        // the joining threshold just changed for everyone
        for (int32_t v = 0; v < n; ++v) {
            if (tot[v] == 0) continue;
            if (!all && !dirty[v] && !sens[v]) continue;
            touched.clear();
            for (int64_t e = g.xadj[v]; e < g.xadj[v + 1]; ++e) {
                const int32_t L = label[g.adj[e]];
                if (conn[L] == 0) touched.push_back(L);
                conn[L] += g.ew[e];
            }
            const int64_t need = ((level == 0 && s == 0) || tot[v] < 2) ? 1 : 2;
            const int32_t cur = label[v], w = g.nw[v];
            const int64_t own = conn[cur];
            // strongest admissible neighbouring label; equal strength -> smallest id
            int32_t cand = -1;
            int64_t cand_conn = 0;
            bool blocked = false;                       // a label that would win is full
            for (int32_t L : touched) {
                const int64_t c = conn[L];
                conn[L] = 0;
                if (L == cur || c < need) continue;
                if (size[L] + w > cap) {
                    if (c > own || own < need) blocked = true;
                    continue;
                }
                if (c > cand_conn || (c == cand_conn && L < cand)) { cand_conn = c; cand = L; }
            }
            int32_t target = cur;
            if (own >= need) {
                if (cand >= 0 && cand_conn > own) target = cand;      // the current label wins ties
            } else if (cand >= 0) {
                target = cand;                                          // weakly attached: any admissible label
            } else if (size[cur] > w && size[v] == 0) {
                target = v;                                             // ... or back to its own empty label
            }
            dirty[v] = 0;
            sens[v] = blocked || own < need;
            if (target != cur) {
                size[cur] -= w;
                size[target] += w;
                label[v] = target;
                ++moved;
                dirty[v] = 1;
                for (int64_t e = g.xadj[v]; e < g.xadj[v + 1]; ++e) dirty[g.adj[e]] = 1;
            }
        }
        if (!moved) break;
    }
    std::vector<int32_t> dense_id(n, -1);
    int32_t k = 0;
    cluster.resize(n);
    for (int32_t v = 0; v < n; ++v) {
        int32_t &d = dense_id[label[v]];
        if (d < 0) d = k++;
        cluster[v] = d;
    }
    return k;
}

// Clusters become nodes; node weights add, parallel edges add, inner edges vanish.  The neighbours
// of a cluster are listed in order of first appearance while its members are walked in ascending
// order, so the result does not depend on how the clusters are shared out among the threads.
void contract(const WGraph &g, const std::vector<int32_t> &cluster, int32_t k, WGraph &c)
{
    const int32_t n = g.n;
    // members of every cluster, grouped by a counting sort
    std::vector<int32_t> start(k + 1, 0), member(n);
    for (int32_t v = 0; v < n; ++v) start[cluster[v] + 1]++;
    for (int32_t q = 0; q < k; ++q) start[q + 1] += start[q];
    {
        std::vector<int32_t> at(start.begin(), start.end() - 1);
        for (int32_t v = 0; v < n; ++v) member[at[cluster[v]]++] = v;
    }
    c.n = k;
    c.nw.assign(k, 0);
    c.xadj.assign(k + 1, 0);
    struct Piece { int64_t lo = 0, hi = 0; std::vector<int32_t> adj, ew; };
    std::vector<Piece> piece(16);
    const int nt = parallel_ranges(k, [&](int t, int64_t lo, int64_t hi) {
        Piece &P = piece[t];
        P.lo = lo; P.hi = hi;
        std::vector<int64_t> wsum(k, 0);
        std::vector<int32_t> seen;
        for (int64_t q = lo; q < hi; ++q) {
            seen.clear();
            int32_t w = 0;
            for (int32_t mi = start[q]; mi < start[q + 1]; ++mi) {
                const int32_t v = member[mi];
                w += g.nw[v];
                for (int64_t e = g.xadj[v]; e < g.xadj[v + 1]; ++e) {
                    const int32_t t2 = cluster[g.adj[e]];
                    if (t2 == q) continue;
                    if (wsum[t2] == 0) seen.push_back(t2);
                    wsum[t2] += g.ew[e];
                }
            }
            c.nw[q] = w;
            for (int32_t t2 : seen) {
                P.adj.push_back(t2);
                P.ew.push_back((int32_t)wsum[t2]);
                wsum[t2] = 0;
            }
            c.xadj[q + 1] = (int64_t)seen.size();
        }
    }, n >= 65536 ? 64 : (int64_t)1 << 40);              // a cluster stands for many vertices; small graphs stay on one thread
    for (int32_t q = 0; q < k; ++q) c.xadj[q + 1] += c.xadj[q];
    c.adj.resize((size_t)c.xadj[k]);
    c.ew.resize((size_t)c.xadj[k]);
    for (int t = 0; t < nt; ++t) {
        const Piece &P = piece[t];
        if (P.adj.empty()) continue;
        std::copy(P.adj.begin(), P.adj.end(), c.adj.begin() + c.xadj[P.lo]);
        std::copy(P.ew.begin(), P.ew.end(), c.ew.begin() + c.xadj[P.lo]);
    }
}

// The second community detection (the partitioner is the user's choice, Sec. 4.2): one pass of
// agglomeration under the size cap, vertices visited in ascending degree (a counting sort keeps
// equal degrees in ascending id).  The visited vertex stands for the community rooted at it; it
// joins the neighbouring community with the largest positive integer modularity gain
//     conn * M2 - deg[u] * deg[r]        (M2 = sum of all degrees)
// that still has room, smallest root id among equal gains.  Returns the community count and
// fills `cluster` with dense ids numbered by first appearance in ascending vertex order.
int32_t agglomerate(const WGraph &g, int32_t cap, std::vector<int32_t> &cluster)
{
    const int32_t n = g.n;
    std::vector<int64_t> deg(n, 0);
    int64_t M2 = 0, maxdeg = 0;
    for (int32_t v = 0; v < n; ++v) {
        for (int64_t e = g.xadj[v]; e < g.xadj[v + 1]; ++e) deg[v] += g.ew[e];
        M2 += deg[v];
        maxdeg = std::max(maxdeg, deg[v]);
    }
    // visiting order: by degree, then id
    std::vector<int32_t> order(n);
    {
        std::vector<int64_t> first((size_t)maxdeg + 2, 0);
        for (int32_t v = 0; v < n; ++v) first[deg[v] + 1]++;
        for (int64_t d = 0; d <= maxdeg; ++d) first[d + 1] += first[d];
        for (int32_t v = 0; v < n; ++v) order[first[deg[v]]++] = v;
    }
    std::vector<int32_t> root(n), size(g.nw);
    std::iota(root.begin(), root.end(), 0);
    std::vector<std::vector<int32_t>> members(n);       // of roots that absorbed somebody (the root itself excluded)
    std::vector<int64_t> conn(n, 0);
    std::vector<int32_t> stamp(n, -1), touched;
    for (int32_t u : order) {
        if (deg[u] == 0) continue;
        touched.clear();
        auto scan = [&](int32_t x) {
            for (int64_t e = g.xadj[x]; e < g.xadj[x + 1]; ++e) {
                const int32_t r = root[g.adj[e]];
                if (r == u) continue;
                if (stamp[r] != u) { stamp[r] = u; conn[r] = 0; touched.push_back(r); }
                conn[r] += g.ew[e];
            }
        };
        scan(u);
        for (int32_t x : members[u]) scan(x);
        int32_t best = -1;
        int64_t best_gain = 0;
        for (int32_t r : touched) {
            if (size[u] + size[r] > cap) continue;
            const int64_t gain = conn[r] * M2 - deg[u] * deg[r];
            if (gain <= 0) continue;
            if (best < 0 || gain > best_gain || (gain == best_gain && r < best)) { best = r; best_gain = gain; }
        }
        if (best < 0) continue;
        std::vector<int32_t> &mb = members[best];
        root[u] = best;
        mb.push_back(u);
        for (int32_t x : members[u]) { root[x] = best; mb.push_back(x); }
        std::vector<int32_t>().swap(members[u]);
        size[best] += size[u];
        deg[best] += deg[u];
    }
    std::vector<int32_t> dense_id(n, -1);
    int32_t k = 0;
    cluster.resize(n);
    for (int32_t v = 0; v < n; ++v) {
        int32_t &d = dense_id[root[v]];
        if (d < 0) d = k++;
        cluster[v] = d;
    }
    return k;
}

}  // namespace

void community_reorder(const WGraph &g0, int32_t method, int32_t cap, int32_t min_block, int32_t sweeps,
                       int32_t max_levels, int32_t order_levels, ReorderResult &out)
{
    const int32_t n = g0.n;
    out.comm.resize(n);
    std::iota(out.comm.begin(), out.comm.end(), 0);
    int32_t n_comm = n;
    WGraph coarse;
    const WGraph *g = &g0;
    std::vector<int32_t> cluster;
    if (method == AG_METHOD_MODULARITY && n > 0) {
        n_comm = agglomerate(g0, cap, out.comm);
        g = &coarse;                                     // empty: no propagation levels
    }
    for (int32_t level = 0; g->n > 0;) {
        const int32_t k = propagate(*g, level, cap, sweeps, cluster);
        for (int32_t v = 0; v < n; ++v) out.comm[v] = cluster[out.comm[v]];
        n_comm = k;
        ++level;
        // another level only while the last one shrank the graph by at least 5 %
        if (k == g->n || (int64_t)20 * k > (int64_t)19 * g->n || level >= max_levels) break;
        WGraph next;
        contract(*g, cluster, k, next);
        coarse = std::move(next);
        g = &coarse;
    }
    // Order of the communities: up to three more propagation levels on the graph of communities,
    // the cap growing 8x per level, decide only who sits next to whom (strongly connected
    // communities become neighbours, so the remainder's gathers find their rows in a nearby L2);
    // communities are sorted by (top-level cluster, ..., first-level cluster, id).
    std::vector<int32_t> order(n_comm);
    std::iota(order.begin(), order.end(), 0);
    if (order_levels > 0 && n_comm > 1) {
        std::vector<std::array<int32_t, 3>> key(n_comm, std::array<int32_t, 3>{0, 0, 0});
        std::vector<int32_t> node(n_comm);
        std::iota(node.begin(), node.end(), 0);
        WGraph cg, nx;
        contract(g0, out.comm, n_comm, cg);
        int64_t cap2 = cap;
        for (int32_t ol = 0; ol < std::min(order_levels, 3) && cg.n > 1; ++ol) {
            cap2 = std::min<int64_t>(cap2 * 8, 0x3fffffff);
            const int32_t kk = propagate(cg, 1 + ol, (int32_t)cap2, sweeps, cluster);
            if (kk == cg.n) break;
            for (int32_t c = 0; c < n_comm; ++c) {
                node[c] = cluster[node[c]];
                key[c][2 - ol] = node[c];
            }
            contract(cg, cluster, kk, nx);
            cg = std::move(nx);
        }
        std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            return key[a] != key[b] ? key[a] < key[b] : a < b;
        });
    }
    // layout: blocks (communities >= min_block in that order, members ascending), then the tail
    std::vector<int32_t> csize(n_comm, 0), slot(n_comm, -1);
    for (int32_t v = 0; v < n; ++v) csize[out.comm[v]]++;
    out.blk_ptr.assign(1, 0);
    int32_t at = 0;
    for (int32_t c : order)
        if (csize[c] >= min_block) {
            slot[c] = at;
            at += csize[c];
            out.blk_ptr.push_back(at);
        }
    out.n_blocks = (int32_t)out.blk_ptr.size() - 1;
    int32_t tail = at;
    out.perm.resize(n);
    out.iperm.resize(n);
    for (int32_t v = 0; v < n; ++v) {
        int32_t &s = slot[out.comm[v]];
        const int32_t p = (s >= 0) ? s++ : tail++;
        out.perm[p] = v;
        out.iperm[v] = p;
    }
}

}  // namespace ag
