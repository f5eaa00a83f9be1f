// Host side of plan creation: input checks, transpose, the intra / inter decomposition
// (paper Sec. 3.3: an entry whose source and destination fall in the same diagonal block is
// intra-community, every other entry is inter-community; Sec. 4.2 second stage) and the
// per-kernel storage formats (dense / CSR of Sec. 2.1 "Graph Format", specialised per block).
#include <algorithm>
#include <cstring>
#include <thread>

#include "ag_internal.h"

namespace ag {

int ingest_csr(const ag_csr *in, HostCsr &out, std::string &err)
{
    if (!in || in->n < 0 || in->nnz < 0 || (in->n + 1 > 0 && !in->rowptr) || (in->nnz > 0 && !in->colidx)) {
        err = "null or negative-sized CSR input";
        return AG_ERR_INVALID;
    }
    if (in->n >= (int64_t)1 << 31 || in->nnz >= (int64_t)1 << 31) {
        err = "matrix too large for 32-bit indices";
        return AG_ERR_UNSUPPORTED;
    }
    const int64_t n = in->n;
    if (in->rowptr[0] != 0 || in->rowptr[n] != in->nnz) {
        err = "rowptr[0] must be 0 and rowptr[n] must equal nnz";
        return AG_ERR_INVALID;
    }
    for (int64_t i = 0; i < n; ++i)
        if (in->rowptr[i + 1] < in->rowptr[i]) {
            err = "rowptr is not monotone at row " + std::to_string(i);
            return AG_ERR_INVALID;
        }
    for (int64_t e = 0; e < in->nnz; ++e)
        if (in->colidx[e] < 0 || in->colidx[e] >= n) {
            err = "column index out of range at entry " + std::to_string(e);
            return AG_ERR_INVALID;
        }
    out.n = n;
    out.rowptr.assign(in->rowptr, in->rowptr + n + 1);
    out.col.assign(in->colidx, in->colidx + in->nnz);
    if (in->vals) out.val.assign(in->vals, in->vals + in->nnz);
    else out.val.clear();
    // sort unsorted rows (carrying values), then look for duplicates
    std::vector<std::pair<int32_t, float>> tmp;
    for (int64_t i = 0; i < n; ++i) {
        const int32_t b = out.rowptr[i], e = out.rowptr[i + 1];
        bool sorted = true;
        for (int32_t p = b + 1; p < e; ++p)
            if (out.col[p] < out.col[p - 1]) { sorted = false; break; }
        if (!sorted) {
            tmp.resize(e - b);
            for (int32_t p = b; p < e; ++p) tmp[p - b] = {out.col[p], in->vals ? out.val[p] : 1.0f};
            std::stable_sort(tmp.begin(), tmp.end(),
                             [](const auto &x, const auto &y) { return x.first < y.first; });
            for (int32_t p = b; p < e; ++p) {
                out.col[p] = tmp[p - b].first;
                if (in->vals) out.val[p] = tmp[p - b].second;
            }
        }
        for (int32_t p = b + 1; p < e; ++p)
            if (out.col[p] == out.col[p - 1]) {
                err = "duplicate entry in row " + std::to_string(i);
                return AG_ERR_INVALID;
            }
    }
    return AG_OK;
}

void transpose_csr(const HostCsr &A, HostCsr &At)
{
    const int64_t n = A.n, nnz = A.nnz();
    At.n = n;
    At.rowptr.assign(n + 1, 0);
    At.col.resize(nnz);
    At.val.resize(A.val.empty() ? 0 : nnz);
    // Row ranges of A go to threads; every thread counts its entries per column, the counts become
    // write positions ordered by (column, thread), and every thread scatters its rows in ascending
    // order: each row of A^T comes out sorted by source row, whatever the thread count.
    std::vector<std::vector<int32_t>> cnt(16);
    std::vector<int64_t> lo_of(16, 0), hi_of(16, 0);
    const int nt = parallel_ranges(n, [&](int t, int64_t lo, int64_t hi) {
        lo_of[t] = lo; hi_of[t] = hi;
        cnt[t].assign(n, 0);
        for (int32_t e = A.rowptr[lo]; e < A.rowptr[hi]; ++e) cnt[t][A.col[e]]++;
    }, 65536);
    int32_t run = 0;
    for (int64_t c = 0; c < n; ++c) {
        At.rowptr[c] = run;
        for (int t = 0; t < nt; ++t) {
            const int32_t k = cnt[t][c];
            cnt[t][c] = run;                          // becomes thread t's write position in column c
            run += k;
        }
    }
    At.rowptr[n] = run;
    parallel_ranges(n, [&](int t, int64_t lo, int64_t hi) {
        std::vector<int32_t> &at = cnt[t];
        for (int64_t i = lo; i < hi; ++i)
            for (int32_t e = A.rowptr[i]; e < A.rowptr[i + 1]; ++e) {
                const int32_t p = at[A.col[e]]++;
                At.col[p] = (int32_t)i;
                if (!A.val.empty()) At.val[p] = A.val[e];
            }
    }, 65536);
}

bool bitwise_equal(const HostCsr &A, const HostCsr &B)
{
    if (A.n != B.n || A.rowptr != B.rowptr || A.col != B.col || A.val.size() != B.val.size()) return false;
    return A.val.empty() || std::memcmp(A.val.data(), B.val.data(), A.val.size() * sizeof(float)) == 0;
}

// Renumber rows and columns with the permutation, sort every row by its new column, and
// route each entry to the intra part (same diagonal block) or to the inter part.
void permute_and_split(const HostCsr &A, const ReorderResult &r, HostCsr &full, HostCsr &intra,
                       HostCsr &inter)
{
    const int64_t n = A.n, nnz = A.nnz();
    const bool weighted = !A.val.empty();
    const int32_t nbr = r.blk_ptr.back();
    std::vector<int32_t> block_of(n, -1);
    for (int32_t b = 0; b < r.n_blocks; ++b)
        std::fill(block_of.begin() + r.blk_ptr[b], block_of.begin() + r.blk_ptr[b + 1], b);
    (void)nbr;
    full.n = intra.n = inter.n = n;
    full.rowptr.assign(n + 1, 0);
    intra.rowptr.assign(n + 1, 0);
    inter.rowptr.assign(n + 1, 0);
    // pass 1: per-row counts
    parallel_ranges(n, [&](int, int64_t lo, int64_t hi) {
        for (int64_t row = lo; row < hi; ++row) {
            const int32_t old = r.perm[row], b = block_of[row];
            int32_t in = 0;
            for (int32_t e = A.rowptr[old]; e < A.rowptr[old + 1]; ++e)
                in += (b >= 0 && block_of[r.iperm[A.col[e]]] == b);
            const int32_t d = A.rowptr[old + 1] - A.rowptr[old];
            full.rowptr[row + 1] = d;
            intra.rowptr[row + 1] = in;
            inter.rowptr[row + 1] = d - in;
        }
    });
    for (int64_t i = 0; i < n; ++i) {
        full.rowptr[i + 1] += full.rowptr[i];
        intra.rowptr[i + 1] += intra.rowptr[i];
        inter.rowptr[i + 1] += inter.rowptr[i];
    }
    full.col.resize(nnz);
    intra.col.resize(intra.rowptr[n]);
    inter.col.resize(inter.rowptr[n]);
    if (weighted) {
        full.val.resize(nnz);
        intra.val.resize(intra.rowptr[n]);
        inter.val.resize(inter.rowptr[n]);
    } else {
        full.val.clear(); intra.val.clear(); inter.val.clear();
    }
    // pass 2: fill
    parallel_ranges(n, [&](int, int64_t lo, int64_t hi) {
        std::vector<std::pair<int32_t, float>> ent;
        for (int64_t row = lo; row < hi; ++row) {
            const int32_t old = r.perm[row], b = block_of[row];
            ent.clear();
            for (int32_t e = A.rowptr[old]; e < A.rowptr[old + 1]; ++e)
                ent.emplace_back(r.iperm[A.col[e]], weighted ? A.val[e] : 1.0f);
            std::sort(ent.begin(), ent.end(),
                      [](const auto &x, const auto &y) { return x.first < y.first; });
            int32_t pf = full.rowptr[row], pi = intra.rowptr[row], po = inter.rowptr[row];
            for (const auto &en : ent) {
                full.col[pf] = en.first;
                if (weighted) full.val[pf] = en.second;
                ++pf;
                if (b >= 0 && block_of[en.first] == b) {
                    intra.col[pi] = en.first;
                    if (weighted) intra.val[pi] = en.second;
                    ++pi;
                } else {
                    inter.col[po] = en.first;
                    if (weighted) inter.val[po] = en.second;
                    ++po;
                }
            }
        }
    });
}

// Rows with more than kLongThresh entries are cut into segments of kSegLen entries.
void build_segments(const HostCsr &A, HostDir::Segs &s)
{
    s = HostDir::Segs();
    s.lr_seg0.push_back(0);
    for (int64_t i = 0; i < A.n; ++i) {
        const int32_t b = A.rowptr[i], e = A.rowptr[i + 1];
        if (e - b <= kLongThresh) continue;
        for (int32_t p = b; p < e; p += kSegLen) {
            s.seg_row.push_back((int32_t)i);
            s.seg_beg.push_back(p);
            s.seg_end.push_back(std::min(e, p + kSegLen));
        }
        s.lr_row.push_back((int32_t)i);
        s.lr_seg0.push_back((int32_t)s.seg_row.size());
    }
}

// Block-local one-byte columns for the block-sparse kernel; for every dense-class block a
// 128 x 128 bit map (row-major, 4 words per row) and, for weighted matrices, the values laid
// out in the operand order of the 32x32x2 fp32 matrix instruction:
//   tile[wave w][step s][lane l] = A_block[32 w + (l & 31)][2 s + (l >> 5)].
void build_block_formats(const ReorderResult &r, const std::vector<int32_t> &dense_blocks,
                         bool unit, HostDir &d)
{
    const HostCsr &I = d.intra;
    d.intra_col8.resize(I.col.size());
    for (int32_t b = 0; b < r.n_blocks; ++b) {
        const int32_t r0 = r.blk_ptr[b];
        for (int32_t row = r0; row < r.blk_ptr[b + 1]; ++row)
            for (int32_t e = I.rowptr[row]; e < I.rowptr[row + 1]; ++e)
                d.intra_col8[e] = (uint8_t)(I.col[e] - r0);
    }
    d.bitmap.assign(dense_blocks.size() * (size_t)kMaxBlock * 4, 0u);
    d.tiles.assign(unit ? 0 : dense_blocks.size() * (size_t)kMaxBlock * kMaxBlock, 0.0f);
    for (size_t k = 0; k < dense_blocks.size(); ++k) {
        const int32_t b = dense_blocks[k], r0 = r.blk_ptr[b];
        uint32_t *bm = d.bitmap.data() + k * kMaxBlock * 4;
        float *tl = unit ? nullptr : d.tiles.data() + k * (size_t)kMaxBlock * kMaxBlock;
        for (int32_t row = r0; row < r.blk_ptr[b + 1]; ++row) {
            const int32_t i = row - r0;
            for (int32_t e = I.rowptr[row]; e < I.rowptr[row + 1]; ++e) {
                const int32_t c = I.col[e] - r0;
                bm[i * 4 + (c >> 5)] |= 1u << (c & 31);
                if (tl) {
                    const int32_t w = i >> 5, lane = (i & 31) + 32 * (c & 1), step = c >> 1;
                    tl[(size_t)w * 4096 + step * 64 + lane] = I.val[e];
                }
            }
        }
    }
}

}  // namespace ag
