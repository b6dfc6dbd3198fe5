// Census of the sparsity pattern.  The paper prunes the operator search with the sparsity
// pattern of the input (Section VI-B); this pass collects what those rules need: row-length
// statistics (an "irregular" matrix has row-length variance > 100, Section I), the mass of the
// long-row tail, well-populated diagonals and the fill of aligned dense blocks.
#include <algorithm>
#include <cmath>
#include <map>

#include "internal.h"

namespace spmv {

Census take_census(const HostCsr &A, int threads) {
    Census c;
    c.nrows = A.nrows;
    c.ncols = A.ncols;
    c.nnz = A.nnz;
    if (A.nrows == 0) return c;

    // row lengths
    struct Acc {
        int64_t mn = INT64_MAX, mx = 0, empty = 0;
        long double s = 0, s2 = 0;
        int64_t rows_over[21] = {0}, nnz_over[21] = {0};
        bool sorted = true;
    };
    std::vector<Acc> acc((size_t)threads);
    parallel_for(A.nrows, 1 << 14, threads, [&](int64_t b, int64_t e, int t) {
        Acc &a = acc[(size_t)t];
        for (int64_t r = b; r < e; ++r) {
            const int64_t L = A.len(r);
            a.mn = std::min(a.mn, L);
            a.mx = std::max(a.mx, L);
            a.empty += (L == 0);
            a.s += (long double)L;
            a.s2 += (long double)L * (long double)L;
            for (int k = 0; k <= 20 && L > ((int64_t)1 << k); ++k) {
                a.rows_over[k] += 1;
                a.nnz_over[k] += L;
            }
            const int32_t *cc = A.col + A.row_ptr[r];
            for (int64_t k = 1; k < L; ++k)
                if (cc[k] < cc[k - 1]) { a.sorted = false; break; }
        }
    });
    long double s = 0, s2 = 0;
    c.min_len = INT64_MAX;
    for (const Acc &a : acc) {
        c.min_len = std::min(c.min_len, a.mn);
        c.max_len = std::max(c.max_len, a.mx);
        c.empty_rows += a.empty;
        s += a.s;
        s2 += a.s2;
        c.cols_sorted = c.cols_sorted && a.sorted;
        for (int k = 0; k <= 20; ++k) {
            c.rows_over[k] += a.rows_over[k];
            c.nnz_over[k] += a.nnz_over[k];
        }
    }
    c.mean_len = (double)(s / (long double)A.nrows);
    c.var_len = (double)(s2 / (long double)A.nrows) - c.mean_len * c.mean_len;
    if (c.var_len < 0) c.var_len = 0;

    // diagonals: offsets seen in >= 25 % of a sample of rows are counted exactly
    {
        const int64_t nsample = std::min<int64_t>(A.nrows, 4096);
        std::map<int64_t, int64_t> seen;
        for (int64_t i = 0; i < nsample; ++i) {
            const int64_t r = (i * A.nrows) / nsample;
            const int64_t L = std::min<int64_t>(A.len(r), 256);
            int64_t prev = INT64_MIN;
            for (int64_t k = 0; k < L; ++k) {
                const int64_t off = (int64_t)A.col[A.row_ptr[r] + k] - r;
                if (off != prev) seen[off] += 1;
                prev = off;
            }
        }
        std::vector<std::pair<int64_t, int64_t>> cand;   // (count, offset)
        for (auto &kv : seen)
            if (kv.second * 4 >= nsample) cand.push_back({kv.second, kv.first});
        std::sort(cand.rbegin(), cand.rend());
        if (cand.size() > 64) cand.resize(64);
        std::vector<int64_t> offs;
        for (auto &p : cand) offs.push_back(p.second);
        std::sort(offs.begin(), offs.end());
        if (!offs.empty()) {
            const size_t nd = offs.size();
            std::vector<std::vector<int64_t>> cnt((size_t)threads, std::vector<int64_t>(nd, 0));
            parallel_for(A.nrows, 1 << 13, threads, [&](int64_t b, int64_t e, int t) {
                auto &cn = cnt[(size_t)t];
                for (int64_t r = b; r < e; ++r)
                    for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                        const int64_t off = (int64_t)A.col[k] - r;
                        auto it = std::lower_bound(offs.begin(), offs.end(), off);
                        if (it != offs.end() && *it == off) cn[(size_t)(it - offs.begin())] += 1;
                    }
            });
            for (size_t d = 0; d < nd; ++d) {
                int64_t n = 0;
                for (auto &cn : cnt) n += cn[d];
                const int64_t off = offs[d];
                const int64_t lo = std::max<int64_t>(0, -off);
                const int64_t hi = std::min<int64_t>(A.nrows, A.ncols - off);
                const int64_t valid = hi - lo;
                if (valid > 0 && n * 2 >= valid) {
                    c.diag_offsets.push_back((int32_t)off);
                    c.diag_nnz += n;
                }
            }
        }
    }

    // aligned b x b blocks: fill estimated on a sample of block rows (the sampled block columns are
    // sorted here, so the order of the columns inside a row does not matter)
    {
        for (int bsz = 2; bsz <= 4; ++bsz) {
            if (A.nrows < bsz || A.ncols < bsz) continue;   // a ragged edge is not sampled: whole block rows only
            const int64_t nb = A.nrows / bsz;
            const int64_t nsample = std::min<int64_t>(nb, 2048);
            int64_t blocks = 0, entries = 0;
            std::vector<int32_t> tmp;
            for (int64_t i = 0; i < nsample; ++i) {
                const int64_t br = (i * nb) / nsample;
                tmp.clear();
                for (int64_t r = br * bsz; r < (br + 1) * bsz; ++r)
                    for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) tmp.push_back(A.col[k] / bsz);
                entries += (int64_t)tmp.size();
                std::sort(tmp.begin(), tmp.end());
                blocks += (int64_t)(std::unique(tmp.begin(), tmp.end()) - tmp.begin());
            }
            c.blocks[bsz] = blocks;
            c.block_fill[bsz] = blocks ? (double)entries / (double)(blocks * bsz * bsz) : 0.0;
        }
    }
    return c;
}

}  // namespace spmv
