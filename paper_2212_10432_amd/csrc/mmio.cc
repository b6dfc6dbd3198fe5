// Matrix Market coordinate files -> CSR (the input the paper's tool takes: Section III, and the
// artifact description).  Written from the published format description: a banner line
//   %%MatrixMarket matrix coordinate <real|integer|pattern|complex> <general|symmetric|skew-symmetric|hermitian>
// comment lines starting with '%', a size line "rows cols entries", then one "i j [value]" line per
// stored entry with 1-based indices.  Supported: coordinate; real, integer (read as floating
// point) and pattern (every value 1); general, symmetric (entry (i,j), i != j, also stands for
// (j,i)) and skew-symmetric ((j,i) = -(i,j)).  Dense "array" files and complex values are refused.
#include <algorithm>
#include <cctype>
#include <cerrno>
#include <cstdio>
#include <numeric>

#include "internal.h"

namespace spmv {

namespace {

struct FileBuf {
    char *p = nullptr;
    size_t n = 0;
    ~FileBuf() { std::free(p); }
};

void slurp(const char *path, FileBuf &b) {
    std::FILE *f = std::fopen(path, "rb");
    if (!f) fail(SPMV_ERR_INVALID_ARG, std::string("cannot open ") + path);
    std::vector<char> chunk(1 << 20);
    size_t cap = 0;
    for (;;) {
        const size_t got = std::fread(chunk.data(), 1, chunk.size(), f);
        if (got == 0) break;
        if (b.n + got + 1 > cap) {
            cap = std::max(cap * 2, b.n + got + 1);
            char *q = (char *)std::realloc(b.p, cap);
            if (!q) {
                std::fclose(f);
                fail(SPMV_ERR_ALLOC, "host allocation failed while reading the file");
            }
            b.p = q;
        }
        std::memcpy(b.p + b.n, chunk.data(), got);
        b.n += got;
    }
    const bool err = std::ferror(f) != 0;
    std::fclose(f);
    if (err) fail(SPMV_ERR_INVALID_ARG, std::string("read error on ") + path);
    if (!b.p) {
        b.p = (char *)std::malloc(1);
        if (!b.p) fail(SPMV_ERR_ALLOC, "host allocation failed");
    }
    b.p[b.n] = 0;
}

std::string lower(std::string s) {
    for (char &c : s) c = (char)std::tolower((unsigned char)c);
    return s;
}

// next line of the buffer as [b, e); false at the end
bool next_line(const char *&cur, const char *end, const char *&b, const char *&e) {
    if (cur >= end) return false;
    b = cur;
    while (cur < end && *cur != '\n') ++cur;
    e = cur;
    if (cur < end) ++cur;
    while (e > b && (e[-1] == '\r' || e[-1] == ' ' || e[-1] == '\t')) --e;
    return true;
}

}  // namespace

void read_matrix_market(const char *path, spmv_dtype_t dtype, MmCsr &out) {
    FileBuf buf;
    slurp(path, buf);
    const char *cur = buf.p, *end = buf.p + buf.n, *b = nullptr, *e = nullptr;
    if (!next_line(cur, end, b, e)) fail(SPMV_ERR_INVALID_ARG, "Matrix Market: empty file");
    std::vector<std::string> words;
    {
        std::string line(b, e), w;
        std::stringstream ss(line);
        while (ss >> w) words.push_back(lower(w));
    }
    if (words.size() < 5 || words[0] != "%%matrixmarket" || words[1] != "matrix")
        fail(SPMV_ERR_INVALID_ARG, "Matrix Market: the first line is not a '%%MatrixMarket matrix ...' banner");
    if (words[2] != "coordinate") fail(SPMV_ERR_UNSUPPORTED, "Matrix Market: only the coordinate format is read (got " + words[2] + ")");
    const std::string field = words[3], sym = words[4];
    if (field != "real" && field != "integer" && field != "pattern" && field != "double")
        fail(SPMV_ERR_UNSUPPORTED, "Matrix Market: field " + field + " is not supported");
    if (sym != "general" && sym != "symmetric" && sym != "skew-symmetric")
        fail(SPMV_ERR_UNSUPPORTED, "Matrix Market: symmetry " + sym + " is not supported");
    const bool pattern = field == "pattern";
    // size line: the first line that is neither a comment nor blank
    long long M = -1, N = -1, L = -1;
    while (next_line(cur, end, b, e)) {
        if (b == e || *b == '%') continue;
        char *q = nullptr;
        errno = 0;
        M = std::strtoll(b, &q, 10);
        const char *q1 = q;
        N = std::strtoll(q1, &q, 10);
        const char *q2 = q;
        L = std::strtoll(q2, &q, 10);
        // a number that starts after the end of this line was taken from the next one
        if (q1 == b || q2 == q1 || q == q2 || errno || q > e) fail(SPMV_ERR_INVALID_ARG, "Matrix Market: bad size line");
        break;
    }
    if (M < 0 || N < 0 || L < 0) fail(SPMV_ERR_INVALID_ARG, "Matrix Market: missing or negative size line");
    if (M >= (1LL << 31) - 64 || N >= (1LL << 31) - 64) fail(SPMV_ERR_UNSUPPORTED, "Matrix Market: dimensions must be below 2^31");
    if (sym != "general" && M != N) fail(SPMV_ERR_INVALID_ARG, "Matrix Market: a symmetric matrix must be square");
    std::vector<int32_t> ri, ci;
    std::vector<double> va;
    // an entry line is at least four bytes ("1 1\n"): a count the file cannot hold is malformed
    if (L > (long long)(end - cur) / 4 + 1)
        fail(SPMV_ERR_INVALID_ARG, "Matrix Market: the size line announces " + std::to_string(L) + " entries, more than the file can hold");
    // The entry lines are parsed in pieces that start at line starts, one piece per thread at a time;
    // a piece keeps its entries and, when a line is malformed, which of its entries that was.
    struct Piece {
        std::vector<int32_t> ri, ci;
        std::vector<double> va;
        long long bad_at = -1;   // number of well-formed entries of the piece in front of the first bad line
        spmv_status_t bad_code = SPMV_OK;
        const char *bad_text = "";
    };
    const int threads = default_threads();
    const int64_t bytes = (int64_t)(end - cur);
    const int64_t npieces = std::max<int64_t>(1, std::min<int64_t>((int64_t)threads * 4, bytes / (1 << 16)));
    std::vector<const char *> cut((size_t)npieces + 1);
    cut[0] = cur;
    cut[(size_t)npieces] = end;
    for (int64_t t = 1; t < npieces; ++t) {
        const char *q = cur + bytes * t / npieces;
        while (q < end && q[-1] != '\n') ++q;   // a piece starts right after a newline
        cut[(size_t)t] = q;
    }
    for (int64_t t = 1; t <= npieces; ++t) cut[(size_t)t] = std::max(cut[(size_t)t], cut[(size_t)t - 1]);
    std::vector<Piece> pieces((size_t)npieces);
    const bool skew = sym == "skew-symmetric";
    parallel_for(npieces, 1, threads, [&](int64_t tb, int64_t te, int) {
        for (int64_t t = tb; t < te; ++t) {
            Piece &pc = pieces[(size_t)t];
            const char *c2 = cut[(size_t)t], *e2 = cut[(size_t)t + 1], *lb = nullptr, *le = nullptr;
            auto bad = [&](spmv_status_t code, const char *text) {
                pc.bad_at = (long long)pc.ri.size();
                pc.bad_code = code;
                pc.bad_text = text;
            };
            while (pc.bad_at < 0 && next_line(c2, e2, lb, le)) {
                if (lb == le || *lb == '%') continue;
                char *q = nullptr;
                errno = 0;
                const long long i = std::strtoll(lb, &q, 10);
                const char *q1 = q;
                const long long j = std::strtoll(q1, &q, 10);
                // a number that starts after the end of this line was taken from the next one
                if (q1 == lb || q == q1 || errno || q > le) { bad(SPMV_ERR_INVALID_ARG, "bad entry line"); break; }
                double v = 1.0;
                if (!pattern) {
                    const char *q2 = q;
                    v = std::strtod(q2, &q);
                    if (q == q2 || q > le) { bad(SPMV_ERR_INVALID_ARG, "an entry has no value"); break; }
                }
                if (i < 1 || i > M || j < 1 || j > N) { bad(SPMV_ERR_BAD_CSR, "an entry lies outside the matrix"); break; }
                if (skew && i == j) { bad(SPMV_ERR_INVALID_ARG, "a skew-symmetric file stores no diagonal entry"); break; }
                pc.ri.push_back((int32_t)(i - 1));
                pc.ci.push_back((int32_t)(j - 1));
                pc.va.push_back(v);
            }
        }
    });
    // in file order: the first L entries count, a malformed line among them is an error, what follows
    // the L-th entry is not looked at
    long long seen = 0;
    for (const Piece &pc : pieces) {
        if (seen >= L) break;
        const long long take = std::min<long long>(L - seen, (long long)pc.ri.size());
        if (pc.bad_at >= 0 && pc.bad_at < L - seen)
            fail(pc.bad_code, "Matrix Market: entry " + std::to_string(seen + pc.bad_at + 1) + ": " + pc.bad_text);
        seen += take;
    }
    if (seen != L) fail(SPMV_ERR_INVALID_ARG, "Matrix Market: the file ends after " + std::to_string(seen) + " of " + std::to_string(L) + " entries");
    ri.reserve((size_t)L);
    ci.reserve((size_t)L);
    va.reserve((size_t)L);
    for (const Piece &pc : pieces) {
        const size_t take = (size_t)std::min<long long>(L - (long long)ri.size(), (long long)pc.ri.size());
        ri.insert(ri.end(), pc.ri.begin(), pc.ri.begin() + (std::ptrdiff_t)take);
        ci.insert(ci.end(), pc.ci.begin(), pc.ci.begin() + (std::ptrdiff_t)take);
        va.insert(va.end(), pc.va.begin(), pc.va.begin() + (std::ptrdiff_t)take);
        if ((long long)ri.size() >= L) break;
    }
    pieces.clear();
    // expand the symmetric forms
    if (sym != "general") {
        const double s = sym == "symmetric" ? 1.0 : -1.0;
        const size_t n0 = ri.size();
        for (size_t k = 0; k < n0; ++k)
            if (ri[k] != ci[k]) {
                ri.push_back(ci[k]);
                ci.push_back(ri[k]);
                va.push_back(s * va[k]);
            }
    }
    const int64_t nnz = (int64_t)ri.size();
    if (nnz >= ((int64_t)1 << 31)) fail(SPMV_ERR_UNSUPPORTED, "Matrix Market: nnz must be below 2^31");
    const size_t vs = dtype == SPMV_F64 ? 8 : 4;
    out.nrows = M;
    out.ncols = N;
    out.nnz = nnz;
    out.row_ptr = (int32_t *)std::calloc((size_t)M + 1, sizeof(int32_t));
    out.col = (int32_t *)std::malloc(std::max<size_t>((size_t)nnz, 1) * sizeof(int32_t));
    out.val = std::malloc(std::max<size_t>((size_t)nnz, 1) * vs);
    if (!out.row_ptr || !out.col || !out.val) {
        std::free(out.row_ptr);
        std::free(out.col);
        std::free(out.val);
        out = MmCsr();
        fail(SPMV_ERR_ALLOC, "host allocation failed");
    }
    // CSR: rows ascending (a counting sort, which keeps the file order inside a row), then columns
    // ascending inside a row with repeated positions in file order (a stable sort per row, rows in parallel)
    for (int64_t k = 0; k < nnz; ++k) out.row_ptr[ri[(size_t)k] + 1] += 1;
    for (int64_t r = 0; r < M; ++r) out.row_ptr[r + 1] += out.row_ptr[r];
    std::vector<int32_t> where((size_t)nnz);
    {
        std::vector<int32_t> fill(out.row_ptr, out.row_ptr + M);
        for (int64_t k = 0; k < nnz; ++k) where[(size_t)fill[(size_t)ri[(size_t)k]]++] = (int32_t)k;
    }
    parallel_for(M, 4096, threads, [&](int64_t rb, int64_t re, int) {
        for (int64_t r = rb; r < re; ++r) {
            int32_t *w0 = where.data() + out.row_ptr[r], *w1 = where.data() + out.row_ptr[r + 1];
            bool sorted = true;
            for (int32_t *w = w0; w + 1 < w1 && sorted; ++w) sorted = ci[(size_t)w[0]] <= ci[(size_t)w[1]];
            if (!sorted) std::stable_sort(w0, w1, [&](int32_t a, int32_t c) { return ci[(size_t)a] < ci[(size_t)c]; });
            for (int64_t k = out.row_ptr[r]; k < out.row_ptr[r + 1]; ++k) {
                const size_t src = (size_t)where[(size_t)k];
                out.col[k] = ci[src];
                if (dtype == SPMV_F64) ((double *)out.val)[k] = va[src];
                else ((float *)out.val)[k] = (float)va[src];
            }
        }
    });
}

}  // namespace spmv
