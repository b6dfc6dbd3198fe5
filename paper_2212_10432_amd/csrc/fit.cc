// Model-driven format compression (Section V-D): an index array of the format is tested against
// three models -- linear, step, periodic-linear -- each with a handful of "if" patches for
// outliers.  A model is only accepted when it reproduces EVERY element of the array; the run-time
// kernel compile then replaces the loads of that array by the model's arithmetic.
#include <algorithm>
#include <sstream>

#include "internal.h"

namespace spmv {

int64_t ArrayModel::at(int64_t i) const {
    for (const auto &p : patches)
        if (p.first == i) return p.second;
    return base + step * (i / period) + inner * (i % period);
}

std::string ArrayModel::text() const {
    if (kind == 0) return "";
    std::ostringstream o;
    o << (kind == 1 ? "linear" : kind == 2 ? "step" : "periodic-linear") << "(base=" << base << ",step=" << step;
    if (kind != 1) o << ",period=" << period;
    if (kind == 3) o << ",inner=" << inner;
    for (const auto &p : patches) o << ",if[" << p.first << "]=" << p.second;
    o << ")";
    return o.str();
}

// C expression in the index `var` (64-bit arithmetic), patches first.
std::string ArrayModel::expr(const std::string &var) const {
    std::ostringstream o;
    o << "(";
    for (const auto &p : patches) o << "(" << var << ")==" << p.first << "LL?" << p.second << "LL:";
    o << "(" << base << "LL";
    if (period == 1) {
        o << "+" << step << "LL*(long long)(" << var << ")";
    } else {
        o << "+" << step << "LL*((long long)(" << var << ")/" << period << "LL)";
        if (inner) o << "+" << inner << "LL*((long long)(" << var << ")%" << period << "LL)";
    }
    o << "))";
    return o.str();
}

namespace {

template <typename V>
bool accept(const V *a, int64_t n, ArrayModel &m) {
    const int64_t most = std::min<int64_t>(4, n / 8);
    m.patches.clear();
    for (int64_t i = 0; i < n; ++i) {
        const int64_t want = m.base + m.step * (i / m.period) + m.inner * (i % m.period);
        if ((int64_t)a[i] != want) {
            if ((int64_t)m.patches.size() >= most) return false;
            m.patches.push_back({i, (int64_t)a[i]});
        }
    }
    return true;
}

template <typename V>
ArrayModel fit_typed(const V *a, int64_t n) {
    ArrayModel m;
    if (n < 2) return m;
    // linear, from the first two and from the last two elements (either pair may hold an outlier)
    for (int end = 0; end < 2; ++end) {
        ArrayModel c;
        c.kind = 1;
        c.period = 1;
        if (!end) {
            c.step = (int64_t)a[1] - (int64_t)a[0];
            c.base = (int64_t)a[0];
        } else {
            c.step = (int64_t)a[n - 1] - (int64_t)a[n - 2];
            c.base = (int64_t)a[n - 1] - c.step * (n - 1);
        }
        if (accept(a, n, c)) return c;
    }
    // step (constant over runs of `period` indices) and periodic-linear (linear inside a period, a
    // jump from one period to the next).  The period is read off between two consecutive jumps after
    // an anchor; three anchors, so that an outlier near one of them does not hide the pattern.
    for (int anchor = 0; anchor < 3 && n >= 4; ++anchor) {
        const int64_t s0 = anchor * (n / 3);
        if (s0 + 1 >= n) break;
        const int64_t inner = (int64_t)a[s0 + 1] - (int64_t)a[s0];
        int64_t c1 = s0 + 2;
        while (c1 < n && (int64_t)a[c1] - (int64_t)a[c1 - 1] == inner) ++c1;
        if (c1 >= n) continue;
        int64_t c2 = c1 + 1;
        while (c2 < n && (int64_t)a[c2] - (int64_t)a[c2 - 1] == inner) ++c2;
        const int64_t cand[2] = {c2 < n ? c2 - c1 : c1 - s0, c1};   // between two jumps; or from the start to the first jump
        for (int64_t p : cand) {
            if (p < 2 || c1 % p != 0 || c1 + p > n) continue;
            ArrayModel c;
            c.kind = inner == 0 ? 2 : 3;
            c.period = p;
            c.inner = inner;
            c.step = (int64_t)a[c1 + p - 1] - (int64_t)a[c1 - 1];          // one period apart, same place in the period
            c.base = (int64_t)a[c1] - c.step * (c1 / p);
            if (accept(a, n, c)) return c;
        }
    }
    return m;
}

}  // namespace

ArrayModel fit_array(const void *data, int elem_bytes, int64_t n) {
    if (!data || n < 2) return ArrayModel();
    if (elem_bytes == 4) return fit_typed((const int32_t *)data, n);
    if (elem_bytes == 8) return fit_typed((const int64_t *)data, n);
    return ArrayModel();
}

// The metadata arrays of the format (offsets, row maps, windows, work items): everything a kernel
// indexes by block, slice, segment or row rather than by stored entry.
bool is_metadata_array(const std::string &name) {
    static const char *suffix[] = {".slice_ptr", ".seg_ptr", ".unit_ptr", ".gptr", ".tile_row", ".xwin", ".items", ".origin_rows",
                                   ".origin_brows", ".rows", ".pptr", ".bbase", ".xbase", ".offsets", ".open_slots"};
    for (const char *s : suffix) {
        const size_t k = std::strlen(s);
        if (name.size() >= k && name.compare(name.size() - k, k, s) == 0) return true;
    }
    return false;
}

}  // namespace spmv
