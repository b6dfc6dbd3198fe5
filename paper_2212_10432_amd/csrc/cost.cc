// Learned cost model of the search (Section VI-A, level three: the paper fits a regression model to
// the measured points of the coarse grid and uses it to decide which further points are worth a
// run; it names XGBoost).  Here: one regression tree (CART, squared error) over features of the
// census and of the plan spec, trained when a search starts from a corpus of earlier measurements
// (one line per timed candidate, appended by every search that is given a log path).  The search
// uses the prediction to order its candidates and to skip those predicted far slower than the best.
//
// Corpus line (tab separated):
//   v1 dtype nrows ncols nnz mean_len var_len max_len nnz_over_64 nnz_over_1024 rows_over_1024
//   diag_nnz block_fill_3 spec measured_us
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <fstream>

#include "internal.h"

namespace spmv {

namespace {

const PlanSpec &first_leaf(const PlanSpec &p) { return p.node == N_LEAF ? p : first_leaf(p.kids[0]); }
int count_leaves(const PlanSpec &p) {
    if (p.node == N_LEAF) return 1;
    int n = 0;
    for (const PlanSpec &k : p.kids) n += count_leaves(k);
    return n;
}
bool any_leaf(const PlanSpec &p, const std::function<bool(const PlanSpec &)> &f) {
    if (p.node == N_LEAF) return f(p);
    for (const PlanSpec &k : p.kids)
        if (any_leaf(k, f)) return true;
    return false;
}
double lg(double v) { return std::log2(v < 1 ? 1.0 : v); }

}  // namespace

std::vector<double> cost_features(const CostCensus &c, const PlanSpec &spec) {
    std::vector<double> f;
    const double nnz = (double)std::max<int64_t>(c.nnz, 1);
    const double v = c.dtype == SPMV_F64 ? 8 : 4;
    f.push_back(lg(nnz));
    f.push_back(lg((double)c.nrows));
    f.push_back(c.mean_len);
    f.push_back(lg((double)c.max_len + 1));
    f.push_back(c.mean_len > 0 ? std::sqrt(std::max(0.0, c.var_len)) / c.mean_len : 0.0);
    f.push_back((double)c.nnz_over_64 / nnz);
    f.push_back((double)c.nnz_over_1024 / nnz);
    f.push_back(lg((double)c.rows_over_1024 + 1));
    f.push_back(lg((double)c.ncols * v));
    f.push_back(v);
    f.push_back((double)c.diag_nnz / nnz);
    f.push_back(c.block_fill_3);
    // the plan: shape of the tree, then the parameters of its first leaf
    f.push_back((double)spec.node);
    f.push_back((double)count_leaves(spec));
    f.push_back(any_leaf(spec, [](const PlanSpec &q) { return q.heavy > 0; }) ? 1 : 0);
    f.push_back(any_leaf(spec, [](const PlanSpec &q) { return q.light == L_XL; }) ? 1 : 0);
    const PlanSpec &q = first_leaf(spec);
    for (int l = 0; l <= L_WBM; ++l) f.push_back(q.light == l ? 1 : 0);   // one-hot: a tree splits on "is design l"
    f.push_back(q.dia);
    f.push_back(q.drows);
    f.push_back(lg((double)q.heavy + 1));
    f.push_back(lg((double)q.tile));
    f.push_back(q.hd);
    f.push_back(q.sigma < 0 ? 40.0 : lg((double)q.sigma + 1));
    f.push_back(q.lpr);
    f.push_back(lg((double)q.chunk + 1));
    f.push_back(q.block);
    f.push_back(q.xwin);
    f.push_back(q.smax);
    f.push_back(q.wg);
    f.push_back(q.remap);
    f.push_back(q.r);
    f.push_back(q.k);
    f.push_back(lg(q.w ? (double)q.w : 65536.0 / v));
    f.push_back(lg((double)q.rb));
    f.push_back(lg((double)q.piece + 1));
    return f;
}

CostCensus cost_census(const Census &c, spmv_dtype_t dtype) {
    CostCensus o;
    o.dtype = dtype;
    o.nrows = c.nrows;
    o.ncols = c.ncols;
    o.nnz = c.nnz;
    o.mean_len = c.mean_len;
    o.var_len = c.var_len;
    o.max_len = c.max_len;
    o.nnz_over_64 = c.nnz_over[6];
    o.nnz_over_1024 = c.nnz_over[10];
    o.rows_over_1024 = c.rows_over[10];
    o.diag_nnz = c.diag_nnz;
    o.block_fill_3 = c.block_fill[3];
    return o;
}

std::string cost_line(const CostCensus &c, const std::string &spec, double us) {
    char buf[512];
    std::snprintf(buf, sizeof buf, "v1\t%d\t%lld\t%lld\t%lld\t%.9g\t%.9g\t%lld\t%lld\t%lld\t%lld\t%lld\t%.6g\t", (int)c.dtype,
                  (long long)c.nrows, (long long)c.ncols, (long long)c.nnz, c.mean_len, c.var_len, (long long)c.max_len,
                  (long long)c.nnz_over_64, (long long)c.nnz_over_1024, (long long)c.rows_over_1024, (long long)c.diag_nnz,
                  c.block_fill_3);
    char tail[64];
    std::snprintf(tail, sizeof tail, "\t%.6g", us);
    return std::string(buf) + spec + tail;
}

void cost_append(const std::string &path, const std::vector<std::string> &lines) {
    if (path.empty() || lines.empty()) return;
    std::ofstream f(path, std::ios::app);
    if (!f) return;   // a log that cannot be written is not an error of the search
    for (const std::string &l : lines) f << l << "\n";
}

// ---- the regression tree -----------------------------------------------------------------------
int CostModel::grow(std::vector<int> &idx, int b, int e, int depth) {
    double sum = 0;
    for (int i = b; i < e; ++i) sum += y_[(size_t)idx[(size_t)i]];
    const double mean = sum / (e - b);
    Node nd;
    nd.value = mean;
    const int me = (int)nodes_.size();
    nodes_.push_back(nd);
    if (e - b < 4 || depth >= 12) return me;
    double sse = 0;
    for (int i = b; i < e; ++i) sse += (y_[(size_t)idx[(size_t)i]] - mean) * (y_[(size_t)idx[(size_t)i]] - mean);
    if (sse < 1e-9) return me;
    const size_t nf = x_[0].size();
    double best = sse * (1 - 1e-9);
    int bf = -1;
    double bt = 0;
    std::vector<std::pair<double, double>> col((size_t)(e - b));
    for (size_t f = 0; f < nf; ++f) {
        for (int i = b; i < e; ++i) col[(size_t)(i - b)] = {x_[(size_t)idx[(size_t)i]][f], y_[(size_t)idx[(size_t)i]]};
        std::sort(col.begin(), col.end());
        if (col.front().first == col.back().first) continue;
        double ls = 0, ls2 = 0, ts = 0, ts2 = 0;
        for (auto &p : col) {
            ts += p.second;
            ts2 += p.second * p.second;
        }
        const int n = e - b;
        for (int i = 0; i + 1 < n; ++i) {
            ls += col[(size_t)i].second;
            ls2 += col[(size_t)i].second * col[(size_t)i].second;
            if (col[(size_t)i].first == col[(size_t)i + 1].first) continue;
            const int nl = i + 1, nr = n - nl;
            const double rs = ts - ls, rs2 = ts2 - ls2;
            const double cost = (ls2 - ls * ls / nl) + (rs2 - rs * rs / nr);
            if (cost < best) {
                best = cost;
                bf = (int)f;
                bt = 0.5 * (col[(size_t)i].first + col[(size_t)i + 1].first);
            }
        }
    }
    if (bf < 0) return me;
    const int mid = (int)(std::partition(idx.begin() + b, idx.begin() + e, [&](int i) { return x_[(size_t)i][(size_t)bf] <= bt; }) - idx.begin());
    if (mid == b || mid == e) return me;
    nodes_[(size_t)me].feature = bf;
    nodes_[(size_t)me].threshold = bt;
    const int l = grow(idx, b, mid, depth + 1);
    const int r = grow(idx, mid, e, depth + 1);
    nodes_[(size_t)me].left = l;
    nodes_[(size_t)me].right = r;
    return me;
}

void CostModel::add(const CostCensus &c, const PlanSpec &spec, double us) {
    if (!(us > 0) || c.nnz < 1) return;
    x_.push_back(cost_features(c, spec));
    y_.push_back(std::log2(us) - std::log2((double)c.nnz));   // time per stored entry: sizes become comparable
}

void CostModel::train() {
    nodes_.clear();
    if (x_.size() < 8) return;   // too little to say anything
    std::vector<int> idx(x_.size());
    for (size_t i = 0; i < idx.size(); ++i) idx[i] = (int)i;
    grow(idx, 0, (int)idx.size(), 0);
}

double CostModel::predict_us(const CostCensus &c, const PlanSpec &spec) const {
    if (nodes_.empty() || c.nnz < 1) return -1;
    const std::vector<double> f = cost_features(c, spec);
    int n = 0;
    while (nodes_[(size_t)n].feature >= 0) n = f[(size_t)nodes_[(size_t)n].feature] <= nodes_[(size_t)n].threshold ? nodes_[(size_t)n].left : nodes_[(size_t)n].right;
    return std::exp2(nodes_[(size_t)n].value + std::log2((double)c.nnz));
}

int CostModel::load(const std::string &path) {
    std::ifstream f(path);
    if (!f) return 0;
    std::string line;
    int used = 0;
    while (std::getline(f, line)) {
        if (line.empty() || line[0] == '#') continue;
        std::vector<std::string> t;
        size_t b = 0;
        for (;;) {
            const size_t e = line.find('\t', b);
            t.push_back(line.substr(b, e == std::string::npos ? std::string::npos : e - b));
            if (e == std::string::npos) break;
            b = e + 1;
        }
        if (t.size() != 15 || t[0] != "v1") continue;
        try {
            CostCensus c;
            c.dtype = std::stoi(t[1]) ? SPMV_F64 : SPMV_F32;
            c.nrows = std::stoll(t[2]);
            c.ncols = std::stoll(t[3]);
            c.nnz = std::stoll(t[4]);
            c.mean_len = std::stod(t[5]);
            c.var_len = std::stod(t[6]);
            c.max_len = std::stoll(t[7]);
            c.nnz_over_64 = std::stoll(t[8]);
            c.nnz_over_1024 = std::stoll(t[9]);
            c.rows_over_1024 = std::stoll(t[10]);
            c.diag_nnz = std::stoll(t[11]);
            c.block_fill_3 = std::stod(t[12]);
            const PlanSpec spec = parse_spec(t[13]);
            add(c, spec, std::stod(t[14]));
            ++used;
        } catch (...) {
            continue;   // a line written by another version of the grammar: skipped
        }
    }
    return used;
}

}  // namespace spmv
