// Learned cost model of the search (Section VI-A, level three: the paper fits a regression model to
// the measured points of the coarse grid and uses it to decide which further points are worth a
// run; it names XGBoost).  Here: gradient-boosted regression trees (squared error) over features of the
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

// ---- gradient-boosted regression trees --------------------------------------------------------
// Squared loss on log2(microseconds per stored entry): the model starts from the mean and every round
// fits a shallow tree to what is still unexplained and adds a tenth of it.  Many shallow trees carry
// over to matrices the corpus has not seen better than one deep tree, which only looks measurements up.
namespace {
constexpr int kRounds = 300, kMaxDepth = 4, kMinSplit = 6;
constexpr double kRate = 0.1;
}  // namespace

// Best split of the samples marked `node` in mark[]: every feature's samples are walked in the order
// sorted once in train().
int CostModel::grow(std::vector<Node> &tree, const std::vector<double> &target, std::vector<int> &mark, int node,
                    int count, int depth) {
    double sum = 0;
    const int n = (int)x_.size();
    for (int i = 0; i < n; ++i)
        if (mark[(size_t)i] == node) sum += target[(size_t)i];
    Node nd;
    nd.value = sum / count;
    const int me = (int)tree.size();
    tree.push_back(nd);
    if (count < kMinSplit || depth >= kMaxDepth) return me;
    double sse = 0;
    for (int i = 0; i < n; ++i)
        if (mark[(size_t)i] == node) sse += (target[(size_t)i] - nd.value) * (target[(size_t)i] - nd.value);
    if (sse < 1e-12) return me;
    double best = sse * (1 - 1e-9), bt = 0;
    int bf = -1;
    const size_t nf = x_[0].size();
    for (size_t f = 0; f < nf; ++f) {
        double ls = 0, ls2 = 0;
        double ts = sum, ts2 = sse + sum * sum / count;
        int nl = 0;
        double prev = 0;
        bool have = false;
        for (int i : order_[f]) {
            if (mark[(size_t)i] != node) continue;
            const double v = x_[(size_t)i][f], t = target[(size_t)i];
            if (have && v != prev && nl >= 2 && count - nl >= 2) {
                const double rs = ts - ls, rs2 = ts2 - ls2;
                const double cost = (ls2 - ls * ls / nl) + (rs2 - rs * rs / (count - nl));
                if (cost < best) {
                    best = cost;
                    bf = (int)f;
                    bt = 0.5 * (prev + v);
                }
            }
            ls += t;
            ls2 += t * t;
            ++nl;
            prev = v;
            have = true;
        }
    }
    if (bf < 0) return me;
    const int left_id = next_mark_++, right_id = next_mark_++;
    int nl = 0;
    for (int i = 0; i < n; ++i)
        if (mark[(size_t)i] == node) {
            const bool l = x_[(size_t)i][(size_t)bf] <= bt;
            mark[(size_t)i] = l ? left_id : right_id;
            nl += l;
        }
    tree[(size_t)me].feature = bf;
    tree[(size_t)me].threshold = bt;
    const int l = grow(tree, target, mark, left_id, nl, depth + 1);
    const int r = grow(tree, target, mark, right_id, count - nl, depth + 1);
    tree[(size_t)me].left = l;
    tree[(size_t)me].right = r;
    return me;
}

static double tree_value(const std::vector<CostModel::Node> &t, const std::vector<double> &f) {
    int n = 0;
    while (t[(size_t)n].feature >= 0) n = f[(size_t)t[(size_t)n].feature] <= t[(size_t)n].threshold ? t[(size_t)n].left : t[(size_t)n].right;
    return t[(size_t)n].value;
}

void CostModel::add(const CostCensus &c, const PlanSpec &spec, double us) {
    if (!(us > 0) || c.nnz < 1) return;
    x_.push_back(cost_features(c, spec));
    y_.push_back(std::log2(us) - std::log2((double)c.nnz));   // time per stored entry: sizes become comparable
}

void CostModel::train() {
    trees_.clear();
    const int n = (int)x_.size();
    if (n < 8) return;   // too little to say anything
    const size_t nf = x_[0].size();
    order_.assign(nf, std::vector<int>());
    for (size_t f = 0; f < nf; ++f) {
        order_[f].resize((size_t)n);
        for (int i = 0; i < n; ++i) order_[f][(size_t)i] = i;
        std::stable_sort(order_[f].begin(), order_[f].end(), [&](int a, int b) { return x_[(size_t)a][f] < x_[(size_t)b][f]; });
    }
    base_ = 0;
    for (double v : y_) base_ += v;
    base_ /= n;
    std::vector<double> resid((size_t)n);
    for (int i = 0; i < n; ++i) resid[(size_t)i] = y_[(size_t)i] - base_;
    std::vector<int> mark((size_t)n);
    for (int m = 0; m < kRounds; ++m) {
        std::fill(mark.begin(), mark.end(), 0);
        next_mark_ = 1;
        std::vector<Node> tree;
        grow(tree, resid, mark, 0, n, 0);
        double worst = 0;
        for (int i = 0; i < n; ++i) {
            resid[(size_t)i] -= kRate * tree_value(tree, x_[(size_t)i]);
            worst = std::max(worst, std::fabs(resid[(size_t)i]));
        }
        trees_.push_back(std::move(tree));
        if (worst < 1e-3) break;   // every sample explained to a tenth of a percent
    }
    order_.clear();
}

double CostModel::predict_us(const CostCensus &c, const PlanSpec &spec) const {
    if (trees_.empty() || c.nnz < 1) return -1;
    const std::vector<double> f = cost_features(c, spec);
    double v = base_;
    for (const std::vector<Node> &t : trees_) v += kRate * tree_value(t, f);
    return std::exp2(v + std::log2((double)c.nnz));
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
