// Host threading helpers and the plan-spec grammar.
#include <algorithm>
#include <cstring>
#include <sstream>

#include "internal.h"

namespace spmv {

int default_threads() {
    unsigned n = std::thread::hardware_concurrency();
    if (const char *e = std::getenv("OMP_NUM_THREADS")) {   // the box exports its CPU share here
        int v = std::atoi(e);
        if (v > 0) n = (unsigned)v;
    }
    if (n < 1) n = 1;
    if (n > 64) n = 64;
    return (int)n;
}

void parallel_for(int64_t n, int64_t chunk, int threads,
                  const std::function<void(int64_t, int64_t, int)> &body) {
    if (n <= 0) return;
    if (chunk < 1) chunk = 1;
    const int64_t nchunks = (n + chunk - 1) / chunk;
    if (threads > nchunks) threads = (int)nchunks;
    if (threads <= 1) {
        body(0, n, 0);
        return;
    }
    std::atomic<int64_t> next{0};
    std::vector<Error> errors;
    std::atomic<bool> failed{false};
    std::vector<std::thread> pool;
    std::vector<std::string> what((size_t)threads);
    std::vector<int> codes((size_t)threads, 0);
    for (int t = 0; t < threads; ++t) {
        pool.emplace_back([&, t] {
            try {
                for (;;) {
                    const int64_t c = next.fetch_add(1, std::memory_order_relaxed);
                    if (c >= nchunks || failed.load(std::memory_order_relaxed)) break;
                    const int64_t b = c * chunk;
                    body(b, std::min(n, b + chunk), t);
                }
            } catch (const Error &e) {
                codes[(size_t)t] = (int)e.code;
                what[(size_t)t] = e.msg;
                failed = true;
            } catch (const std::exception &e) {
                codes[(size_t)t] = (int)SPMV_ERR_INTERNAL;
                what[(size_t)t] = e.what();
                failed = true;
            }
        });
    }
    for (auto &th : pool) th.join();
    for (int t = 0; t < threads; ++t)
        if (codes[(size_t)t]) fail((spmv_status_t)codes[(size_t)t], what[(size_t)t]);
}

// ---- plan-spec strings: "key=value,key=value" ------------------------------------------------
static const char *light_name(int l) {
    switch (l) {
    case L_CSRV: return "csrv";
    case L_SELL: return "sell";
    case L_BSELL: return "bsell";
    case L_BIN: return "bin";
    case L_XS: return "xs";
    case L_NNZB: return "nnzb";
    case L_XNB: return "xnb";
    case L_COO: return "coo";
    case L_XL: return "xl";
    case L_WBM: return "wbm";
    }
    return "?";
}

static bool pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

static PlanSpec parse_leaf(const std::string &s);

// node := leaf | ("rows" | "bin2" | "cut" | "cols") "(" n (":" n)* ")" ("{" node "}")+
static PlanSpec parse_node(const std::string &s, int depth) {
    if (depth > 6) fail(SPMV_ERR_INVALID_ARG, "plan spec: nested too deeply");
    size_t b = 0, e = s.size();
    while (b < e && (s[b] == ' ' || s[b] == '\t')) ++b;
    while (e > b && (s[e - 1] == ' ' || s[e - 1] == '\t')) --e;
    const std::string t = s.substr(b, e - b);
    static const struct { const char *word; int kind; } heads[] = {{"rows(", N_ROWS}, {"bin2(", N_BIN2}, {"cut(", N_CUT}, {"cols(", N_COLS}};
    int kind = N_LEAF;
    size_t open = 0;
    for (const auto &h : heads)
        if (t.compare(0, std::strlen(h.word), h.word) == 0) {
            kind = h.kind;
            open = std::strlen(h.word);
        }
    if (kind == N_LEAF) {
        if (t.find_first_of("{}()") != std::string::npos) fail(SPMV_ERR_INVALID_ARG, "plan spec: stray bracket in " + t);
        return parse_leaf(t);
    }
    PlanSpec p;
    p.node = kind;
    const size_t close = t.find(')', open);
    if (close == std::string::npos) fail(SPMV_ERR_INVALID_ARG, "plan spec: missing ')' in " + t);
    {
        std::stringstream ss(t.substr(open, close - open));
        std::string tok;
        while (std::getline(ss, tok, ':')) {
            char *end = nullptr;
            const long long v = std::strtoll(tok.c_str(), &end, 10);
            if (tok.empty() || *end || v < 0) fail(SPMV_ERR_INVALID_ARG, "plan spec: bad number in " + t.substr(0, close + 1));
            p.cuts.push_back((int64_t)v);
        }
    }
    size_t pos = close + 1;
    while (pos < t.size()) {
        if (t[pos] != '{') fail(SPMV_ERR_INVALID_ARG, "plan spec: '{' expected in " + t);
        int level = 0;
        size_t q = pos;
        for (; q < t.size(); ++q) {
            if (t[q] == '{') ++level;
            if (t[q] == '}' && --level == 0) break;
        }
        if (q == t.size()) fail(SPMV_ERR_INVALID_ARG, "plan spec: missing '}' in " + t);
        p.kids.push_back(parse_node(t.substr(pos + 1, q - pos - 1), depth + 1));
        pos = q + 1;
    }
    const size_t nk = p.kids.size();
    auto need = [&](bool ok, const char *msg) {
        if (!ok) fail(SPMV_ERR_INVALID_ARG, std::string("plan spec: ") + msg);
    };
    switch (kind) {
    case N_ROWS:
        need(!p.cuts.empty() && p.cuts.size() <= 16, "rows() takes 1 to 16 lengths");
        for (size_t i = 1; i < p.cuts.size(); ++i) need(p.cuts[i] > p.cuts[i - 1], "rows(): lengths must ascend");
        need(nk == 1 || nk == p.cuts.size() + 1, "rows(c1:..:cn) takes one design or n + 1");
        break;
    case N_BIN2:
        need(p.cuts.size() == 1 && p.cuts[0] >= 1 && p.cuts[0] <= 20, "bin2(k) takes one exponent in [1, 20]");
        need(nk == 2, "bin2(k) takes two designs: the bins below 2^k, the rows from 2^k on");
        break;
    case N_CUT:
        need(p.cuts.size() == 2 && p.cuts[0] >= 2 && p.cuts[1] >= 1, "cut(rho:minrows) needs rho >= 2 and minrows >= 1");
        need(nk == 1, "cut() takes one design");
        break;
    case N_COLS:
        need(p.cuts.size() == 1 && p.cuts[0] >= 2 && p.cuts[0] <= 64, "cols(k) takes a stripe count in [2, 64]");
        need(nk == 1 || (int64_t)nk == p.cuts[0], "cols(k) takes one design or k");
        break;
    }
    std::function<void(const PlanSpec &)> no_whole = [&](const PlanSpec &q) {
        if (q.node == N_LEAF) need(!q.dia && q.light != L_BSELL, "dia and bsell work on the whole matrix and cannot sit inside rows/bin2/cut/cols");
        for (const PlanSpec &k : q.kids) no_whole(k);
    };
    for (const PlanSpec &k : p.kids) no_whole(k);
    return p;
}

PlanSpec parse_spec(const std::string &s) { return parse_node(s, 0); }

static PlanSpec parse_leaf(const std::string &s) {
    PlanSpec p;
    std::stringstream ss(s);
    std::string tok;
    while (std::getline(ss, tok, ',')) {
        if (tok.empty()) continue;
        const size_t eq = tok.find('=');
        if (eq == std::string::npos) fail(SPMV_ERR_INVALID_ARG, "plan spec: token without '=': " + tok);
        const std::string k = tok.substr(0, eq), v = tok.substr(eq + 1);
        auto num = [&]() -> double {
            char *end = nullptr;
            const double d = std::strtod(v.c_str(), &end);
            if (v.empty() || *end) fail(SPMV_ERR_INVALID_ARG, "plan spec: bad number in " + tok);
            return d;
        };
        if (k == "light") {
            if (v == "csrv") p.light = L_CSRV;
            else if (v == "sell") p.light = L_SELL;
            else if (v == "bsell") p.light = L_BSELL;
            else if (v == "bin") p.light = L_BIN;
            else if (v == "xs") p.light = L_XS;
            else if (v == "nnzb") p.light = L_NNZB;
            else if (v == "xnb") p.light = L_XNB;
            else if (v == "coo") p.light = L_COO;
            else if (v == "xl") p.light = L_XL;
            else if (v == "wbm") p.light = L_WBM;
            else fail(SPMV_ERR_INVALID_ARG, "plan spec: unknown light design " + v);
        } else if (k == "dia") p.dia = (int)num();
        else if (k == "dia_fill") p.dia_fill = num();
        else if (k == "drows") p.drows = (int)num();
        else if (k == "heavy") p.heavy = (int64_t)num();
        else if (k == "tile") p.tile = (int)num();
        else if (k == "hd") p.hd = (int)num();
        else if (k == "piece") p.piece = (int)num();
        else if (k == "lpr") p.lpr = (int)num();
        else if (k == "chunk") p.chunk = (int64_t)num();
        else if (k == "sigma") p.sigma = (int)num();
        else if (k == "block") p.block = (int)num();
        else if (k == "smax") p.smax = (int)num();
        else if (k == "wg") p.wg = (int)num();
        else if (k == "remap") p.remap = (int)num();
        else if (k == "xwin") p.xwin = (int)num();
        else if (k == "k") p.k = (int)num();
        else if (k == "r") p.r = (int)num();
        else if (k == "w") p.w = (int)num();
        else if (k == "rb") p.rb = (int)num();
        else if (k == "jit") p.jit = (int)num();
        else fail(SPMV_ERR_INVALID_ARG, "plan spec: unknown key " + k);
    }
    if (p.dia != 0 && p.dia != 1) fail(SPMV_ERR_INVALID_ARG, "plan spec: dia must be 0 or 1");
    if (!(p.dia_fill > 0 && p.dia_fill <= 1)) fail(SPMV_ERR_INVALID_ARG, "plan spec: dia_fill must be in (0,1]");
    if (p.drows != 1 && p.drows != 2 && p.drows != 4) fail(SPMV_ERR_INVALID_ARG, "plan spec: drows must be 1, 2 or 4");
    if (p.drows != 1 && !p.dia) fail(SPMV_ERR_INVALID_ARG, "plan spec: drows needs dia=1");
    if (p.heavy < 0) fail(SPMV_ERR_INVALID_ARG, "plan spec: heavy must be >= 0");
    if (p.tile < 64 || p.tile > 65536 || p.tile % 64) fail(SPMV_ERR_INVALID_ARG, "plan spec: tile must be a multiple of 64 in [64, 65536]");
    if (p.lpr != 0 && p.lpr != 256 && (!pow2(p.lpr) || p.lpr > 64))
        fail(SPMV_ERR_INVALID_ARG, "plan spec: lpr must be 0, a power of two <= 64, or 256 (one workgroup per row)");
    if (p.wg != 0 && p.wg != 1) fail(SPMV_ERR_INVALID_ARG, "plan spec: wg must be 0 or 1");
    if (p.wg && p.light != L_BIN) fail(SPMV_ERR_INVALID_ARG, "plan spec: wg needs light=bin");
    if (p.chunk < 0 || (p.chunk > 0 && p.chunk < 64)) fail(SPMV_ERR_INVALID_ARG, "plan spec: chunk must be 0 or >= 64");
    if (p.sigma < -1) fail(SPMV_ERR_INVALID_ARG, "plan spec: sigma must be >= -1");
    if (p.block < 2 || p.block > 4) fail(SPMV_ERR_INVALID_ARG, "plan spec: block must be 2, 3 or 4");
    if (p.smax < 0 || p.smax > 1024) fail(SPMV_ERR_INVALID_ARG, "plan spec: smax must be in [0, 1024]");
    if (p.remap != 0 && p.remap != 1) fail(SPMV_ERR_INVALID_ARG, "plan spec: remap must be 0 or 1");
    if (p.k != 8 && p.k != 16 && p.k != 24 && p.k != 32) fail(SPMV_ERR_INVALID_ARG, "plan spec: k must be 8, 16, 24 or 32");
    if (p.r != 4 && p.r != 8 && p.r != 16) fail(SPMV_ERR_INVALID_ARG, "plan spec: r must be 4, 8 or 16");
    if (p.w != 0 && (p.w < 64 || p.w > 32768 || p.w % 64)) fail(SPMV_ERR_INVALID_ARG, "plan spec: w must be 0 or a multiple of 64 in [64, 32768]");
    if (p.rb < 64 || p.rb > 16384 || p.rb % 64) fail(SPMV_ERR_INVALID_ARG, "plan spec: rb must be a multiple of 64 in [64, 16384]");
    if (p.jit != 0 && p.jit != 1) fail(SPMV_ERR_INVALID_ARG, "plan spec: jit must be 0 or 1");
    if (p.hd != 0 && p.hd != 1) fail(SPMV_ERR_INVALID_ARG, "plan spec: hd must be 0 or 1");
    if (p.hd && !p.heavy) fail(SPMV_ERR_INVALID_ARG, "plan spec: hd needs heavy");
    if (p.piece < 0 || p.piece > 8192 || (p.piece & 3)) fail(SPMV_ERR_INVALID_ARG, "plan spec: piece must be 0 or a multiple of 4 up to 8192");
    if (p.piece && !p.heavy) fail(SPMV_ERR_INVALID_ARG, "plan spec: piece needs heavy");
    if (p.xwin != 0 && p.xwin != 1) fail(SPMV_ERR_INVALID_ARG, "plan spec: xwin must be 0 or 1");
    if (p.xwin && p.light != L_BSELL) fail(SPMV_ERR_INVALID_ARG, "plan spec: xwin needs light=bsell");
    if (p.light == L_BSELL && (p.dia || p.heavy)) fail(SPMV_ERR_INVALID_ARG, "plan spec: bsell cannot be combined with dia or heavy");
    return p;
}

std::string print_spec(const PlanSpec &p) {
    std::ostringstream o;
    if (p.node != N_LEAF) {
        o << (p.node == N_ROWS ? "rows(" : p.node == N_BIN2 ? "bin2(" : p.node == N_CUT ? "cut(" : "cols(");
        for (size_t i = 0; i < p.cuts.size(); ++i) o << (i ? ":" : "") << p.cuts[i];
        o << ")";
        for (const PlanSpec &k : p.kids) o << "{" << print_spec(k) << "}";
        return o.str();
    }
    if (p.dia) o << "dia=1,dia_fill=" << p.dia_fill << ",";
    if (p.dia && p.drows != 1) o << "drows=" << p.drows << ",";
    if (p.heavy) {
        o << "heavy=" << p.heavy << ",tile=" << p.tile << (p.hd ? ",hd=1" : "");
        if (p.piece) o << ",piece=" << p.piece;
        o << ",";
    }
    o << "light=" << light_name(p.light);
    switch (p.light) {
    case L_CSRV: o << ",lpr=" << p.lpr << ",chunk=" << p.chunk << ",sigma=" << p.sigma; break;
    case L_SELL: o << ",sigma=" << p.sigma; break;
    case L_BSELL: o << ",block=" << p.block << ",sigma=" << p.sigma << ",xwin=" << p.xwin; break;
    case L_BIN:
        o << ",smax=" << p.smax << ",sigma=" << p.sigma << ",chunk=" << p.chunk;
        if (p.wg) o << ",wg=1";
        break;
    case L_XS: o << ",k=" << p.k << ",sigma=" << p.sigma; break;
    case L_NNZB: o << ",r=" << p.r; break;
    case L_XNB: o << ",k=" << p.k << ",r=" << p.r; break;
    case L_XL: o << ",w=" << p.w << ",rb=" << p.rb << ",chunk=" << p.chunk; break;
    }
    o << ",remap=" << p.remap;
    if (p.jit) o << ",jit=1";
    return o.str();
}

// The same design as a chain of the paper's operators (Table II).  DIA_EXTRACT, HEAVY_SPLIT and
// DENSE_BLOCK name the three strategies Section VII-F lists as not yet supported by the paper.
static std::string leaf_chain(const PlanSpec &p, bool root);

std::string operator_chain(const PlanSpec &p) {
    if (p.node == N_LEAF) return leaf_chain(p, true);
    std::function<std::string(const PlanSpec &)> walk = [&](const PlanSpec &q) -> std::string {
        if (q.node == N_LEAF) {
            const std::string c = leaf_chain(q, false);
            return c.size() > 4 ? c.substr(4) : c;   // without the leading " -> "
        }
        std::ostringstream o;
        switch (q.node) {
        case N_ROWS:
            o << "ROW_DIV(len";
            for (int64_t c : q.cuts) o << "|" << c;
            o << ")";
            break;
        case N_BIN2: o << "BIN(2^0..2^" << q.cuts[0] << ")"; break;
        case N_CUT: o << "SORT -> ROW_DIV(len[i]>=" << q.cuts[0] << "*len[i+1], >=" << q.cuts[1] << " rows)"; break;
        default: o << "COL_DIV(" << q.cuts[0] << ")"; break;
        }
        o << "{";
        for (size_t i = 0; i < q.kids.size(); ++i) o << (i ? " | " : "") << walk(q.kids[i]);
        o << "}";
        return o.str();
    };
    return "COMPRESS -> " + walk(p);
}

static std::string leaf_chain(const PlanSpec &p, bool root) {
    std::ostringstream o;
    if (root) o << "COMPRESS";
    if (p.dia) o << " -> DIA_EXTRACT(fill>=" << p.dia_fill << ")[BMT_ROW_BLOCK(" << p.drows << ") -> THREAD_TOTAL_RED]";
    if (p.heavy)
        o << " -> ROW_DIV(len>" << p.heavy << ")[HEAVY_SPLIT: COL_DIV(" << p.tile
          << ") -> BMTB_COL_BLOCK" << (p.piece ? " -> BMT_COL_BLOCK(" + std::to_string(p.piece) + ")" : std::string())
          << " -> SORT_BMTB -> BMW_ROW_BLOCK(64) -> BMT_ROW_BLOCK(1) -> BMW_PAD"
          << (p.hd ? " -> COMPRESS(8-bit column deltas)" : "")
          << " -> THREAD_TOTAL_RED -> GMEM_ATOM_RED]";
    auto sort = [&]() {
        if (p.sigma == -1) o << " -> SORT";
        else if (p.sigma > 0) o << " -> SORT_SUB(" << p.sigma << ")";
    };
    switch (p.light) {
    case L_CSRV:
        sort();
        if (p.lpr == 256) o << " -> BMTB_ROW_BLOCK(1) -> BMT_COL_BLOCK(256 lanes)";
        else o << " -> BMW_ROW_BLOCK -> BMT_COL_BLOCK(" << (p.lpr ? std::to_string(p.lpr) : std::string("auto")) << " lanes)";
        if (p.chunk) o << " -> BMW_COL_BLOCK(" << p.chunk << ")";
        o << " -> WARP_TOTAL_RED";
        if (p.lpr == 256) o << " -> SHMEM_TOTAL_RED";
        if (p.chunk) o << " -> GMEM_ATOM_RED";
        break;
    case L_SELL:
        sort();
        o << " -> BMW_ROW_BLOCK(64) -> BMT_ROW_BLOCK(1) -> BMW_PAD -> THREAD_TOTAL_RED";
        break;
    case L_BSELL:
        o << " -> DENSE_BLOCK(" << p.block << "x" << p.block << ")";
        sort();
        if (p.xwin) o << " -> BMTB_ROW_BLOCK(2048)[x window in LDS]";
        o << " -> BMW_ROW_BLOCK(64) -> BMT_ROW_BLOCK(1) -> BMW_PAD -> THREAD_TOTAL_RED";
        break;
    case L_NNZB:
        o << " -> BMW_NNZ_BLOCK(" << 64 * p.r << ") -> BMT_NNZ_BLOCK(" << p.r
          << ") -> THREAD_BITMAP_RED -> WARP_SEG_RED -> GMEM_ATOM_RED(tile borders)";
        break;
    case L_COO:
        o << " -> BMT_NNZ_BLOCK(1) -> GMEM_ATOM_RED";
        break;
    case L_WBM:
        o << " -> BMW_NNZ_BLOCK(" << 64 * kWbmTileSteps << ") -> BMT_NNZ_BLOCK(1) -> WARP_BITMAP_RED -> GMEM_ATOM_RED(tile borders)";
        break;
    case L_XNB:
        o << " -> COL_DIV(" << p.k << " stripes, stripe s on XCD s mod 8) -> BMW_NNZ_BLOCK(" << 64 * p.r
          << ") -> BMT_NNZ_BLOCK(" << p.r << ") -> THREAD_BITMAP_RED -> WARP_SEG_RED -> SCRATCH_ROW_RED(bitmap)";
        break;
    case L_XL:
        o << " -> COL_DIV(" << (p.w ? std::to_string(p.w) : std::string("64 KiB of")) << " columns, x window in LDS) -> BMTB_NNZ_BLOCK("
          << (p.chunk ? std::to_string(p.chunk) : std::string("auto")) << ") -> BMT_NNZ_BLOCK(" << "16 bytes) -> SCRATCH_PRODUCTS"
          << " -> ROW_DIV(" << p.rb << " rows) -> SHMEM_OFFSET_RED";
        break;
    case L_XS:
        o << " -> COL_DIV(" << p.k << " stripes, stripe s on XCD s mod 8)";
        sort();
        o << " -> BMW_ROW_BLOCK(64) -> BMT_ROW_BLOCK(1) -> BMW_PAD -> THREAD_TOTAL_RED -> SCRATCH_ROW_RED";
        break;
    case L_BIN:
        o << " -> BIN(len<=" << p.smax << " | <=128 | >128)";
        sort();
        o << " -> {BMW_ROW_BLOCK(64) -> BMT_ROW_BLOCK(1) -> BMW_PAD -> THREAD_TOTAL_RED"
          << " | BMT_COL_BLOCK(8 lanes) -> WARP_TOTAL_RED"
          << (p.wg ? " | BMTB_ROW_BLOCK(1) -> BMT_COL_BLOCK(256 lanes)" : " | BMT_COL_BLOCK(64 lanes)");
        if (p.chunk) o << " -> BMW_COL_BLOCK(" << p.chunk << ")";
        o << " -> WARP_TOTAL_RED";
        if (p.wg) o << " -> SHMEM_TOTAL_RED";
        if (p.chunk) o << " -> GMEM_ATOM_RED";
        o << "}";
        break;
    }
    if (p.remap) o << " -> SET_RESOURCES(xcd_contiguous)";
    return o.str();
}

}  // namespace spmv
