// Host format builder: CSR + plan spec -> device layout.
//
// This is the paper's Designer plus Format Construction (Sections IV, V-A, V-B): the converting
// operators (ROW_DIV, COL_DIV, SORT, SORT_SUB, BIN) decide which rows go to which part and in
// which order, the mapping operators (*_ROW_BLOCK, *_COL_BLOCK, *_PAD) decide which lane reads
// which stored entry, and only the arrays the part's kernel reads are materialised.  Arrays that
// follow a closed form by construction (first row of a slice = 64 * slice id, origin row of an
// unsorted part = its position) are never built (Section V-D, model-driven compression).
//
// Readings of points the paper leaves open:
//   - SORT / SORT_SUB are stable: rows of equal length keep ascending original order; the windows
//     of SORT_SUB start at the first row of the part and the last one may be short.
//   - PAD fills a slice to the longest row of that slice with value 0 and the column of the row's
//     last real entry (for an empty row: the first column of the slice's first row, 0 if that row
//     is empty too), so padded gathers stay in bounds and inside the slice's window of x.
//   - A row cut by *_COL_BLOCK into several segments reduces through atomics into a y element that
//     an earlier launch set to zero.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <numeric>

#include "internal.h"

namespace spmv {

Plan::~Plan() {
    jit_release_plan(*this);
    for (DevArray &a : arrays)
        if (a.ptr) mem.free(a.ptr, mem.user);
    for (DevArray &a : scratch)
        if (a.ptr) mem.free(a.ptr, mem.user);
}

int64_t Plan::bytes_csr() const {
    const int64_t v = (int64_t)vsize();
    return nnz * (v + 4) + 4 * (nrows + 1) + v * ncols + v * nrows;
}

int64_t Plan::bytes_plan() const {
    int64_t b = 0;
    for (const Part &p : parts) b += p.bytes;
    return b;
}

namespace {

template <typename V>
struct HostBuf {   // uninitialised host storage (large arrays are written exactly once)
    V *p = nullptr;
    int64_t n = 0;
    explicit HostBuf(int64_t count) : n(count) {
        p = (V *)std::malloc((size_t)std::max<int64_t>(count, 1) * sizeof(V));
        if (!p) fail(SPMV_ERR_ALLOC, "host allocation failed");
    }
    ~HostBuf() { std::free(p); }
    HostBuf(const HostBuf &) = delete;
    HostBuf &operator=(const HostBuf &) = delete;
    V &operator[](int64_t i) { return p[i]; }
};

const void *upload(Plan &plan, const std::string &name, int elem_bytes, int64_t count,
                   const void *host, bool read_per_run = true) {
    const size_t bytes = (size_t)std::max<int64_t>(count, 1) * (size_t)elem_bytes;
    void *d = plan.mem.alloc(bytes, plan.mem.user);
    if (!d) fail(SPMV_ERR_ALLOC, "device allocation of " + std::to_string(bytes) + " bytes failed (" + name + ")");
    DevArray a;
    a.name = plan.prefix + name;
    a.ptr = d;
    a.elem_bytes = elem_bytes;
    a.count = count;
    a.read_per_run = read_per_run;
    if (count >= 2 && is_metadata_array(a.name)) a.model = fit_array(host, elem_bytes, count);
    plan.arrays.push_back(a);   // owned from here on, freed by ~Plan
    if (count > 0 && plan.mem.host_only) {
        std::memcpy(d, host, (size_t)count * (size_t)elem_bytes);
    } else if (count > 0) {
        hipError_t err = hipMemcpy(d, host, (size_t)count * (size_t)elem_bytes, hipMemcpyHostToDevice);
        if (err != hipSuccess) fail(SPMV_ERR_HIP, std::string("hipMemcpy H2D (") + name + "): " + hipGetErrorString(err));
    }
    return d;
}

// Algorithmic bytes of one launch of a part: the format arrays it reads (those uploaded since
// `first_array`), plus what it reads of x, reads/writes of scratch and writes (or updates) of y.
void add_part(Plan &plan, Part p, size_t first_array, int64_t x_elems, int64_t scratch_elems,
              int64_t y_elems) {
    const int64_t v = (int64_t)plan.vsize();
    int64_t b = 0;
    for (size_t i = first_array; i < plan.arrays.size(); ++i)
        if (plan.arrays[i].read_per_run) b += plan.arrays[i].count * plan.arrays[i].elem_bytes;
    b += v * (x_elems + scratch_elems + y_elems * (p.accumulate ? 2 : 1));
    p.bytes = b;
    p.name = plan.prefix + p.name;
    plan.parts.push_back(p);
}

// Row order of a part: stable sort by decreasing length inside windows of sigma rows
// (sigma == -1: one window; sigma == 0: untouched).
void sort_rows(std::vector<int32_t> &rows, const std::vector<int64_t> &len_of_row, int sigma, int threads) {
    if (sigma == 0 || rows.size() < 2) return;
    const int64_t n = (int64_t)rows.size();
    const int64_t win = sigma < 0 ? n : (int64_t)sigma;
    const int64_t nwin = (n + win - 1) / win;
    auto cmp = [&](int32_t a, int32_t b) { return len_of_row[(size_t)a] > len_of_row[(size_t)b]; };
    if (nwin == 1) {
        std::stable_sort(rows.begin(), rows.end(), cmp);
        return;
    }
    parallel_for(nwin, 4, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t w = b; w < e; ++w)
            std::stable_sort(rows.begin() + w * win, rows.begin() + std::min(n, (w + 1) * win), cmp);
    });
}

bool is_identity(const std::vector<int32_t> &rows, int64_t nrows) {
    if ((int64_t)rows.size() != nrows) return false;
    for (int64_t i = 0; i < nrows; ++i)
        if (rows[(size_t)i] != (int32_t)i) return false;
    return true;
}

// ---- SELL: slices of 64 rows, lane-interleaved, padded per slice --------------------------------
template <typename T>
void build_sell(Plan &plan, const HostCsr &A, std::vector<int32_t> rows, int sigma, bool acc,
                int remap, const std::string &name, const std::vector<int64_t> &lens, int threads) {
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    const bool ident = (sigma == 0) && is_identity(rows, A.nrows);
    sort_rows(rows, lens, sigma, threads);
    const int64_t nsl = (n + kWave - 1) / kWave;
    std::vector<int64_t> slice_ptr((size_t)nsl + 1, 0);
    int64_t real = 0;
    for (int64_t s = 0; s < nsl; ++s) {
        int64_t w = 0;
        for (int64_t i = s * kWave; i < std::min(n, (s + 1) * kWave); ++i) {
            w = std::max(w, lens[(size_t)rows[(size_t)i]]);
            real += lens[(size_t)rows[(size_t)i]];
        }
        slice_ptr[(size_t)s + 1] = slice_ptr[(size_t)s] + w * kWave;
    }
    const int64_t total = slice_ptr[(size_t)nsl];
    if (total >= ((int64_t)1 << 33)) fail(SPMV_ERR_UNSUPPORTED, "sell: padded size too large");
    HostBuf<int32_t> cols(total);
    HostBuf<T> vals(total);
    const T *av = (const T *)A.val;
    parallel_for(nsl, 64, threads, [&](int64_t sb, int64_t se, int) {
        for (int64_t s = sb; s < se; ++s) {
            const int64_t base = slice_ptr[(size_t)s];
            const int64_t w = (slice_ptr[(size_t)s + 1] - base) / kWave;
            // padding column of empty lanes: the first column of the slice's first row
            const int32_t r0 = rows[(size_t)(s * kWave)];
            const int32_t fallback = lens[(size_t)r0] > 0 ? A.col[A.row_ptr[r0]] : 0;
            for (int lane = 0; lane < kWave; ++lane) {
                const int64_t i = s * kWave + lane;
                int64_t L = 0, src = 0;
                if (i < n) {
                    const int32_t r = rows[(size_t)i];
                    L = lens[(size_t)r];
                    src = A.row_ptr[r];
                }
                int64_t j = 0;
                for (; j < L; ++j) {
                    cols[base + j * kWave + lane] = A.col[src + j];
                    vals[base + j * kWave + lane] = av[src + j];
                }
                const int32_t padc = L > 0 ? A.col[src + L - 1] : fallback;
                for (; j < w; ++j) {
                    cols[base + j * kWave + lane] = padc;
                    vals[base + j * kWave + lane] = T(0);
                }
            }
        }
    });
    Part p;
    p.kind = K_SELL;
    p.name = name;
    p.nrows = n;
    p.nnz = real;
    p.stored = total;
    p.units = nsl;
    p.accumulate = acc;
    p.has_rows = !ident;
    p.remap = remap;
    bool uniform = true;
    for (int64_t s = 1; s < nsl && uniform; ++s)
        uniform = slice_ptr[(size_t)s + 1] - slice_ptr[(size_t)s] == slice_ptr[1] - slice_ptr[0];
    if (uniform) p.uniform_w = (int)((slice_ptr[1] - slice_ptr[0]) / kWave);
    // with one width for all slices the kernel computes the offsets; the array is kept for inspection only
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, name + ".slice_ptr", 8, nsl + 1, slice_ptr.data(), !uniform);
    p.p1 = upload(plan, name + ".cols", 4, total, cols.p);
    p.p2 = upload(plan, name + ".vals", (int)sizeof(T), total, vals.p);
    if (p.has_rows) p.p3 = upload(plan, name + ".origin_rows", 4, n, rows.data());
    add_part(plan, p, a0, std::min<int64_t>(A.ncols, real), 0, n);
}

// ---- CSR segments ----------------------------------------------------------------------------
// zero_rows collects the rows whose segments reduce through atomics.
template <typename T>
void build_csrv(Plan &plan, const HostCsr &A, std::vector<int32_t> rows, int lpr, int64_t chunk,
                int sigma, bool acc, int remap, const std::string &name,
                const std::vector<int64_t> &lens, std::vector<int32_t> &zero_rows, int threads) {
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    int64_t total = 0, maxlen = 0;
    for (int32_t r : rows) {
        total += lens[(size_t)r];
        maxlen = std::max(maxlen, lens[(size_t)r]);
    }
    if (lpr == 0) {   // about four entries per lane, from the mean length of the part
        const double mean = (double)total / (double)n;
        lpr = 1;
        while (lpr < kWave && lpr * 4 < mean) lpr <<= 1;
    }
    const bool split = chunk > 0 && maxlen > chunk;
    const bool ident = !split && sigma == 0 && is_identity(rows, A.nrows);
    Part p;
    p.kind = K_CSRV;
    p.name = name;
    p.nrows = n;
    p.nnz = total;
    p.stored = total;
    p.accumulate = acc;
    p.lanes = lpr;
    p.remap = remap;
    if (ident) {   // the input arrays already are the layout; origin row = segment id
        p.units = n;
        p.has_rows = false;
        // one length for all rows: the kernel computes the offsets, the array is kept for inspection only
        bool uniform = A.nnz < ((int64_t)1 << 31);
        for (int64_t i = 1; i < n && uniform; ++i) uniform = lens[(size_t)i] == lens[0];
        if (uniform) p.uniform_w = (int)lens[0];
        const size_t a0 = plan.arrays.size();
        p.p0 = upload(plan, name + ".seg_ptr", 4, n + 1, A.row_ptr, !uniform);
        p.p2 = upload(plan, name + ".cols", 4, A.nnz, A.col);
        p.p3 = upload(plan, name + ".vals", (int)sizeof(T), A.nnz, A.val);
        add_part(plan, p, a0, std::min<int64_t>(A.ncols, total), 0, n);
        return;
    }
    sort_rows(rows, lens, sigma, threads);
    std::vector<int32_t> seg_ptr, seg_row;
    std::vector<int64_t> row_dst((size_t)n);
    seg_ptr.reserve((size_t)n + 1);
    seg_row.reserve((size_t)n);
    int64_t pos = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int32_t r = rows[(size_t)i];
        const int64_t L = lens[(size_t)r];
        row_dst[(size_t)i] = pos;
        if (split && L > chunk) {
            if (!acc) zero_rows.push_back(r);
            for (int64_t o = 0; o < L; o += chunk) {
                seg_ptr.push_back((int32_t)(pos + o));
                seg_row.push_back(~r);
            }
        } else {
            seg_ptr.push_back((int32_t)pos);
            seg_row.push_back(r);
        }
        pos += L;
    }
    seg_ptr.push_back((int32_t)pos);
    HostBuf<int32_t> cols(total);
    HostBuf<T> vals(total);
    const T *av = (const T *)A.val;
    parallel_for(n, 1024, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = rows[(size_t)i];
            const int64_t L = lens[(size_t)r], src = A.row_ptr[r], dst = row_dst[(size_t)i];
            std::memcpy(cols.p + dst, A.col + src, (size_t)L * 4);
            std::memcpy(vals.p + dst, av + src, (size_t)L * sizeof(T));
        }
    });
    p.units = (int64_t)seg_row.size();
    p.has_rows = true;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, name + ".seg_ptr", 4, (int64_t)seg_ptr.size(), seg_ptr.data());
    p.p1 = upload(plan, name + ".seg_row", 4, (int64_t)seg_row.size(), seg_row.data());
    p.p2 = upload(plan, name + ".cols", 4, total, cols.p);
    p.p3 = upload(plan, name + ".vals", (int)sizeof(T), total, vals.p);
    add_part(plan, p, a0, std::min<int64_t>(A.ncols, total), 0, n);
}

// ---- DIA extraction --------------------------------------------------------------------------
// Entries on the selected diagonals move to a dense (ndiag x ld) array, duplicates add; everything
// else goes to the remainder matrix.
template <typename T>
void build_dia(Plan &plan, const HostCsr &A, const std::vector<int32_t> &offs, OwnedCsr &rem,
               int drows, int threads) {
    const int64_t nd = (int64_t)offs.size();
    const int64_t ld = (A.nrows + kWave - 1) / kWave * kWave;
    HostBuf<T> dv(nd * ld);
    const T *av = (const T *)A.val;
    rem.row_ptr.assign((size_t)A.nrows + 1, 0);
    // pass 1: fill the diagonals, count what is left per row
    parallel_for(A.nrows, 1 << 13, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t r = b; r < e; ++r) {
            for (int64_t d = 0; d < nd; ++d) dv[d * ld + r] = T(0);
            int32_t left = 0;
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                const int32_t off = (int32_t)((int64_t)A.col[k] - r);
                auto it = std::lower_bound(offs.begin(), offs.end(), off);
                if (it != offs.end() && *it == off) dv[(int64_t)(it - offs.begin()) * ld + r] += av[k];
                else ++left;
            }
            rem.row_ptr[(size_t)r + 1] = left;
        }
    });
    for (int64_t d = 0; d < nd; ++d)
        for (int64_t r = A.nrows; r < ld; ++r) dv[d * ld + r] = T(0);
    for (int64_t r = 0; r < A.nrows; ++r) rem.row_ptr[(size_t)r + 1] += rem.row_ptr[(size_t)r];
    const int64_t left = rem.row_ptr[(size_t)A.nrows];
    rem.col.resize((size_t)left);
    rem.val.resize((size_t)left * sizeof(T));
    T *rv = (T *)rem.val.data();
    parallel_for(A.nrows, 1 << 13, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t r = b; r < e; ++r) {
            int64_t dst = rem.row_ptr[(size_t)r];
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                const int32_t off = (int32_t)((int64_t)A.col[k] - r);
                if (!std::binary_search(offs.begin(), offs.end(), off)) {
                    rem.col[(size_t)dst] = A.col[k];
                    rv[dst] = av[k];
                    ++dst;
                }
            }
        }
    });
    rem.view = A;
    rem.view.nnz = left;
    rem.view.row_ptr = rem.row_ptr.data();
    rem.view.col = rem.col.data();
    rem.view.val = rem.val.data();
    Part p;
    p.kind = K_DIA;
    p.name = "dia";
    p.nrows = A.nrows;
    p.nnz = A.nnz - left;
    p.stored = nd * ld;
    p.units = A.nrows;
    p.ndiag = (int)nd;
    p.lanes = nd <= 8 ? drows : 1;   // rows per lane (the kernel for more than eight diagonals has one)
    for (int64_t d = 0; d < std::min<int64_t>(nd, 8); ++d) p.dia_offsets[d] = offs[(size_t)d];
    p.ld = ld;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, "dia.offsets", 4, nd, offs.data());
    p.p1 = upload(plan, "dia.vals", (int)sizeof(T), nd * ld, dv.p);
    add_part(plan, p, a0, A.ncols, 0, A.nrows);
}

// ---- dense B x B blocks in SELL order ----------------------------------------------------------
template <typename T>
void build_bsell(Plan &plan, const HostCsr &A, int B, int sigma, int remap, int xwin, int threads) {
    if (A.nrows % B || A.ncols % B)   // the caller takes a ragged edge off first
        fail(SPMV_ERR_INTERNAL, "bsell: matrix dimensions are not multiples of the block edge");
    const int64_t nb = A.nrows / B;
    if (nb == 0) return;
    // block columns of a block row: merge of the B rows' (col / B), ascending, distinct
    auto block_cols = [&](int64_t br, std::vector<int32_t> &out) {
        out.clear();
        for (int64_t r = br * B; r < (br + 1) * B; ++r)
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) out.push_back(A.col[k] / B);
        std::sort(out.begin(), out.end());
        out.erase(std::unique(out.begin(), out.end()), out.end());
    };
    std::vector<int64_t> nblk((size_t)nb);
    parallel_for(nb, 2048, threads, [&](int64_t b, int64_t e, int) {
        std::vector<int32_t> tmp;
        for (int64_t br = b; br < e; ++br) {
            block_cols(br, tmp);
            nblk[(size_t)br] = (int64_t)tmp.size();
        }
    });
    std::vector<int32_t> brows((size_t)nb);
    std::iota(brows.begin(), brows.end(), 0);
    sort_rows(brows, nblk, sigma, threads);
    const int64_t nsl = (nb + kWave - 1) / kWave;
    std::vector<int64_t> slice_ptr((size_t)nsl + 1, 0);
    int64_t real_blocks = 0;
    for (int64_t s = 0; s < nsl; ++s) {
        int64_t w = 0;
        for (int64_t i = s * kWave; i < std::min(nb, (s + 1) * kWave); ++i) {
            w = std::max(w, nblk[(size_t)brows[(size_t)i]]);
            real_blocks += nblk[(size_t)brows[(size_t)i]];
        }
        slice_ptr[(size_t)s + 1] = slice_ptr[(size_t)s] + w * kWave;
    }
    const int64_t total = slice_ptr[(size_t)nsl];
    const int BB = B * B;
    const int V = 16 / (int)sizeof(T), NV = BB / V;   // values packed per 16-byte load, vectors per block
    if (total * BB >= ((int64_t)1 << 33)) fail(SPMV_ERR_UNSUPPORTED, "bsell: padded size too large");
    HostBuf<int32_t> bcols(total);
    HostBuf<T> vals(total * BB);
    const T *av = (const T *)A.val;
    parallel_for(nsl, 16, threads, [&](int64_t sb, int64_t se, int) {
        std::vector<int32_t> bc;
        for (int64_t s = sb; s < se; ++s) {
            const int64_t base = slice_ptr[(size_t)s];
            const int64_t w = (slice_ptr[(size_t)s + 1] - base) / kWave;
            T *vs = vals.p + base * BB;
            for (int64_t q = 0; q < w * BB * kWave; ++q) vs[q] = T(0);
            int32_t fallback = 0;   // padding column of empty lanes: first block column of the slice's first row
            block_cols(brows[(size_t)(s * kWave)], bc);
            if (!bc.empty()) fallback = bc[0];
            for (int lane = 0; lane < kWave; ++lane) {
                const int64_t i = s * kWave + lane;
                bc.clear();
                if (i < nb) {
                    const int64_t br = brows[(size_t)i];
                    block_cols(br, bc);
                    for (int ri = 0; ri < B; ++ri) {
                        const int64_t r = br * B + ri;
                        size_t j = 0;
                        for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                            const int32_t b = A.col[k] / B;
                            while (bc[j] != b) ++j;   // columns ascend, so j only moves forward
                            const int q = ri * B + (A.col[k] - b * B);
                            // record of block j: NV vectors of V values per lane, then the rest
                            T *rec = vs + (int64_t)j * BB * kWave;
                            if (q < NV * V) rec[((int64_t)(q / V) * kWave + lane) * V + (q % V)] += av[k];
                            else rec[(int64_t)NV * V * kWave + (int64_t)(q - NV * V) * kWave + lane] += av[k];
                        }
                    }
                }
                const int64_t L = (int64_t)bc.size();
                for (int64_t j = 0; j < L; ++j) bcols[base + j * kWave + lane] = bc[(size_t)j];
                const int32_t padc = L > 0 ? bc[(size_t)L - 1] : fallback;
                for (int64_t j = L; j < w; ++j) bcols[base + j * kWave + lane] = padc;
            }
        }
    });
    Part p;
    p.kind = K_BSELL;
    p.name = "bsell";
    p.nrows = nb;
    p.nnz = A.nnz;
    p.stored = total * BB;
    p.units = nsl;
    p.block = B;
    p.has_rows = sigma != 0;
    p.remap = remap;
    const size_t a0 = plan.arrays.size();
    std::vector<uint16_t> bcols16;
    if (xwin) {
        // x window of each group of 32 slices: [lo, lo + n) in scalar columns
        const int64_t ng = (nsl + kXwinGroup - 1) / kXwinGroup;
        std::vector<int32_t> win((size_t)(2 * ng), 0);
        std::atomic<int64_t> widest{0};
        parallel_for(ng, 4, threads, [&](int64_t gb, int64_t ge, int) {
            for (int64_t g = gb; g < ge; ++g) {
                const int64_t b0 = slice_ptr[(size_t)(g * kXwinGroup)];
                const int64_t b1 = slice_ptr[(size_t)std::min(nsl, (g + 1) * kXwinGroup)];
                int32_t lo = INT32_MAX, hi = -1;
                for (int64_t i = b0; i < b1; ++i) {
                    lo = std::min(lo, bcols[i]);
                    hi = std::max(hi, bcols[i]);
                }
                if (hi < 0) lo = 0;
                win[(size_t)(2 * g)] = lo * B;
                win[(size_t)(2 * g + 1)] = (hi - lo + 1) * B;
                int64_t n = (int64_t)(hi - lo + 1) * B, cur = widest.load();
                while (n > cur && !widest.compare_exchange_weak(cur, n)) {}
            }
        });
        if (widest.load() * (int64_t)sizeof(T) > kXwinMaxBytes)
            fail(SPMV_ERR_UNSUPPORTED, "bsell: the x window of a workgroup does not fit the LDS");
        p.lds_bytes = std::max<int64_t>(widest.load() * (int64_t)sizeof(T), 16);
        // Do the block rows of every group stay inside the group's own range of 64 * 32 block rows
        // (no sort, or SORT_SUB windows that are whole groups)?  Then the kernel collects a group's
        // results in LDS, where the x window was, and writes them to y as one contiguous piece.
        bool confined = true;
        for (int64_t i = 0; i < nb && confined; ++i)
            confined = brows[(size_t)i] / (kWave * kXwinGroup) == i / (kWave * kXwinGroup);
        if (confined) {
            p.uniform_w = 1;   // bsell with a window: results staged in LDS
            p.lds_bytes = std::max<int64_t>(p.lds_bytes, (int64_t)kWave * kXwinGroup * B * (int64_t)sizeof(T));
        }
        p.p4 = upload(plan, "bsell.xwin", 4, 2 * ng, win.data());
        // index compression: a block's column as a 16-bit offset from its group's window
        if (widest.load() / B >= 65536) fail(SPMV_ERR_UNSUPPORTED, "bsell: the x window of a workgroup is too wide for 16-bit columns");
        bcols16.resize((size_t)total);
        parallel_for(ng, 4, threads, [&](int64_t gb, int64_t ge, int) {
            for (int64_t g = gb; g < ge; ++g) {
                const int64_t b0 = slice_ptr[(size_t)(g * kXwinGroup)];
                const int64_t b1 = slice_ptr[(size_t)std::min(nsl, (g + 1) * kXwinGroup)];
                const int32_t lo = win[(size_t)(2 * g)] / B;
                for (int64_t i = b0; i < b1; ++i) bcols16[(size_t)i] = (uint16_t)(bcols[i] - lo);
            }
        });
    }
    p.p0 = upload(plan, "bsell.slice_ptr", 8, nsl + 1, slice_ptr.data());
    if (xwin) p.p1 = upload(plan, "bsell.bcols16", 2, total, bcols16.data());
    else p.p1 = upload(plan, "bsell.bcols", 4, total, bcols.p);
    p.p2 = upload(plan, "bsell.vals", (int)sizeof(T), total * BB, vals.p);
    if (p.has_rows) p.p3 = upload(plan, "bsell.origin_brows", 4, nb, brows.data());
    add_part(plan, p, a0, A.ncols, 0, A.nrows);
    (void)real_blocks;
}

// A heavy part whose partial sums are added by the two-pass reduce launch of the same leaf instead
// of a launch of their own.
struct HeavyFold {
    // made by the leaf: heavy rows hptr[b] .. hptr[b+1]-1 lie in block b of the two-pass part, at local rows hloc
    std::vector<int32_t> hptr;
    std::vector<uint16_t> hloc;
    // made by the heavy part: workgroup g leaves the sum of heavy row h at partial[g * nh + h]
    void *partial = nullptr;
    int64_t ngroups = 0;
};

// ---- heavy rows in column stripes --------------------------------------------------------------
// COL_DIV into stripes of `tile` columns; inside a stripe SORT_BMTB orders the heavy rows by the
// number of entries they have there (stable, decreasing), slices of 64 rows are padded to their
// longest segment (value 0, local column 0) and stored lane-interleaved.
//
// delta = 1 (index compression): a lane's columns are stored as 8-bit differences to the previous
// column of the same (row, stripe) segment.  lane_meta[u*64 + lane] = first local column << 16 |
// heavy row (0xFFFF: none); the difference of the first entry is 0; a gap g > 255 is bridged by
// (g - 1) / 255 entries (difference 255, value 0) in front of the real entry; padding is
// (difference 0, value 0).  The rows of a stripe are ordered by the stored length of their segments
// (entries + bridges), and a slice's width is rounded up to a multiple of 4: the differences of
// entries 4q .. 4q+3 of a lane form one 32-bit word (entry 4q in the low byte) at word
// unit_ptr[u] / 4 + 64*q + lane.
//
// piece = P > 0: the entries of a (row, stripe) segment are cut into runs of at most P stored entries
// (greedily: a run takes entries while its stored length, bridging entries included, stays within P),
// each run a lane of its own, so that a few very long segments no longer set the padded width of a
// whole slice; rows without entries in a stripe take no lane there.  sunits[s] is the
// first unit of stripe s (piece = 0: every stripe has ceil(nh / 64) units and there is no such
// array).  A stripe that would need more than 8192 lanes doubles its P until it does not.
template <typename T>
void build_stripe(Plan &plan, const HostCsr &A, const std::vector<int32_t> &hrows, int tile, int delta, int piece,
                  bool acc, const std::vector<int64_t> &lens, int threads, HeavyFold *fold = nullptr) {
    const int64_t nh = (int64_t)hrows.size();
    if (nh == 0) return;
    // the x tile and one accumulator per heavy row share the 160 KiB of a compute unit (tiles above 64 KiB
    // leave room for one workgroup only, which then has 1024 lanes)
    if (((size_t)tile + (size_t)hrows.size()) * sizeof(T) > 160 * 1024 || (size_t)tile * sizeof(T) > 128 * 1024)
        fail(SPMV_ERR_UNSUPPORTED, "heavy: x tile and row accumulators do not fit the LDS");
    if (nh > 8192) fail(SPMV_ERR_UNSUPPORTED, "heavy: more than 8192 heavy rows (their accumulators live in LDS)");
    const int64_t ns = (A.ncols + tile - 1) / tile;
    int64_t total = 0;
    for (int32_t r : hrows) total += lens[(size_t)r];
    auto bridges = [](int64_t gap) { return gap > 255 ? (gap - 1) / 255 : (int64_t)0; };
    // seg_len[s * nh + h] and seg_off[s * nh + h]: the entries of heavy row h inside stripe s are
    // A[row_ptr[r] + seg_off .. + seg_len)   (columns ascend inside a row)
    std::vector<int32_t> seg_len((size_t)(ns * nh), 0), seg_off((size_t)(ns * nh), 0);
    parallel_for(nh, 4, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t h = b; h < e; ++h) {
            const int32_t r = hrows[(size_t)h];
            const int64_t beg = A.row_ptr[r];
            for (int64_t k = beg; k < A.row_ptr[r + 1]; ++k) {
                const size_t i = (size_t)((int64_t)(A.col[k] / tile) * nh + h);
                if (seg_len[i]++ == 0) seg_off[i] = (int32_t)(k - beg);
            }
        }
    });
    // A lane holds one run of consecutive entries of a heavy row inside a stripe: the whole
    // (row, stripe) segment, or (piece > 0) one piece of it.  key = its stored length.
    struct Lane {
        int32_t h, off, len, key;
    };
    auto stored_len = [&](int32_t h, int32_t off, int32_t len) -> int32_t {
        if (!delta || len == 0) return len;
        const int64_t src = (int64_t)A.row_ptr[hrows[(size_t)h]] + off;
        int64_t n = len;
        for (int64_t k = 1; k < len; ++k) n += bridges((int64_t)A.col[src + k] - A.col[src + k - 1]);
        return (int32_t)n;
    };
    std::vector<std::vector<Lane>> lanes((size_t)ns);
    parallel_for(ns, 1, threads, [&](int64_t sb, int64_t se, int) {
        for (int64_t s = sb; s < se; ++s) {
            std::vector<Lane> &ls = lanes[(size_t)s];
            const int32_t *sl = seg_len.data() + s * nh, *so = seg_off.data() + s * nh;
            if (piece <= 0) {
                for (int32_t h = 0; h < (int32_t)nh; ++h) ls.push_back({h, so[h], sl[h], stored_len(h, so[h], sl[h])});
            } else {
                // A piece takes entries while its stored length stays within P (with column differences a
                // piece that ends in front of a wide gap starts the next one at that gap's far side, so the
                // bridging entries of the gap are not stored at all).  P doubles until the stripe has at
                // most 8192 lanes (128 units).
                for (int64_t P = piece;; P *= 2) {
                    ls.clear();
                    for (int32_t h = 0; h < (int32_t)nh; ++h) {
                        const int64_t src = (int64_t)A.row_ptr[hrows[(size_t)h]] + so[h];
                        int32_t o = 0;
                        while (o < sl[h]) {
                            int32_t len = 1;
                            int64_t stored = 1;
                            while (o + len < sl[h]) {
                                const int64_t add = 1 + (delta ? bridges((int64_t)A.col[src + o + len] - A.col[src + o + len - 1]) : 0);
                                if (stored + add > P) break;
                                stored += add;
                                ++len;
                            }
                            ls.push_back({h, so[h] + o, len, (int32_t)stored});
                            o += len;
                        }
                    }
                    if (ls.size() <= 8192) break;
                }
            }
            std::stable_sort(ls.begin(), ls.end(), [](const Lane &a, const Lane &b) { return a.key > b.key; });
        }
    });
    // units: slices of 64 lanes, padded to their first (longest) lane
    std::vector<int32_t> sunits((size_t)ns + 1, 0);
    for (int64_t s = 0; s < ns; ++s) {
        const int64_t nu = ((int64_t)lanes[(size_t)s].size() + kWave - 1) / kWave;
        if (sunits[(size_t)s] + nu >= ((int64_t)1 << 22)) fail(SPMV_ERR_UNSUPPORTED, "heavy: too many (row, stripe) segments");
        sunits[(size_t)s + 1] = (int32_t)(sunits[(size_t)s] + nu);
    }
    const int64_t nunits = sunits[(size_t)ns];
    int64_t nsl = 0;   // units of the largest stripe
    for (int64_t s = 0; s < ns; ++s) nsl = std::max<int64_t>(nsl, sunits[(size_t)s + 1] - sunits[(size_t)s]);
    std::vector<int32_t> unit_ptr((size_t)nunits + 1, 0), unit_stripe((size_t)nunits, 0);
    int64_t padded = 0;
    for (int64_t s = 0; s < ns; ++s)
        for (int64_t u = sunits[(size_t)s]; u < sunits[(size_t)s + 1]; ++u) {
            int64_t w = lanes[(size_t)s][(size_t)((u - sunits[(size_t)s]) * kWave)].key;
            if (delta) w = (w + 3) / 4 * 4;
            padded += w * kWave;
            if (padded >= ((int64_t)1 << 31)) fail(SPMV_ERR_UNSUPPORTED, "heavy: too many entries");
            unit_ptr[(size_t)u + 1] = (int32_t)padded;
            unit_stripe[(size_t)u] = (int32_t)s;
        }
    std::vector<uint16_t> lane_row;
    std::vector<uint32_t> lane_meta;
    if (delta) lane_meta.assign((size_t)(nunits * kWave), 0xFFFFu);
    else lane_row.assign((size_t)(nunits * kWave), (uint16_t)0xFFFF);
    HostBuf<uint16_t> lcol(delta ? 0 : padded);
    HostBuf<uint8_t> dcol(delta ? padded : 0);
    HostBuf<T> vals(padded);
    const T *av = (const T *)A.val;
    parallel_for(nunits, 8, threads, [&](int64_t ub, int64_t ue, int) {
        for (int64_t u = ub; u < ue; ++u) {
            const int64_t s = unit_stripe[(size_t)u], base = unit_ptr[(size_t)u];
            const int64_t w = (unit_ptr[(size_t)u + 1] - base) / kWave;
            const std::vector<Lane> &ls = lanes[(size_t)s];
            for (int lane = 0; lane < kWave; ++lane) {
                const int64_t li = (u - sunits[(size_t)s]) * kWave + lane;
                const bool have = li < (int64_t)ls.size();
                const uint16_t h = have ? (uint16_t)ls[(size_t)li].h : (uint16_t)0xFFFF;
                const int64_t L = have ? ls[(size_t)li].len : 0;
                const int64_t src = have ? (int64_t)A.row_ptr[hrows[h]] + ls[(size_t)li].off : 0;
                int64_t j = 0;
                if (!delta) {
                    lane_row[(size_t)(u * kWave + lane)] = h;
                    for (; j < L; ++j) {
                        lcol[base + j * kWave + lane] = (uint16_t)(A.col[src + j] - s * tile);
                        vals[base + j * kWave + lane] = av[src + j];
                    }
                    for (; j < w; ++j) {
                        lcol[base + j * kWave + lane] = 0;
                        vals[base + j * kWave + lane] = T(0);
                    }
                    continue;
                }
                // byte of entry j: word base/4 + 64*(j/4) + lane, byte j%4 (little endian)
                auto put = [&](int64_t jj, uint8_t d, T v) {
                    dcol[base + (jj / 4) * 4 * kWave + (int64_t)lane * 4 + jj % 4] = d;
                    vals[base + jj * kWave + lane] = v;
                };
                const uint32_t col0 = L ? (uint32_t)(A.col[src] - s * tile) : 0u;
                lane_meta[(size_t)(u * kWave + lane)] = (col0 << 16) | (uint32_t)h;
                for (int64_t k = 0; k < L; ++k) {
                    int64_t gap = k ? (int64_t)A.col[src + k] - A.col[src + k - 1] : 0;
                    for (; gap > 255; gap -= 255) put(j++, 255, T(0));
                    put(j++, (uint8_t)gap, av[src + k]);
                }
                for (; j < w; ++j) put(j, 0, T(0));
            }
        }
    });
    // workgroups: a few consecutive stripes each, about two workgroups per compute unit
    // Two workgroups of 512 lanes per compute unit when their x tiles and row accumulators both fit its
    // LDS (160 KiB), else one of 1024 lanes: sixteen wavefronts per compute unit either way.
    const bool big = 2 * ((int64_t)tile + nh) * (int64_t)sizeof(T) > 160 * 1024;
    const int64_t per_group = std::max<int64_t>(1, ns / (big ? 256 : 512));
    const int64_t ngroups = (ns + per_group - 1) / per_group;
    void *scratch = plan.mem.alloc((size_t)(ngroups * nh) * sizeof(T), plan.mem.user);
    if (!scratch) fail(SPMV_ERR_ALLOC, "device allocation of the heavy part's scratch failed");
    {
        DevArray a;
        a.name = plan.prefix + "heavy.scratch";
        a.ptr = scratch;
        a.elem_bytes = (int)sizeof(T);
        a.count = ngroups * nh;
        plan.scratch.push_back(a);
    }
    Part p;
    p.kind = K_STRIPE;
    p.name = "heavy";
    p.nrows = nh;
    p.nnz = total;
    p.stored = padded;
    p.units = ns;
    p.nslices = nsl;
    p.ngroups = ngroups;
    p.per_group = per_group;
    p.scratch = scratch;
    p.tile = tile;
    p.delta = delta;
    p.lanes = big ? 1024 : 512;
    p.has_rows = true;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, "heavy.unit_ptr", 4, nunits + 1, unit_ptr.data());
    if (delta) p.p1 = upload(plan, "heavy.dcols", 4, padded / 4, dcol.p);
    else p.p1 = upload(plan, "heavy.lcols", 2, padded, lcol.p);
    p.p2 = upload(plan, "heavy.vals", (int)sizeof(T), padded, vals.p);
    p.p3 = upload(plan, "heavy.rows", 4, nh, hrows.data());
    if (delta) p.p4 = upload(plan, "heavy.lane_meta", 4, nunits * kWave, lane_meta.data());
    else p.p4 = upload(plan, "heavy.lane_row", 2, nunits * kWave, lane_row.data());
    if (piece > 0) p.p5 = upload(plan, "heavy.sunits", 4, ns + 1, sunits.data());
    plan.arrays[a0 + 3].read_per_run = false;   // heavy.rows is read by the reduce launch
    add_part(plan, p, a0, A.ncols, ngroups * nh, 0);
    plan.arrays[a0 + 3].read_per_run = fold == nullptr;
    if (fold) {   // the two-pass reduce launch of the same leaf adds the partial sums
        fold->partial = scratch;
        fold->ngroups = ngroups;
        return;
    }
    Part r;   // sums the workgroups' partial sums into y (overwrites, or adds after a DIA part)
    r.kind = K_REDUCE_WIDE;
    r.name = "heavy.reduce";
    r.nrows = nh;
    r.units = nh;
    r.ngroups = ngroups;
    r.scratch = scratch;
    r.accumulate = acc;
    r.has_rows = true;
    r.p3 = p.p3;
    add_part(plan, r, plan.arrays.size(), 0, ngroups * nh + nh / 2, nh);   // + heavy.rows (4 bytes each)
}

// ---- COO -----------------------------------------------------------------------------------------
// One (row, column, value) triple per stored entry of the part's rows, in row order.  Every row of
// the part is zeroed first: all sums go through atomics.
template <typename T>
void build_coo(Plan &plan, const HostCsr &A, const std::vector<int32_t> &rows, bool acc,
               const std::vector<int64_t> &lens, std::vector<int32_t> &zero_rows, int threads) {
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    std::vector<int64_t> start((size_t)n + 1, 0);
    for (int64_t i = 0; i < n; ++i) start[(size_t)i + 1] = start[(size_t)i] + lens[(size_t)rows[(size_t)i]];
    const int64_t total = start[(size_t)n];
    if (!acc) zero_rows.insert(zero_rows.end(), rows.begin(), rows.end());
    HostBuf<int32_t> er(total), ec(total);
    HostBuf<T> ev(total);
    const T *av = (const T *)A.val;
    parallel_for(n, 1024, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = rows[(size_t)i];
            const int64_t src = A.row_ptr[r], L = lens[(size_t)r], dst = start[(size_t)i];
            for (int64_t k = 0; k < L; ++k) er[dst + k] = r;
            std::memcpy(ec.p + dst, A.col + src, (size_t)L * 4);
            std::memcpy(ev.p + dst, av + src, (size_t)L * sizeof(T));
        }
    });
    Part p;
    p.kind = K_COO;
    p.name = "coo";
    p.nrows = n;
    p.nnz = total;
    p.stored = total;
    p.units = total;
    p.has_rows = true;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, "coo.rows", 4, total, er.p);
    p.p1 = upload(plan, "coo.cols", 4, total, ec.p);
    p.p2 = upload(plan, "coo.vals", (int)sizeof(T), total, ev.p);
    add_part(plan, p, a0, std::min<int64_t>(A.ncols, total), 0, 2 * total);   // one read-modify-write of y per entry
}

// ---- nnz-balanced tiles ----------------------------------------------------------------------------
// The non-empty rows of the part, in order, form one stream of entries; tile i holds entries
// [64*R*i, 64*R*(i+1)), lane l of the tile the R consecutive entries from 64*R*i + R*l, stored
// transposed (entry t of lane l at 64*R*i + 64*t + l).  The stream's tail is padded with
// (value 0, column 0).  bits[64*i + l] marks the entries of the lane that start a row.  Rows open
// at a tile border are accumulated with atomics and therefore zeroed first; empty rows too.
template <typename T>
void build_nnzb(Plan &plan, const HostCsr &A, const std::vector<int32_t> &rows_in, int R, bool acc,
                const std::vector<int64_t> &lens, std::vector<int32_t> &zero_rows, int threads) {
    std::vector<int32_t> rows;
    rows.reserve(rows_in.size());
    for (int32_t r : rows_in) {
        if (lens[(size_t)r] > 0) rows.push_back(r);
        else if (!acc) zero_rows.push_back(r);
    }
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    std::vector<int64_t> start((size_t)n + 1, 0);   // position of each row's first entry in the stream
    for (int64_t i = 0; i < n; ++i) start[(size_t)i + 1] = start[(size_t)i] + lens[(size_t)rows[(size_t)i]];
    const int64_t total = start[(size_t)n];
    const int64_t tile_sz = (int64_t)kWave * R;
    const int64_t ntiles = (total + tile_sz - 1) / tile_sz;
    if (ntiles * tile_sz >= ((int64_t)1 << 31)) fail(SPMV_ERR_UNSUPPORTED, "nnzb: too many entries");
    HostBuf<int32_t> cols(ntiles * tile_sz);
    HostBuf<T> vals(ntiles * tile_sz);
    std::vector<uint16_t> bits((size_t)(ntiles * kWave), 0);
    std::vector<int32_t> tile_row((size_t)ntiles + 1, 0);
    const T *av = (const T *)A.val;
    // entries: parallel over rows; marks: one per row
    parallel_for(n, 1024, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = rows[(size_t)i];
            const int64_t src = A.row_ptr[r], L = lens[(size_t)r];
            for (int64_t k = 0; k < L; ++k) {
                const int64_t g = start[(size_t)i] + k;          // position in the stream
                const int64_t tile = g / tile_sz, in = g % tile_sz;
                const int64_t dst = tile * tile_sz + (in % R) * kWave + in / R;
                cols[dst] = A.col[src + k];
                vals[dst] = av[src + k];
            }
        }
    });
    for (int64_t g = total; g < ntiles * tile_sz; ++g) {
        const int64_t tile = g / tile_sz, in = g % tile_sz;
        const int64_t dst = tile * tile_sz + (in % R) * kWave + in / R;
        cols[dst] = 0;
        vals[dst] = T(0);
    }
    for (int64_t i = 0; i < n; ++i) {
        const int64_t g = start[(size_t)i];
        const int64_t tile = g / tile_sz, in = g % tile_sz;
        bits[(size_t)(tile * kWave + in / R)] |= (uint16_t)(1u << (in % R));
        tile_row[(size_t)tile + 1] += 1;
    }
    for (int64_t t = 0; t < ntiles; ++t) tile_row[(size_t)t + 1] += tile_row[(size_t)t];
    // rows open at a tile border: the row holding a tile's last entry, and the row holding its
    // first entry when that entry does not start a row
    if (!acc) {
        for (int64_t t = 0; t < ntiles; ++t) {
            const int64_t last = std::min(total, (t + 1) * tile_sz) - 1;
            const int64_t i_last = (int64_t)(std::upper_bound(start.begin(), start.end(), last) - start.begin()) - 1;
            zero_rows.push_back(rows[(size_t)i_last]);
            const int64_t first = t * tile_sz;
            const int64_t i_first = (int64_t)(std::upper_bound(start.begin(), start.end(), first) - start.begin()) - 1;
            if (start[(size_t)i_first] != first) zero_rows.push_back(rows[(size_t)i_first]);
        }
        std::sort(zero_rows.begin(), zero_rows.end());
        zero_rows.erase(std::unique(zero_rows.begin(), zero_rows.end()), zero_rows.end());
    }
    Part p;
    p.kind = K_NNZB;
    p.name = "nnzb";
    p.nrows = n;
    p.nnz = total;
    p.stored = ntiles * tile_sz;
    p.units = ntiles;
    p.lanes = R;
    p.accumulate = acc;
    p.has_rows = true;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, "nnzb.cols", 4, ntiles * tile_sz, cols.p);
    p.p1 = upload(plan, "nnzb.vals", (int)sizeof(T), ntiles * tile_sz, vals.p);
    if (R <= 8) {
        std::vector<uint8_t> b8(bits.begin(), bits.end());
        p.p2 = upload(plan, "nnzb.bits", 1, ntiles * kWave, b8.data());
    } else {
        p.p2 = upload(plan, "nnzb.bits", 2, ntiles * kWave, bits.data());
    }
    p.p3 = upload(plan, "nnzb.tile_row", 4, ntiles + 1, tile_row.data());
    p.p4 = upload(plan, "nnzb.rows", 4, n, rows.data());
    add_part(plan, p, a0, std::min<int64_t>(A.ncols, total), 0, n);
}

// ---- one entry per lane, one bitmap per wavefront step ----------------------------------------------
// The same stream as build_nnzb (the non-empty rows' entries in order), stored as it is: entry g at
// position g, padded with (value 0, column 0) to a whole tile of 64 * kWbmTileSteps entries.
// mask[g / 64] has bit g % 64 set when entry g starts a row; tile_row[i] = row starts before tile i.
// Rows open at a tile border are accumulated with atomics and therefore zeroed first; empty rows too.
template <typename T>
void build_wbm(Plan &plan, const HostCsr &A, const std::vector<int32_t> &rows_in, bool acc,
               const std::vector<int64_t> &lens, std::vector<int32_t> &zero_rows, int threads) {
    std::vector<int32_t> rows;
    rows.reserve(rows_in.size());
    for (int32_t r : rows_in) {
        if (lens[(size_t)r] > 0) rows.push_back(r);
        else if (!acc) zero_rows.push_back(r);
    }
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    std::vector<int64_t> start((size_t)n + 1, 0);
    for (int64_t i = 0; i < n; ++i) start[(size_t)i + 1] = start[(size_t)i] + lens[(size_t)rows[(size_t)i]];
    const int64_t total = start[(size_t)n];
    const int64_t tile_sz = (int64_t)kWave * kWbmTileSteps;
    const int64_t ntiles = (total + tile_sz - 1) / tile_sz;
    if (ntiles * tile_sz >= ((int64_t)1 << 31)) fail(SPMV_ERR_UNSUPPORTED, "wbm: too many entries");
    HostBuf<int32_t> cols(ntiles * tile_sz);
    HostBuf<T> vals(ntiles * tile_sz);
    std::vector<uint64_t> mask((size_t)(ntiles * kWbmTileSteps), 0);
    std::vector<int32_t> tile_row((size_t)ntiles + 1, 0);
    const T *av = (const T *)A.val;
    parallel_for(n, 1024, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = rows[(size_t)i];
            const int64_t L = lens[(size_t)r], src = A.row_ptr[r], dst = start[(size_t)i];
            std::memcpy(cols.p + dst, A.col + src, (size_t)L * 4);
            std::memcpy(vals.p + dst, av + src, (size_t)L * sizeof(T));
        }
    });
    for (int64_t g = total; g < ntiles * tile_sz; ++g) {
        cols[g] = 0;
        vals[g] = T(0);
    }
    for (int64_t i = 0; i < n; ++i) {
        const int64_t g = start[(size_t)i];
        mask[(size_t)(g / kWave)] |= (uint64_t)1 << (g % kWave);
        tile_row[(size_t)(g / tile_sz) + 1] += 1;
    }
    for (int64_t t = 0; t < ntiles; ++t) tile_row[(size_t)t + 1] += tile_row[(size_t)t];
    if (!acc) {
        for (int64_t t = 0; t < ntiles; ++t) {
            const int64_t last = std::min(total, (t + 1) * tile_sz) - 1;
            const int64_t i_last = (int64_t)(std::upper_bound(start.begin(), start.end(), last) - start.begin()) - 1;
            zero_rows.push_back(rows[(size_t)i_last]);
            const int64_t first = t * tile_sz;
            const int64_t i_first = (int64_t)(std::upper_bound(start.begin(), start.end(), first) - start.begin()) - 1;
            if (start[(size_t)i_first] != first) zero_rows.push_back(rows[(size_t)i_first]);
        }
        std::sort(zero_rows.begin(), zero_rows.end());
        zero_rows.erase(std::unique(zero_rows.begin(), zero_rows.end()), zero_rows.end());
    }
    Part p;
    p.kind = K_WBM;
    p.name = "wbm";
    p.nrows = n;
    p.nnz = total;
    p.stored = ntiles * tile_sz;
    p.units = ntiles;
    p.accumulate = acc;
    p.has_rows = true;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, "wbm.cols", 4, ntiles * tile_sz, cols.p);
    p.p1 = upload(plan, "wbm.vals", (int)sizeof(T), ntiles * tile_sz, vals.p);
    p.p2 = upload(plan, "wbm.mask", 8, ntiles * kWbmTileSteps, mask.data());
    p.p3 = upload(plan, "wbm.tile_row", 4, ntiles + 1, tile_row.data());
    p.p4 = upload(plan, "wbm.rows", 4, n, rows.data());
    add_part(plan, p, a0, std::min<int64_t>(A.ncols, total), 0, n);
}

// ---- XCD-striped nnz-balanced tiles ------------------------------------------------------------------
// COL_DIV into K stripes of W columns as for the striped SELL.  The (row, stripe) segments of a
// stripe follow each other in part order as one stream, cut into tiles of 64*R entries (transposed
// as in build_nnzb); a stripe's stream is padded to a whole tile with (value 0, the stripe's first
// column).  Streams are laid out XCD by XCD.  Segments are numbered in stream order; segment q sums
// into scratch[q].  For the reduce launch, mask[w*K + s] has bit b set when row 64w+b of the part has
// entries in stripe s, and pbase[w*K + s] is the number of the first such segment.
template <typename T>
void build_xnb(Plan &plan, const HostCsr &A, const std::vector<int32_t> &rows, int K, int R, bool acc,
               const std::vector<int64_t> &lens, int threads) {
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    const bool ident = is_identity(rows, A.nrows);
    int64_t W = (A.ncols + K - 1) / K;
    W = std::max<int64_t>(kWave, (W + kWave - 1) / kWave * kWave);
    const int64_t tsz = (int64_t)kWave * R;
    const int64_t chunk = 1 << 16;                    // rows per work item, a multiple of 1024
    const int64_t nchunks = (n + chunk - 1) / chunk;
    int64_t real = 0;
    for (int32_t r : rows) real += lens[(size_t)r];
    // pass A: entries and segments per (chunk, stripe)
    std::vector<int64_t> cnt_e((size_t)(nchunks * K), 0), cnt_q((size_t)(nchunks * K), 0);
    parallel_for(nchunks, 1, threads, [&](int64_t cb, int64_t ce, int) {
        for (int64_t c = cb; c < ce; ++c)
            for (int64_t i = c * chunk; i < std::min(n, (c + 1) * chunk); ++i) {
                const int32_t r = rows[(size_t)i];
                int64_t prev = -1;
                for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                    const int64_t s = A.col[k] / W;
                    cnt_e[(size_t)(c * K + s)] += 1;
                    if (s != prev) cnt_q[(size_t)(c * K + s)] += 1;
                    prev = s;
                }
            }
    });
    // stream layout: XCD k owns stripes k, k+8, ...; every stripe starts on a tile boundary
    std::vector<int64_t> stream_base((size_t)K, 0), seg_base((size_t)K, 0), seg_cnt((size_t)K, 0), stripe_len((size_t)K, 0), xbase(9, 0);
    int64_t ntiles = 0, nsegs = 0;
    for (int k = 0; k < 8; ++k) {
        xbase[(size_t)k] = ntiles;
        for (int s = k; s < K; s += 8) {
            int64_t le = 0, lq = 0;
            for (int64_t c = 0; c < nchunks; ++c) {
                le += cnt_e[(size_t)(c * K + s)];
                lq += cnt_q[(size_t)(c * K + s)];
            }
            stream_base[(size_t)s] = ntiles * tsz;
            seg_base[(size_t)s] = nsegs;
            stripe_len[(size_t)s] = le;
            seg_cnt[(size_t)s] = lq;
            ntiles += (le + tsz - 1) / tsz;
            nsegs += lq;
        }
    }
    xbase[8] = ntiles;
    if (ntiles * tsz >= ((int64_t)1 << 31) || nsegs >= ((int64_t)1 << 31))
        fail(SPMV_ERR_UNSUPPORTED, "xnb: too many entries");
    // turn the per-chunk counts into starting positions
    for (int s = 0; s < K; ++s) {
        int64_t e = stream_base[(size_t)s], q = seg_base[(size_t)s];
        for (int64_t c = 0; c < nchunks; ++c) {
            const int64_t de = cnt_e[(size_t)(c * K + s)], dq = cnt_q[(size_t)(c * K + s)];
            cnt_e[(size_t)(c * K + s)] = e;
            cnt_q[(size_t)(c * K + s)] = q;
            e += de;
            q += dq;
        }
    }
    HostBuf<int32_t> cols(ntiles * tsz);
    HostBuf<T> vals(ntiles * tsz);
    HostBuf<uint8_t> mark(ntiles * tsz);
    std::memset(mark.p, 0, (size_t)(ntiles * tsz));
    const int64_t nblk = (n + kReduceBlockRows - 1) / kReduceBlockRows;
    std::vector<uint16_t> seg_row((size_t)std::max<int64_t>(nsegs, 1), 0);
    std::vector<int32_t> bbase((size_t)((nblk + 1) * K), 0);
    const T *av = (const T *)A.val;
    auto transposed = [&](int64_t g) {
        const int64_t tile = g / tsz, in = g % tsz;
        return tile * tsz + (in % R) * kWave + in / R;
    };
    // pass B: place the entries, mark the segment starts, fill the reduce tables
    parallel_for(nchunks, 1, threads, [&](int64_t cb, int64_t ce, int) {
        std::vector<int64_t> run_e((size_t)K), run_q((size_t)K);
        for (int64_t c = cb; c < ce; ++c) {
            for (int s = 0; s < K; ++s) {
                run_e[(size_t)s] = cnt_e[(size_t)(c * K + s)];
                run_q[(size_t)s] = cnt_q[(size_t)(c * K + s)];
            }
            for (int64_t i = c * chunk; i < std::min(n, (c + 1) * chunk); ++i) {
                if (i % kReduceBlockRows == 0)
                    for (int s = 0; s < K; ++s)
                        bbase[(size_t)((i / kReduceBlockRows) * K + s)] = (int32_t)run_q[(size_t)s];
                const int32_t r = rows[(size_t)i];
                int64_t prev = -1;
                for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                    const int64_t s = A.col[k] / W;
                    const int64_t g = run_e[(size_t)s]++;
                    const int64_t dst = transposed(g);
                    cols[dst] = A.col[k];
                    vals[dst] = av[k];
                    if (s != prev) {
                        mark[g] = 1;
                        seg_row[(size_t)run_q[(size_t)s]] = (uint16_t)(i % kReduceBlockRows);
                        run_q[(size_t)s] += 1;
                    }
                    prev = s;
                }
            }
        }
    });
    for (int s = 0; s < K; ++s)   // end of every stripe's segments
        bbase[(size_t)(nblk * K + s)] = (int32_t)(seg_base[(size_t)s] + seg_cnt[(size_t)s]);
    for (int s = 0; s < K; ++s) {   // pad every stripe's last tile
        const int64_t b = stream_base[(size_t)s] + stripe_len[(size_t)s];
        const int64_t e = stream_base[(size_t)s] + (stripe_len[(size_t)s] + tsz - 1) / tsz * tsz;
        const int32_t padc = (int32_t)std::min<int64_t>((int64_t)s * W, A.ncols - 1);
        for (int64_t g = b; g < e; ++g) {
            cols[transposed(g)] = padc < 0 ? 0 : padc;
            vals[transposed(g)] = T(0);
        }
    }
    // lane bitmaps, segment starts per tile, scratch slots open at a tile border
    std::vector<uint16_t> bits((size_t)(ntiles * kWave), 0);
    std::vector<int32_t> tile_row((size_t)ntiles + 1, 0);
    parallel_for(ntiles, 256, threads, [&](int64_t tb, int64_t te, int) {
        for (int64_t t = tb; t < te; ++t) {
            int32_t cnt = 0;
            for (int lane = 0; lane < kWave; ++lane) {
                uint16_t bm = 0;
                for (int q = 0; q < R; ++q)
                    if (mark[t * tsz + (int64_t)lane * R + q]) bm |= (uint16_t)(1u << q);
                bits[(size_t)(t * kWave + lane)] = bm;
                cnt += __builtin_popcount(bm);
            }
            tile_row[(size_t)t + 1] = cnt;
        }
    });
    for (int64_t t = 0; t < ntiles; ++t) tile_row[(size_t)t + 1] += tile_row[(size_t)t];
    std::vector<int32_t> open_slots;
    for (int64_t t = 0; t < ntiles; ++t) {
        if (!mark[t * tsz]) open_slots.push_back(tile_row[(size_t)t] - 1);
        open_slots.push_back(tile_row[(size_t)t + 1] - 1);
    }
    std::sort(open_slots.begin(), open_slots.end());
    open_slots.erase(std::unique(open_slots.begin(), open_slots.end()), open_slots.end());

    void *scratch = plan.mem.alloc((size_t)std::max<int64_t>(nsegs, 1) * sizeof(T), plan.mem.user);
    if (!scratch) fail(SPMV_ERR_ALLOC, "device allocation of the striped part's scratch failed");
    {
        DevArray a;
        a.name = plan.prefix + "xnb.scratch";
        a.ptr = scratch;
        a.elem_bytes = (int)sizeof(T);
        a.count = nsegs;
        plan.scratch.push_back(a);
    }
    if (!open_slots.empty()) {
        Part z;
        z.kind = K_ZERO_SCRATCH;
        z.name = "xnb.zero";
        z.nrows = (int64_t)open_slots.size();
        z.units = z.nrows;
        z.scratch = scratch;
        const size_t a0 = plan.arrays.size();
        z.p0 = upload(plan, "xnb.open_slots", 4, z.nrows, open_slots.data());
        add_part(plan, z, a0, 0, z.nrows, 0);
    }
    int64_t per_xcd = 0;
    for (int k = 0; k < 8; ++k) per_xcd = std::max(per_xcd, xbase[(size_t)k + 1] - xbase[(size_t)k]);
    Part p;
    p.kind = K_XNB;
    p.name = "xnb";
    p.nrows = n;
    p.nnz = real;
    p.stored = ntiles * tsz;
    p.units = ntiles;
    p.ngroups = (per_xcd + 3) / 4;
    p.lanes = R;
    p.scratch = scratch;
    p.has_rows = !ident;
    const size_t a1 = plan.arrays.size();
    p.p0 = upload(plan, "xnb.cols", 4, ntiles * tsz, cols.p);
    p.p1 = upload(plan, "xnb.vals", (int)sizeof(T), ntiles * tsz, vals.p);
    if (R <= 8) {
        std::vector<uint8_t> b8(bits.begin(), bits.end());
        p.p2 = upload(plan, "xnb.bits", 1, ntiles * kWave, b8.data());
    } else {
        p.p2 = upload(plan, "xnb.bits", 2, ntiles * kWave, bits.data());
    }
    p.p3 = upload(plan, "xnb.tile_row", 4, ntiles + 1, tile_row.data());
    p.p4 = upload(plan, "xnb.xbase", 8, 9, xbase.data());
    add_part(plan, p, a1, std::min<int64_t>(A.ncols, real), nsegs, 0);
    Part r;
    r.kind = K_REDUCE_LDS;
    r.name = "xnb.reduce";
    r.nrows = n;
    r.units = n;
    r.lanes = K;
    r.scratch = scratch;
    r.accumulate = acc;
    r.has_rows = !ident;
    const size_t a2 = plan.arrays.size();
    r.p0 = upload(plan, "xnb.seg_row", 2, nsegs, seg_row.data());
    r.p1 = upload(plan, "xnb.bbase", 4, (nblk + 1) * K, bbase.data());
    if (!ident) r.p3 = upload(plan, "xnb.rows", 4, n, rows.data());
    add_part(plan, r, a2, 0, nsegs, n);
}

// ---- two passes with x windows in LDS --------------------------------------------------------------
// COL_DIV into windows of W columns (an LDS-sized piece of x), ROW_DIV of the part into blocks of RB
// rows (an LDS-sized piece of y).  Entry (part position i, column c) belongs to run (s, b) =
// (c / W, i / RB); runs are stored window by window, inside a window block by block, inside a run
// by part position and then in row order.  A run is padded to a whole 16-byte vector (N = 2 doubles or
// 4 floats) and a window to 16 entries, with (value 0, local column 0): padding a run to 16 entries
// would cost 7.5 entries per run, a tenth of everything this part streams when the runs are short.
// Entry g holds vals[g] and lcol[g] = c - s*W; its product goes to scratch[g].  The multiply launch
// works through items (s, first entry, end entry): a window's entries cut into equal pieces of at most
// `chunk` entries (128 KiB of values unless the spec says otherwise), multiples of 16.
// The reduce launch of block b adds the groups glist[gptr[b]] .. glist[gptr[b+1] - 1]: the runs (0, b),
// (1, b), ... in that order, each cut into groups of up to 16 entries; a list entry is
// 8 * (first entry / N) + (entries in the group / N - 1).  The local rows i - b*RB are stored in list
// order, 16 slots per group (lrow[16*p + t] belongs to entry N*(glist[p] >> 3) + t; unused slots 0), so
// a block reads them as one contiguous piece.
// Row r contributes its first lens[r] entries: the caller passes 0 for rows that belong to another
// part but are kept in `rows` so that the part's rows are one contiguous range (no row map to read,
// y written contiguously; the other part's launch overwrites those y elements afterwards).
template <typename T>
void build_xl(Plan &plan, const HostCsr &A, const std::vector<int32_t> &rows, int w_spec, int RB,
              int64_t chunk_spec, bool acc, const std::vector<int64_t> &lens, int threads,
              const HeavyFold *fold = nullptr) {
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    const bool ident = is_identity(rows, A.nrows);
    const int64_t W = w_spec > 0 ? w_spec : (int64_t)(65536 / sizeof(T));
    if (W * (int64_t)sizeof(T) > kXlMaxLds) fail(SPMV_ERR_UNSUPPORTED, "xl: the x window does not fit in LDS");
    if ((int64_t)RB * 8 > kXlMaxLds) fail(SPMV_ERR_UNSUPPORTED, "xl: the row block does not fit in LDS");
    const int64_t S = std::max<int64_t>(1, (A.ncols + W - 1) / W);
    const int64_t B = (n + RB - 1) / RB;
    if (S * B > ((int64_t)1 << 26)) fail(SPMV_ERR_UNSUPPORTED, "xl: too many (window, row block) runs");
    const int64_t G = kXlGroup, N = 16 / (int64_t)sizeof(T);
    int64_t real = 0;
    for (int32_t r : rows) real += lens[(size_t)r];
    // entries per run (run j = s * B + b)
    std::vector<int64_t> start((size_t)(S * B) + 1, 0), cnt((size_t)(S * B), 0);
    parallel_for(B, 1, threads, [&](int64_t bb, int64_t be, int) {
        for (int64_t b = bb; b < be; ++b)
            for (int64_t i = b * RB; i < std::min(n, (b + 1) * RB); ++i) {
                const int32_t r = rows[(size_t)i];
                for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r] + lens[(size_t)r]; ++k)
                    cnt[(size_t)((A.col[k] / W) * B + b)] += 1;
            }
    });
    // first entry of every run: runs padded to N, windows to 16
    {
        int64_t pos = 0;
        for (int64_t s = 0; s < S; ++s) {
            for (int64_t b = 0; b < B; ++b) {
                start[(size_t)(s * B + b)] = pos;
                pos += (cnt[(size_t)(s * B + b)] + N - 1) / N * N;
            }
            pos = (pos + G - 1) / G * G;
        }
        start[(size_t)(S * B)] = pos;
    }
    const int64_t tot = start[(size_t)(S * B)];
    if (tot >= ((int64_t)1 << 28) * N) fail(SPMV_ERR_UNSUPPORTED, "xl: too many entries");
    // group list of the reduce launch: block b reads the groups of runs (0, b), (1, b), ...
    auto groups_of = [&](int64_t j) { return ((cnt[(size_t)j] + N - 1) / N * N + G - 1) / G; };
    std::vector<int32_t> gptr((size_t)B + 1, 0);
    for (int64_t b = 0; b < B; ++b) {
        int64_t c = 0;
        for (int64_t s = 0; s < S; ++s) c += groups_of(s * B + b);
        if (gptr[(size_t)b] + c >= ((int64_t)1 << 27)) fail(SPMV_ERR_UNSUPPORTED, "xl: too many groups");
        gptr[(size_t)b + 1] = (int32_t)(gptr[(size_t)b] + c);
    }
    const int64_t ngroups = gptr[(size_t)B];
    HostBuf<T> vals(tot);
    HostBuf<uint16_t> lcol(tot), lrow(ngroups * G);
    HostBuf<int32_t> glist(ngroups);
    const T *av = (const T *)A.val;
    parallel_for(B, 1, threads, [&](int64_t bb, int64_t be, int) {
        std::vector<int64_t> cur((size_t)S), lpos((size_t)S);
        for (int64_t b = bb; b < be; ++b) {
            int64_t o = gptr[(size_t)b];
            for (int64_t s = 0; s < S; ++s) {
                const int64_t j = s * B + b, g0 = start[(size_t)j], padded = (cnt[(size_t)j] + N - 1) / N * N;
                cur[(size_t)s] = g0;
                lpos[(size_t)s] = o * G;           // the run's place in the block's own order
                for (int64_t off = 0; off < padded; off += G) {
                    const int64_t len = std::min<int64_t>(G, padded - off);
                    for (int64_t t = len; t < G; ++t) lrow[o * G + t] = 0;   // slots past a short group
                    glist[o++] = (int32_t)(((g0 + off) / N) * 8 + (len / N - 1));
                }
            }
            for (int64_t i = b * RB; i < std::min(n, (b + 1) * RB); ++i) {
                const int32_t r = rows[(size_t)i];
                for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r] + lens[(size_t)r]; ++k) {
                    const int64_t s = A.col[k] / W;
                    const int64_t g = cur[(size_t)s]++;
                    vals[g] = av[k];
                    lcol[g] = (uint16_t)(A.col[k] - s * W);
                    lrow[lpos[(size_t)s]++] = (uint16_t)(i - b * RB);
                }
            }
            for (int64_t s = 0; s < S; ++s) {   // the padding of every run to a whole vector
                const int64_t j = s * B + b, pe = start[(size_t)j] + (cnt[(size_t)j] + N - 1) / N * N;
                for (int64_t g = cur[(size_t)s]; g < pe; ++g) {
                    vals[g] = T(0);
                    lcol[g] = 0;
                    lrow[lpos[(size_t)s]++] = 0;
                }
            }
        }
    });
    for (int64_t s = 0; s < S; ++s) {   // the padding of every window to 16 entries
        const int64_t last = s * B + B - 1;
        const int64_t pb = start[(size_t)last] + (cnt[(size_t)last] + N - 1) / N * N, pe = start[(size_t)last + 1];
        for (int64_t g = pb; g < pe; ++g) {
            vals[g] = T(0);
            lcol[g] = 0;
        }
    }
    // Items of the multiply launch.  Workgroup i runs on XCD i mod 8, and every XCD has an L2 of its own:
    // all items of a window get numbers of one residue mod 8, one after the other, so that only the
    // first of them stages the window from memory and the others find it in that XCD's L2.  Windows are
    // dealt, in order, to the residue with the fewest items so far (the lowest on a tie); residues that
    // end up shorter are filled with empty items (0, 0, 0), which return at once.
    const int64_t chunk = chunk_spec > 0 ? (chunk_spec + G - 1) / G * G : 131072 / (int64_t)sizeof(T);
    std::vector<int32_t> lane_items[8];
    int64_t staged = 0;   // elements of x that one launch brings in from memory: every non-empty window once
    for (int64_t s = 0; s < S; ++s) {
        const int64_t b0 = start[(size_t)(s * B)], e0 = start[(size_t)((s + 1) * B)];
        if (e0 == b0) continue;
        staged += std::min<int64_t>(W, A.ncols - s * W);
        const int64_t m = (e0 - b0 + chunk - 1) / chunk;
        const int64_t per = ((e0 - b0 + m - 1) / m + G - 1) / G * G;
        int l = 0;
        for (int k = 1; k < 8; ++k)
            if (lane_items[k].size() < lane_items[l].size()) l = k;
        for (int64_t c = b0; c < e0; c += per) {
            lane_items[l].push_back((int32_t)s);
            lane_items[l].push_back((int32_t)c);
            lane_items[l].push_back((int32_t)std::min(e0, c + per));
        }
    }
    size_t longest = 0;
    for (int k = 0; k < 8; ++k) longest = std::max(longest, lane_items[k].size() / 3);
    std::vector<int32_t> items;
    items.reserve(longest * 24);
    for (size_t j = 0; j < longest; ++j)
        for (int k = 0; k < 8; ++k)
            for (int t = 0; t < 3; ++t) items.push_back(3 * j + t < lane_items[k].size() ? lane_items[k][3 * j + t] : 0);
    const int64_t nitems = (int64_t)items.size() / 3;
    void *scratch = plan.mem.alloc((size_t)std::max<int64_t>(tot, 1) * sizeof(T), plan.mem.user);
    if (!scratch) fail(SPMV_ERR_ALLOC, "device allocation of the xl part's scratch failed");
    {
        DevArray a;
        a.name = plan.prefix + "xl.scratch";
        a.ptr = scratch;
        a.elem_bytes = (int)sizeof(T);
        a.count = tot;
        plan.scratch.push_back(a);
    }
    if (nitems > 0) {
        Part p;
        p.kind = K_XL_MUL;
        p.name = "xl";
        p.nrows = n;
        p.nnz = real;
        p.stored = tot;
        p.units = nitems;
        p.tile = (int)W;
        p.scratch = scratch;
        const size_t a1 = plan.arrays.size();
        p.p0 = upload(plan, "xl.items", 4, 3 * nitems, items.data());
        p.p1 = upload(plan, "xl.vals", (int)sizeof(T), tot, vals.p);
        p.p2 = upload(plan, "xl.lcol", 2, tot, lcol.p);
        add_part(plan, p, a1, staged, tot, 0);
    }
    Part r;
    r.kind = K_XL_REDUCE;
    r.name = "xl.reduce";
    r.nrows = n;
    r.units = B;
    r.tile = RB;
    r.scratch = scratch;
    r.accumulate = acc;
    r.has_rows = !ident;
    const size_t a2 = plan.arrays.size();
    r.p0 = upload(plan, "xl.gptr", 4, B + 1, gptr.data());
    r.p1 = upload(plan, "xl.glist", 4, ngroups, glist.p);
    r.p2 = upload(plan, "xl.lrow", 2, ngroups * G, lrow.p);
    if (!ident) r.p3 = upload(plan, "xl.rows", 4, n, rows.data());
    int64_t partials = 0;
    if (fold) {
        // the leaf's heavy rows are rows of this part (without entries): block b adds the heavy
        // launch's partial sums of the heavy rows hptr[b] .. hptr[b+1]-1, whose local rows are hloc
        if ((int64_t)fold->hptr.size() != B + 1) fail(SPMV_ERR_INTERNAL, "xl: heavy rows counted for other row blocks");
        const int64_t nh = (int64_t)fold->hloc.size();
        r.p4 = upload(plan, "xl.hptr", 4, B + 1, fold->hptr.data());
        r.p5 = upload(plan, "xl.hloc", 2, nh, fold->hloc.data());
        r.scratch2 = fold->partial;
        r.ngroups = fold->ngroups;
        r.nslices = nh;
        partials = fold->ngroups * nh;
    }
    add_part(plan, r, a2, 0, tot + partials, n);
}

// ---- XCD-striped SELL ----------------------------------------------------------------------------
// COL_DIV into K stripes of W = ceil(ncols / K) columns (rounded up to 64).  Per stripe: the rows
// of the part that have entries in it, in windows of sigma part positions, sorted by that count
// (stable, decreasing), cut into slices of 64 and padded per slice.  Units (slices) are laid out
// XCD by XCD (XCD k owns stripes k, k + 8, ...), stripe by stripe, window by window.  Lane l of unit
// u owns scratch slot 64*u + l; pslot lists the slots of every row (stripe order), pptr delimits them.
template <typename T>
void build_xs(Plan &plan, const HostCsr &A, const std::vector<int32_t> &rows, int K, int sigma, bool acc,
              const std::vector<int64_t> &lens, int threads) {
    const int64_t n = (int64_t)rows.size();
    if (n == 0) return;
    const bool ident = is_identity(rows, A.nrows);
    int64_t W = (A.ncols + K - 1) / K;
    W = std::max<int64_t>(kWave, (W + kWave - 1) / kWave * kWave);
    const int64_t win = sigma <= 0 ? n : (int64_t)sigma;
    const int64_t nwin = (n + win - 1) / win;
    // segment lengths, row-major: seg[i * K + s]
    HostBuf<int32_t> seg(n * K);
    std::vector<int32_t> pptr((size_t)n + 1, 0);
    int64_t real = 0;
    for (int32_t r : rows) real += lens[(size_t)r];
    parallel_for(n, 1 << 12, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            int32_t *sg = seg.p + i * K;
            for (int s = 0; s < K; ++s) sg[s] = 0;
            const int32_t r = rows[(size_t)i];
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) sg[A.col[k] / W] += 1;
            int32_t cnt = 0;
            for (int s = 0; s < K; ++s) cnt += sg[s] > 0;
            pptr[(size_t)i + 1] = cnt;
        }
    });
    for (int64_t i = 0; i < n; ++i) pptr[(size_t)i + 1] += pptr[(size_t)i];
    const int64_t nslots = pptr[(size_t)n];
    // participants per (stripe, window), in memory order: XCD, phase (stripe = 8*phase + xcd), window
    std::vector<int> stripe_order;
    for (int k = 0; k < 8; ++k)
        for (int s = k; s < K; s += 8) stripe_order.push_back(s);
    const int64_t ncell = (int64_t)K * nwin;            // cell c = position in stripe_order * nwin + window
    std::vector<int64_t> cell_units((size_t)ncell + 1, 0);
    parallel_for(ncell, 4, threads, [&](int64_t cb, int64_t ce, int) {
        for (int64_t c = cb; c < ce; ++c) {
            const int s = stripe_order[(size_t)(c / nwin)];
            const int64_t w0 = (c % nwin) * win, w1 = std::min(n, w0 + win);
            int64_t cnt = 0;
            for (int64_t i = w0; i < w1; ++i) cnt += seg[i * K + s] > 0;
            cell_units[(size_t)c + 1] = (cnt + kWave - 1) / kWave;
        }
    });
    for (int64_t c = 0; c < ncell; ++c) cell_units[(size_t)c + 1] += cell_units[(size_t)c];
    const int64_t nunits = cell_units[(size_t)ncell];
    std::vector<int64_t> xbase(9, 0);
    {
        size_t pos = 0;
        for (int k = 0; k < 8; ++k) {
            xbase[(size_t)k] = cell_units[pos * (size_t)nwin];
            for (int s = k; s < K; s += 8) ++pos;
        }
        xbase[8] = nunits;
    }
    // sort each cell, record the lanes' part positions and the unit widths
    HostBuf<int32_t> lane_i(nunits * kWave);
    std::vector<int64_t> unit_ptr((size_t)nunits + 1, 0);
    parallel_for(ncell, 1, threads, [&](int64_t cb, int64_t ce, int) {
        std::vector<int32_t> part;
        for (int64_t c = cb; c < ce; ++c) {
            const int s = stripe_order[(size_t)(c / nwin)];
            const int64_t w0 = (c % nwin) * win, w1 = std::min(n, w0 + win);
            part.clear();
            for (int64_t i = w0; i < w1; ++i)
                if (seg[i * K + s] > 0) part.push_back((int32_t)i);
            std::stable_sort(part.begin(), part.end(), [&](int32_t a, int32_t b) {
                return seg[(int64_t)a * K + s] > seg[(int64_t)b * K + s];
            });
            const int64_t u0 = cell_units[(size_t)c];
            const int64_t cnt = (int64_t)part.size();
            for (int64_t q = 0; q < (cnt + kWave - 1) / kWave * kWave; ++q)
                lane_i[u0 * kWave + q] = q < cnt ? part[(size_t)q] : -1;
            for (int64_t u = u0; u < cell_units[(size_t)c + 1]; ++u)
                unit_ptr[(size_t)u + 1] = (int64_t)seg[(int64_t)part[(size_t)((u - u0) * kWave)] * K + s] * kWave;
        }
    });
    for (int64_t u = 0; u < nunits; ++u) unit_ptr[(size_t)u + 1] += unit_ptr[(size_t)u];
    const int64_t total = unit_ptr[(size_t)nunits];
    if (total >= ((int64_t)1 << 33)) fail(SPMV_ERR_UNSUPPORTED, "xs: padded size too large");
    // stripe of every unit (needed to find the segment inside the row)
    std::vector<int32_t> unit_stripe((size_t)nunits);
    for (int64_t c = 0; c < ncell; ++c)
        for (int64_t u = cell_units[(size_t)c]; u < cell_units[(size_t)c + 1]; ++u)
            unit_stripe[(size_t)u] = stripe_order[(size_t)(c / nwin)];
    HostBuf<int32_t> cols(total), pslot(nslots);
    HostBuf<T> vals(total);
    const T *av = (const T *)A.val;
    parallel_for(nunits, 64, threads, [&](int64_t ub, int64_t ue, int) {
        for (int64_t u = ub; u < ue; ++u) {
            const int s = unit_stripe[(size_t)u];
            const int64_t base = unit_ptr[(size_t)u], w = (unit_ptr[(size_t)u + 1] - base) / kWave;
            int32_t fallback = 0;
            for (int lane = 0; lane < kWave; ++lane) {
                const int32_t i = lane_i[u * kWave + lane];
                int64_t L = 0, src = 0;
                if (i >= 0) {
                    const int32_t *sg = seg.p + (int64_t)i * K;
                    int64_t off = 0;
                    int32_t rank = 0;
                    for (int t = 0; t < s; ++t) {
                        off += sg[t];
                        rank += sg[t] > 0;
                    }
                    L = sg[s];
                    src = (int64_t)A.row_ptr[rows[(size_t)i]] + off;
                    pslot[pptr[(size_t)i] + rank] = (int32_t)(u * kWave + lane);
                    if (lane == 0) fallback = A.col[src];
                }
                int64_t j = 0;
                for (; j < L; ++j) {
                    cols[base + j * kWave + lane] = A.col[src + j];
                    vals[base + j * kWave + lane] = av[src + j];
                }
                const int32_t padc = L > 0 ? A.col[src + L - 1] : fallback;
                for (; j < w; ++j) {
                    cols[base + j * kWave + lane] = padc;
                    vals[base + j * kWave + lane] = T(0);
                }
            }
        }
    });
    if (nunits * kWave >= ((int64_t)1 << 31)) fail(SPMV_ERR_UNSUPPORTED, "xs: too many segments");
    void *scratch = plan.mem.alloc((size_t)std::max<int64_t>(nunits * kWave, 1) * sizeof(T), plan.mem.user);
    if (!scratch) fail(SPMV_ERR_ALLOC, "device allocation of the striped part's scratch failed");
    {
        DevArray a;
        a.name = plan.prefix + "xs.scratch";
        a.ptr = scratch;
        a.elem_bytes = (int)sizeof(T);
        a.count = nunits * kWave;
        plan.scratch.push_back(a);
    }
    int64_t per_xcd = 0;
    for (int k = 0; k < 8; ++k) per_xcd = std::max(per_xcd, xbase[(size_t)k + 1] - xbase[(size_t)k]);
    Part p;
    p.kind = K_XS;
    p.name = "xs";
    p.nrows = n;
    p.nnz = real;
    p.stored = total;
    p.units = nunits;
    p.ngroups = (per_xcd + 3) / 4;   // workgroups per XCD, four slices each
    p.scratch = scratch;
    p.has_rows = !ident;
    const size_t a0 = plan.arrays.size();
    p.p0 = upload(plan, "xs.unit_ptr", 8, nunits + 1, unit_ptr.data());
    p.p1 = upload(plan, "xs.cols", 4, total, cols.p);
    p.p2 = upload(plan, "xs.vals", (int)sizeof(T), total, vals.p);
    p.p4 = upload(plan, "xs.xbase", 8, 9, xbase.data());
    add_part(plan, p, a0, std::min<int64_t>(A.ncols, real), nunits * kWave, 0);
    Part r;
    r.kind = K_REDUCE_ROWS;
    r.name = "xs.reduce";
    r.nrows = n;
    r.units = n;
    r.scratch = scratch;
    r.accumulate = acc;
    r.has_rows = !ident;
    const size_t a1 = plan.arrays.size();
    r.p0 = upload(plan, "xs.pptr", 4, n + 1, pptr.data());
    r.p1 = upload(plan, "xs.pslot", 4, nslots, pslot.p);
    if (!ident) r.p3 = upload(plan, "xs.rows", 4, n, rows.data());
    add_part(plan, r, a1, 0, nslots, n);
}

// Copy of A with ascending columns inside each row (stable: repeated columns keep their order).
template <typename T>
void sorted_copy(const HostCsr &A, OwnedCsr &out, int threads) {
    out.row_ptr.assign(A.row_ptr, A.row_ptr + A.nrows + 1);
    out.col.resize((size_t)A.nnz);
    out.val.resize((size_t)A.nnz * sizeof(T));
    const T *av = (const T *)A.val;
    T *ov = (T *)out.val.data();
    parallel_for(A.nrows, 1 << 12, threads, [&](int64_t b, int64_t e, int) {
        std::vector<int32_t> idx;
        for (int64_t r = b; r < e; ++r) {
            const int64_t s = A.row_ptr[r], L = A.len(r);
            idx.resize((size_t)L);
            std::iota(idx.begin(), idx.end(), 0);
            std::stable_sort(idx.begin(), idx.end(), [&](int32_t x, int32_t y) { return A.col[s + x] < A.col[s + y]; });
            for (int64_t k = 0; k < L; ++k) {
                out.col[(size_t)(s + k)] = A.col[s + idx[(size_t)k]];
                ov[s + k] = av[s + idx[(size_t)k]];
            }
        }
    });
    out.view = A;
    out.view.row_ptr = out.row_ptr.data();
    out.view.col = out.col.data();
    out.view.val = out.val.data();
}

// One leaf of the plan tree: a flat design applied to the rows `rows` (ascending) of A.  `whole`:
// the rows are all rows of the matrix the plan was made for and A is that matrix (needed by the
// designs that work on the whole matrix).  `span`, when given, lists the rows a two-pass leaf should
// own as rows without entries beside its own (see build_node); acc: y += instead of y =.
template <typename T>
void build_leaf(Plan &plan, const HostCsr &A0, const Census &cen, const PlanSpec &spec,
                const std::vector<int32_t> &rows, bool whole, bool acc, const std::vector<int32_t> *span,
                int threads) {
    OwnedCsr rem;
    const HostCsr *cur = &A0;
    if (spec.dia) {
        if (!whole || acc) fail(SPMV_ERR_UNSUPPORTED, "dia: works on the whole matrix only");
        // offsets whose population reaches dia_fill (the census kept those >= 0.5)
        std::vector<int32_t> offs = cen.diag_offsets;
        if (spec.dia_fill > 0.5) {
            // recount is not needed for the common case; thresholds above 0.5 filter by an exact pass
            std::vector<int64_t> cnt(offs.size(), 0);
            for (int64_t r = 0; r < cur->nrows; ++r)
                for (int64_t k = cur->row_ptr[r]; k < cur->row_ptr[r + 1]; ++k) {
                    auto it = std::lower_bound(offs.begin(), offs.end(), (int32_t)((int64_t)cur->col[k] - r));
                    if (it != offs.end() && *it == (int32_t)((int64_t)cur->col[k] - r)) cnt[(size_t)(it - offs.begin())] += 1;
                }
            std::vector<int32_t> keep;
            for (size_t d = 0; d < offs.size(); ++d) {
                const int64_t off = offs[d];
                const int64_t valid = std::min<int64_t>(cur->nrows, cur->ncols - off) - std::max<int64_t>(0, -off);
                if (valid > 0 && (double)cnt[d] >= spec.dia_fill * (double)valid) keep.push_back(offs[d]);
            }
            offs.swap(keep);
        }
        if (offs.empty()) fail(SPMV_ERR_UNSUPPORTED, "dia: the matrix has no diagonal populated enough");
        build_dia<T>(plan, *cur, offs, rem, spec.drows, threads);
        cur = &rem.view;
        acc = true;
        if (cur->nnz == 0) return;
    }
    const HostCsr &A = *cur;
    std::vector<int64_t> lens((size_t)A.nrows, 0);
    parallel_for((int64_t)rows.size(), 1 << 16, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) lens[(size_t)rows[(size_t)i]] = A.len(rows[(size_t)i]);
    });

    if (spec.light == L_BSELL) {
        if (!whole || acc) fail(SPMV_ERR_UNSUPPORTED, "bsell: works on the whole matrix only");
        const int B = spec.block;
        const int64_t nrB = A.nrows / B * B, ncB = A.ncols / B * B;
        if (nrB == A.nrows && ncB == A.ncols) {
            build_bsell<T>(plan, A, B, spec.sigma, spec.remap, spec.xwin, threads);
            return;
        }
        // Ragged edge: the last nrows mod B rows and the last ncols mod B columns do not fill whole
        // blocks.  The blocked part takes the matrix without them; their entries form a CSR part
        // that accumulates afterwards, and the rows past the last whole block row are zeroed first.
        if (nrB == 0 || ncB == 0) fail(SPMV_ERR_UNSUPPORTED, "bsell: the matrix is smaller than one block");
        OwnedCsr main, rest;
        main.row_ptr.assign((size_t)nrB + 1, 0);
        rest.row_ptr.assign((size_t)A.nrows + 1, 0);
        for (int64_t r = 0; r < A.nrows; ++r) {
            int64_t in = 0, out = 0;
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) (r < nrB && A.col[k] < ncB ? in : out) += 1;
            if (r < nrB) main.row_ptr[(size_t)r + 1] = (int32_t)(main.row_ptr[(size_t)r] + in);
            rest.row_ptr[(size_t)r + 1] = (int32_t)(rest.row_ptr[(size_t)r] + out);
        }
        const size_t v = sizeof(T);
        main.col.resize((size_t)main.row_ptr[(size_t)nrB]);
        main.val.resize(main.col.size() * v);
        rest.col.resize((size_t)rest.row_ptr[(size_t)A.nrows]);
        rest.val.resize(rest.col.size() * v);
        const T *av = (const T *)A.val;
        for (int64_t r = 0; r < A.nrows; ++r) {
            int64_t im = r < nrB ? main.row_ptr[(size_t)r] : 0, ir = rest.row_ptr[(size_t)r];
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) {
                if (r < nrB && A.col[k] < ncB) {
                    main.col[(size_t)im] = A.col[k];
                    ((T *)main.val.data())[im++] = av[k];
                } else {
                    rest.col[(size_t)ir] = A.col[k];
                    ((T *)rest.val.data())[ir++] = av[k];
                }
            }
        }
        main.view = A;
        main.view.nrows = nrB;
        main.view.ncols = ncB;
        main.view.nnz = (int64_t)main.col.size();
        main.view.row_ptr = main.row_ptr.data();
        main.view.col = main.col.data();
        main.view.val = main.val.data();
        rest.view = A;
        rest.view.nnz = (int64_t)rest.col.size();
        rest.view.row_ptr = rest.row_ptr.data();
        rest.view.col = rest.col.data();
        rest.view.val = rest.val.data();
        build_bsell<T>(plan, main.view, B, spec.sigma, spec.remap, spec.xwin, threads);
        if (nrB < A.nrows) {
            std::vector<int32_t> tail;
            for (int64_t r = nrB; r < A.nrows; ++r) tail.push_back((int32_t)r);
            Part z;
            z.kind = K_ZERO;
            z.name = plan.prefix + "zero";
            z.nrows = (int64_t)tail.size();
            z.units = z.nrows;
            z.has_rows = true;
            z.p0 = upload(plan, "zero.rows", 4, z.nrows, tail.data());
            z.bytes = z.nrows * (4 + (int64_t)plan.vsize());
            plan.parts.push_back(z);
        }
        std::vector<int64_t> rl((size_t)A.nrows, 0);
        std::vector<int32_t> with;
        for (int64_t r = 0; r < A.nrows; ++r) {
            rl[(size_t)r] = rest.view.len(r);
            if (rl[(size_t)r] > 0) with.push_back((int32_t)r);
        }
        std::vector<int32_t> none;
        if (!with.empty()) build_csrv<T>(plan, rest.view, with, 0, 0, 0, true, 0, "csrv", rl, none, threads);
        return;
    }

    // ROW_DIV: heavy rows (longer than the threshold) against the rest.  After an earlier part wrote
    // every y element of these rows, rows with nothing left are skipped.
    std::vector<int32_t> heavy, light;
    for (int32_t r : rows) {
        const int64_t L = lens[(size_t)r];
        if (spec.heavy > 0 && L > spec.heavy) heavy.push_back(r);
        else if (!(acc && L == 0)) light.push_back(r);
    }
    // rows reduced through atomics are zeroed by the first launch
    std::vector<int32_t> zero_rows;
    const size_t zero_slot = plan.parts.size();
    bool heavy_done = false;
    // (heavy rows are written by their own reduce launch and need no zeroing)

    switch (spec.light) {
    case L_CSRV:
        build_csrv<T>(plan, A, light, spec.lpr, spec.chunk, spec.sigma, acc, spec.remap, "csrv", lens, zero_rows, threads);
        break;
    case L_SELL:
        build_sell<T>(plan, A, light, spec.sigma, acc, spec.remap, "sell", lens, threads);
        break;
    case L_XS:
        build_xs<T>(plan, A, light, spec.k, spec.sigma, acc, lens, threads);
        break;
    case L_NNZB:
        build_nnzb<T>(plan, A, light, spec.r, acc, lens, zero_rows, threads);
        break;
    case L_WBM:
        build_wbm<T>(plan, A, light, acc, lens, zero_rows, threads);
        break;
    case L_XNB:
        build_xnb<T>(plan, A, light, spec.k, spec.r, acc, lens, threads);
        break;
    case L_COO:
        build_coo<T>(plan, A, light, acc, lens, zero_rows, threads);
        break;
    case L_XL: {
        // The part may own more rows than it has entries for: the heavy rows of this leaf, or (span)
        // the rows of the sibling leaves that run after it.  They stay in as rows without entries,
        // so that the part's rows are one contiguous range where possible (no row map to read, y
        // written contiguously); the launches of their own parts overwrite those y elements later.
        const std::vector<int32_t> *owner = span ? span : (heavy.empty() ? nullptr : &rows);
        if (!acc && owner) {
            std::vector<int64_t> lens_light((size_t)A.nrows, 0);
            for (int32_t r : light) lens_light[(size_t)r] = lens[(size_t)r];
            // the heavy part runs first and leaves its partial sums to this part's reduce launch
            HeavyFold fold;
            if (!heavy.empty()) {
                const int64_t nb = ((int64_t)owner->size() + spec.rb - 1) / spec.rb;
                fold.hptr.assign((size_t)nb + 1, 0);
                fold.hloc.resize(heavy.size());
                for (size_t h = 0; h < heavy.size(); ++h) {
                    const int64_t pos = std::lower_bound(owner->begin(), owner->end(), heavy[h]) - owner->begin();
                    fold.hptr[(size_t)(pos / spec.rb) + 1] += 1;
                    fold.hloc[h] = (uint16_t)(pos % spec.rb);
                }
                for (int64_t b = 0; b < nb; ++b) fold.hptr[(size_t)b + 1] += fold.hptr[(size_t)b];
                build_stripe<T>(plan, A, heavy, spec.tile, spec.hd, spec.piece, acc, lens, threads, &fold);
                heavy_done = true;
            }
            build_xl<T>(plan, A, *owner, spec.w, spec.rb, spec.chunk, acc, lens_light, threads, heavy.empty() ? nullptr : &fold);
        } else {
            build_xl<T>(plan, A, light, spec.w, spec.rb, spec.chunk, acc, lens, threads);
        }
        break;
    }
    case L_BIN: {
        // BIN: short rows -> SELL, medium rows -> 8 lanes per row, long rows -> one wavefront (or, with
        // wg=1, one workgroup) per row (cut into segments of `chunk`)
        std::vector<int32_t> shorts, mids, longs;
        for (int32_t r : light) {
            const int64_t L = lens[(size_t)r];
            if (L <= spec.smax) shorts.push_back(r);
            else if (L <= 128) mids.push_back(r);
            else longs.push_back(r);
        }
        build_sell<T>(plan, A, shorts, spec.sigma, acc, spec.remap, "bin0.sell", lens, threads);
        build_csrv<T>(plan, A, mids, 8, 0, spec.sigma, acc, spec.remap, "bin1.csrv8", lens, zero_rows, threads);
        if (spec.wg) build_csrv<T>(plan, A, longs, 256, spec.chunk, 0, acc, spec.remap, "bin2.csrwg", lens, zero_rows, threads);
        else build_csrv<T>(plan, A, longs, 64, spec.chunk, 0, acc, spec.remap, "bin2.csrv64", lens, zero_rows, threads);
        break;
    }
    default: fail(SPMV_ERR_INVALID_ARG, "unknown light design");
    }
    if (!heavy.empty() && !heavy_done) build_stripe<T>(plan, A, heavy, spec.tile, spec.hd, spec.piece, acc, lens, threads);

    if (!zero_rows.empty()) {
        std::sort(zero_rows.begin(), zero_rows.end());
        Part z;
        z.kind = K_ZERO;
        z.name = plan.prefix + "zero";
        z.nrows = (int64_t)zero_rows.size();
        z.units = z.nrows;
        z.has_rows = true;
        z.p0 = upload(plan, "zero.rows", 4, z.nrows, zero_rows.data());
        z.bytes = z.nrows * (4 + (int64_t)plan.vsize());
        plan.parts.insert(plan.parts.begin() + (std::ptrdiff_t)zero_slot, z);
    }
}

// Copy of the rows `rows` of A restricted to the columns [c0, c1): same row numbering, other rows empty.
template <typename T>
void column_stripe(const HostCsr &A, const std::vector<int32_t> &rows, int64_t c0, int64_t c1, OwnedCsr &out,
                   int threads) {
    out.row_ptr.assign((size_t)A.nrows + 1, 0);
    parallel_for((int64_t)rows.size(), 1 << 12, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = rows[(size_t)i];
            int32_t cnt = 0;
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k) cnt += A.col[k] >= c0 && A.col[k] < c1;
            out.row_ptr[(size_t)r + 1] = cnt;
        }
    });
    for (int64_t r = 0; r < A.nrows; ++r) out.row_ptr[(size_t)r + 1] += out.row_ptr[(size_t)r];
    const int64_t nnz = out.row_ptr[(size_t)A.nrows];
    out.col.resize((size_t)nnz);
    out.val.resize((size_t)nnz * sizeof(T));
    const T *av = (const T *)A.val;
    T *ov = (T *)out.val.data();
    parallel_for((int64_t)rows.size(), 1 << 12, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = rows[(size_t)i];
            int64_t dst = out.row_ptr[(size_t)r];
            for (int64_t k = A.row_ptr[r]; k < A.row_ptr[r + 1]; ++k)
                if (A.col[k] >= c0 && A.col[k] < c1) {
                    out.col[(size_t)dst] = A.col[k];
                    ov[dst] = av[k];
                    ++dst;
                }
        }
    });
    out.view = A;
    out.view.nnz = nnz;
    out.view.row_ptr = out.row_ptr.data();
    out.view.col = out.col.data();
    out.view.val = out.val.data();
}

// The plan tree (Section IV-B): an inner node hands each child its share of the node's rows or
// columns; the children's launches follow each other in the order of the tree.  Array and launch
// names of a child carry its path ("r1.", "b3.", "p0.", "c2."), so that a tree's arrays stay apart.
template <typename T>
void build_node(Plan &plan, const HostCsr &A, const Census &cen, const PlanSpec &node,
                const std::vector<int32_t> &rows, bool whole, bool acc, const std::vector<int32_t> *span,
                int threads) {
    if (node.node == N_LEAF) {
        build_leaf<T>(plan, A, cen, node, rows, whole, acc, span, threads);
        return;
    }
    const std::string outer = plan.prefix;
    auto kid = [&](size_t i) -> const PlanSpec & { return node.kids.size() == 1 ? node.kids[0] : node.kids[i]; };
    // classes of rows in launch order; a two-pass leaf that comes first may own every row of the node
    auto run_classes = [&](const std::vector<std::vector<int32_t>> &cls, const std::vector<size_t> &design, char tag) {
        bool first = true;
        for (size_t i = 0; i < cls.size(); ++i) {
            if (cls[i].empty()) continue;
            const PlanSpec &k = kid(design[i]);
            plan.prefix = outer + tag + std::to_string(i) + ".";
            const bool can_span = first && !acc && !span && k.node == N_LEAF && k.light == L_XL && !k.heavy && cls[i].size() < rows.size();
            build_node<T>(plan, A, cen, k, cls[i], false, acc, can_span ? &rows : nullptr, threads);
            first = false;
        }
        plan.prefix = outer;
    };
    switch (node.node) {
    case N_ROWS: {
        std::vector<std::vector<int32_t>> cls(node.cuts.size() + 1);
        std::vector<size_t> design(cls.size());
        for (size_t i = 0; i < cls.size(); ++i) design[i] = i;
        for (int32_t r : rows) {
            const int64_t L = A.len(r);
            const size_t c = (size_t)(std::lower_bound(node.cuts.begin(), node.cuts.end(), L) - node.cuts.begin());
            cls[c].push_back(r);   // cuts[c-1] < L <= cuts[c]
        }
        run_classes(cls, design, 'r');
        break;
    }
    case N_BIN2: {
        // bin b: 2^b <= length < 2^(b+1); empty rows go with bin 0; lengths from 2^k on form the last class
        const int k = (int)node.cuts[0];
        std::vector<std::vector<int32_t>> cls((size_t)k + 1);
        std::vector<size_t> design((size_t)k + 1, 0);
        design[(size_t)k] = 1;
        for (int32_t r : rows) {
            const int64_t L = A.len(r);
            int b = 0;
            while (b < k && L >= ((int64_t)2 << b)) ++b;
            cls[(size_t)b].push_back(r);
        }
        run_classes(cls, design, 'b');
        break;
    }
    case N_CUT: {
        // stable sort by decreasing length; a part ends where the next row is rho times shorter and the
        // part has reached its minimum size; inside a part the rows return to ascending order
        std::vector<int32_t> order(rows);
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return A.len(a) > A.len(b); });
        std::vector<std::vector<int32_t>> cls(1);
        const int64_t rho = node.cuts[0], minrows = node.cuts[1];
        for (size_t i = 0; i < order.size(); ++i) {
            cls.back().push_back(order[i]);
            if (i + 1 < order.size() && (int64_t)cls.back().size() >= minrows && A.len(order[i]) > 0 &&
                A.len(order[i]) >= rho * A.len(order[i + 1]))
                cls.emplace_back();
        }
        if (cls.size() > 64) fail(SPMV_ERR_UNSUPPORTED, "cut: more than 64 parts");
        for (auto &c : cls) std::sort(c.begin(), c.end());
        std::vector<size_t> design(cls.size(), 0);
        run_classes(cls, design, 'p');
        break;
    }
    case N_COLS: {
        const int64_t K = node.cuts[0];
        const int64_t W = (A.ncols + K - 1) / K;
        for (int64_t j = 0; j < K; ++j) {
            OwnedCsr stripe;
            column_stripe<T>(A, rows, j * W, std::min(A.ncols, (j + 1) * W), stripe, threads);
            plan.prefix = outer + "c" + std::to_string(j) + ".";
            // the first stripe writes every row of the node (zeros where it has nothing), the others add
            build_node<T>(plan, stripe.view, cen, kid((size_t)j), rows, false, acc || j > 0, nullptr, threads);
        }
        plan.prefix = outer;
        break;
    }
    default: fail(SPMV_ERR_INVALID_ARG, "unknown plan node");
    }
}

template <typename T>
std::unique_ptr<Plan> build_typed(const HostCsr &A0, const Census &cen, const PlanSpec &spec,
                                  const Allocator &mem, int threads) {
    std::unique_ptr<Plan> plan(new Plan);
    plan->dtype = A0.dtype;
    plan->nrows = A0.nrows;
    plan->ncols = A0.ncols;
    plan->nnz = A0.nnz;
    plan->spec = spec;
    plan->mem = mem;
    plan->census = cen;

    OwnedCsr sorted;
    const HostCsr *cur = &A0;
    if (!cen.cols_sorted) {
        sorted_copy<T>(A0, sorted, threads);
        cur = &sorted.view;
    }
    std::vector<int32_t> all((size_t)A0.nrows);
    std::iota(all.begin(), all.end(), 0);
    build_node<T>(*plan, *cur, cen, spec, all, true, false, nullptr, threads);
    plan->prefix.clear();
    if (plan_wants_jit(spec)) jit_compile_plan(*plan);
    return plan;
}

}  // namespace

std::unique_ptr<Plan> build_plan(const HostCsr &A, const Census &cen, const PlanSpec &spec,
                                 const Allocator &mem, int threads) {
    if (A.dtype == SPMV_F64) return build_typed<double>(A, cen, spec, mem, threads);
    return build_typed<float>(A, cen, spec, mem, threads);
}

}  // namespace spmv
