// The C ABI of include/spmv.h: argument and CSR validation, exception -> status translation,
// plan description.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <sstream>

#include "internal.h"

struct spmv_plan {
    std::unique_ptr<spmv::Plan> impl;
};

namespace spmv {

static thread_local std::string g_last_error;

static void *default_alloc(size_t bytes, void *) {
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return p;
}
static void default_free(void *p, void *) { (void)hipFree(p); }
static void *host_alloc(size_t bytes, void *) { return std::malloc(bytes); }
static void host_free(void *p, void *) { std::free(p); }

static void validate_csr(const HostCsr &A, int threads) {
    if (A.row_ptr[0] != 0) fail(SPMV_ERR_BAD_CSR, "row_ptr[0] must be 0");
    if ((int64_t)A.row_ptr[A.nrows] != A.nnz) fail(SPMV_ERR_BAD_CSR, "row_ptr[nrows] must equal nnz");
    std::atomic<int> bad{0};
    parallel_for(A.nrows, 1 << 14, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t r = b; r < e; ++r) {
            const int64_t s = A.row_ptr[r], t = A.row_ptr[r + 1];
            if (t < s || s < 0 || t > A.nnz) {
                bad = 1;
                return;
            }
            for (int64_t k = s; k < t; ++k)
                if (A.col[k] < 0 || (int64_t)A.col[k] >= A.ncols) {
                    bad = 2;
                    return;
                }
        }
    });
    if (bad == 1) fail(SPMV_ERR_BAD_CSR, "row_ptr is not non-decreasing within [0, nnz]");
    if (bad == 2) fail(SPMV_ERR_BAD_CSR, "a column index is outside [0, ncols)");
}

static std::string json_escape(const std::string &s) {
    std::string o;
    for (char ch : s) {
        if (ch == '\n') {
            o += "\\n";
            continue;
        }
        if ((unsigned char)ch < 0x20) ch = ' ';
        if (ch == '"' || ch == '\\') o += '\\';
        o += ch;
    }
    return o;
}

std::string describe_json(const Plan &plan) {
    std::ostringstream o;
    o.precision(12);
    const Census &c = plan.census;
    o << "{\"spec\": \"" << json_escape(print_spec(plan.spec)) << "\", ";
    o << "\"operators\": \"" << json_escape(operator_chain(plan.spec)) << "\", ";
    o << "\"dtype\": \"" << (plan.dtype == SPMV_F64 ? "f64" : "f32") << "\", ";
    o << "\"nrows\": " << plan.nrows << ", \"ncols\": " << plan.ncols << ", \"nnz\": " << plan.nnz << ", ";
    o << "\"bytes_plan\": " << plan.bytes_plan() << ", \"bytes_csr\": " << plan.bytes_csr() << ", ";
    o << "\"census\": {\"min_len\": " << c.min_len << ", \"max_len\": " << c.max_len
      << ", \"mean_len\": " << c.mean_len << ", \"var_len\": " << c.var_len
      << ", \"empty_rows\": " << c.empty_rows << ", \"irregular\": " << (c.var_len > 100 ? "true" : "false")
      << ", \"cols_sorted\": " << (c.cols_sorted ? "true" : "false") << ", \"diag_offsets\": [";
    for (size_t i = 0; i < c.diag_offsets.size(); ++i) o << (i ? ", " : "") << c.diag_offsets[i];
    o << "], \"diag_nnz\": " << c.diag_nnz << ", \"block_fill\": {\"2\": " << c.block_fill[2]
      << ", \"3\": " << c.block_fill[3] << ", \"4\": " << c.block_fill[4] << "}}, ";
    o << "\"parts\": [";
    for (size_t i = 0; i < plan.parts.size(); ++i) {
        const Part &p = plan.parts[i];
        o << (i ? ", " : "") << "{\"name\": \"" << p.name << "\", \"rows\": " << p.nrows
          << ", \"nnz\": " << p.nnz << ", \"stored\": " << p.stored << ", \"units\": " << p.units
          << ", \"bytes\": " << p.bytes << ", \"lanes\": " << p.lanes << ", \"accumulate\": " << (p.accumulate ? "true" : "false")
          << ", \"origin_rows\": " << (p.has_rows ? "true" : "false") << ", \"jit\": " << (p.jit_fn ? "true" : "false")
          << ", \"jit_kernel\": \"" << json_escape(p.jit_kernel) << "\", \"jit_defines\": \"" << json_escape(p.jit_defines) << "\"}";
    }
    o << "], \"arrays\": [";
    for (size_t i = 0; i < plan.arrays.size(); ++i) {
        const DevArray &a = plan.arrays[i];
        o << (i ? ", " : "") << "{\"name\": \"" << a.name << "\", \"elem_bytes\": " << a.elem_bytes
          << ", \"count\": " << a.count << ", \"model\": \"" << a.model.text() << "\"}";
    }
    int64_t scratch_bytes = 0;
    for (const DevArray &a : plan.scratch) scratch_bytes += a.count * a.elem_bytes;
    o << "], \"jit_note\": \"" << json_escape(plan.jit_note) << "\", \"scratch_bytes\": " << scratch_bytes << ", \"search\": [";
    for (size_t i = 0; i < plan.log.size(); ++i) {
        const CandidateLog &l = plan.log[i];
        o << (i ? ", " : "") << "{\"spec\": \"" << json_escape(l.spec) << "\", \"build_ms\": " << l.build_ms
          << ", \"run_us\": " << l.run_us << ", \"pred_us\": " << l.pred_us << ", \"playoff_us\": " << l.playoff_us << ", \"note\": \"" << json_escape(l.note) << "\"}";
    }
    o << "]}";
    return o.str();
}

}  // namespace spmv

using namespace spmv;

#define API_BEGIN try {
#define API_END                                                  \
    }                                                            \
    catch (const Error &e) {                                     \
        g_last_error = e.msg;                                    \
        return e.code;                                           \
    }                                                            \
    catch (const std::bad_alloc &) {                             \
        g_last_error = "host allocation failed";                 \
        return SPMV_ERR_ALLOC;                                   \
    }                                                            \
    catch (const std::exception &e) {                            \
        g_last_error = std::string("internal error: ") + e.what(); \
        return SPMV_ERR_INTERNAL;                                \
    }                                                            \
    catch (...) {                                                \
        g_last_error = "internal error";                         \
        return SPMV_ERR_INTERNAL;                                \
    }

extern "C" {

const char *spmv_last_error(void) { return g_last_error.c_str(); }

spmv_status_t spmv_stream_ceiling(size_t bytes, int repeats, void *stream, double *read_gbps,
                                  double *copy_gbps) {
    API_BEGIN
    if (!read_gbps || !copy_gbps) fail(SPMV_ERR_INVALID_ARG, "spmv_stream_ceiling: NULL result pointer");
    if (bytes < (1u << 20) || repeats < 1 || repeats > 1000)
        fail(SPMV_ERR_INVALID_ARG, "spmv_stream_ceiling: bytes must be at least 1 MiB, repeats in [1, 1000]");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) {
        (void)hipGetLastError();
        fail(SPMV_ERR_HIP, "no HIP device available");
    }
    const int err = stream_ceiling(bytes, repeats, stream, read_gbps, copy_gbps);
    if (err) fail(err == (int)hipErrorOutOfMemory ? SPMV_ERR_ALLOC : SPMV_ERR_HIP, std::string("stream ceiling: ") + hip_error_text(err));
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_mm_read(const char *path, spmv_dtype_t dtype, int64_t *nrows, int64_t *ncols,
                           int64_t *nnz, int32_t **row_ptr, int32_t **col_idx, void **values) {
    if (row_ptr) *row_ptr = nullptr;
    if (col_idx) *col_idx = nullptr;
    if (values) *values = nullptr;
    API_BEGIN
    if (!path || !nrows || !ncols || !nnz || !row_ptr || !col_idx || !values)
        fail(SPMV_ERR_INVALID_ARG, "spmv_mm_read: NULL argument");
    if (dtype != SPMV_F32 && dtype != SPMV_F64) fail(SPMV_ERR_UNSUPPORTED, "unknown dtype");
    MmCsr m;
    read_matrix_market(path, dtype, m);
    *nrows = m.nrows;
    *ncols = m.ncols;
    *nnz = m.nnz;
    *row_ptr = m.row_ptr;
    *col_idx = m.col;
    *values = m.val;
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_mm_free(int32_t *row_ptr, int32_t *col_idx, void *values) {
    std::free(row_ptr);
    std::free(col_idx);
    std::free(values);
    return SPMV_OK;
}

spmv_status_t spmv_plan_create(spmv_plan_t **out, int64_t nrows, int64_t ncols, int64_t nnz,
                               const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                               spmv_dtype_t dtype, const spmv_options_t *opts) {
    if (out) *out = nullptr;
    API_BEGIN
    if (!out) fail(SPMV_ERR_INVALID_ARG, "out is NULL");
    if (nrows < 0 || ncols < 0 || nnz < 0) fail(SPMV_ERR_INVALID_ARG, "negative dimension");
    if (!row_ptr) fail(SPMV_ERR_INVALID_ARG, "row_ptr is NULL");
    if (nnz > 0 && (!col_idx || !values)) fail(SPMV_ERR_INVALID_ARG, "col_idx / values is NULL");
    if (dtype != SPMV_F32 && dtype != SPMV_F64) fail(SPMV_ERR_UNSUPPORTED, "unknown dtype");
    if (nnz >= ((int64_t)1 << 31) || nrows >= ((int64_t)1 << 31) - 64 || ncols >= ((int64_t)1 << 31) - 64)
        fail(SPMV_ERR_UNSUPPORTED, "dimensions and nnz must be below 2^31");
    spmv_options_t o;
    std::memset(&o, 0, sizeof o);
    if (opts) o = *opts;
    if ((o.dev_alloc == nullptr) != (o.dev_free == nullptr))
        fail(SPMV_ERR_INVALID_ARG, "dev_alloc and dev_free must be given together");
    if (o.host_threads < 0 || o.search_repeats < 0) fail(SPMV_ERR_INVALID_ARG, "negative option");
    Allocator mem;
    mem.alloc = o.dev_alloc ? o.dev_alloc : default_alloc;
    mem.free = o.dev_free ? o.dev_free : default_free;
    mem.user = o.user;
    if (o.host_only) {
        mem.alloc = host_alloc;
        mem.free = host_free;
        mem.user = nullptr;
        mem.host_only = true;
    }
    const int threads = o.host_threads > 0 ? o.host_threads : default_threads();

    HostCsr A;
    A.nrows = nrows;
    A.ncols = ncols;
    A.nnz = nnz;
    A.row_ptr = row_ptr;
    A.col = col_idx;
    A.val = values;
    A.dtype = dtype;
    validate_csr(A, threads);

    // a plan-spec string is parsed before anything touches the device
    const bool forced = o.force_plan && o.force_plan[0];
    PlanSpec spec;
    if (forced) spec = parse_spec(o.force_plan);

    if (o.host_only && !forced && !(o.search_budget_ms < 0))
        fail(SPMV_ERR_INVALID_ARG, "host_only needs force_plan or a negative search_budget_ms");
    int ndev = 0;
    if (!o.host_only && (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0)) {
        (void)hipGetLastError();
        fail(SPMV_ERR_HIP, "no HIP device available");
    }
    if (!o.host_only) {
        // everything a launch needs beyond the plan itself is set up here, so that spmv_run only enqueues kernels
        const int err = prepare_device();
        if (err) fail(SPMV_ERR_HIP, std::string("device set-up failed: ") + hip_error_text(err));
    }
    const Census cen = take_census(A, threads);
    std::unique_ptr<Plan> plan;
    if (forced) {
        plan = build_plan(A, cen, spec, mem, threads);
        CandidateLog l;
        l.spec = print_spec(spec);
        l.note = "forced";
        plan->log.push_back(l);
    } else {
        plan = search_plan(A, cen, o, mem, threads);
    }
    if (!o.host_only && hipDeviceSynchronize() != hipSuccess) fail(SPMV_ERR_HIP, "device error after plan construction");
    plan->describe_cache = describe_json(*plan);
    *out = new spmv_plan{std::move(plan)};
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_run(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream) {
    API_BEGIN
    if (!plan || !plan->impl) fail(SPMV_ERR_INVALID_ARG, "plan is NULL");
    const Plan &p = *plan->impl;
    if (p.mem.host_only) fail(SPMV_ERR_UNSUPPORTED, "the plan was built host-only and cannot run");
    if ((!x_dev && p.ncols > 0) || (!y_dev && p.nrows > 0)) fail(SPMV_ERR_INVALID_ARG, "x or y is NULL");
    if (x_dev && x_dev == y_dev) fail(SPMV_ERR_INVALID_ARG, "x and y must not alias");
    for (const Part &part : p.parts) {
        const int err = launch_part(part, p.dtype, p.nrows, p.ncols, x_dev, y_dev, stream);
        if (err) fail(SPMV_ERR_HIP, std::string("launch of ") + part.name + " failed: " + hip_error_text(err));
    }
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_run_noalloc(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream) {
    API_BEGIN
    if (!plan || !plan->impl) fail(SPMV_ERR_INVALID_ARG, "plan is NULL");
    const Plan &p = *plan->impl;
    if (p.mem.host_only) fail(SPMV_ERR_UNSUPPORTED, "the plan was built host-only and cannot run");
    if ((!x_dev && p.ncols > 0) || (!y_dev && p.nrows > 0)) fail(SPMV_ERR_INVALID_ARG, "x or y is NULL");
    if (x_dev && x_dev == y_dev) fail(SPMV_ERR_INVALID_ARG, "x and y must not alias");
    // place the plan's scratch buffers one after the other (256-byte aligned) in the static array
    constexpr int kMaxBuffers = 16;
    const void *owned[kMaxBuffers];
    size_t offset[kMaxBuffers];
    if (p.scratch.size() > (size_t)kMaxBuffers) fail(SPMV_ERR_UNSUPPORTED, "spmv_run_noalloc: the plan has too many scratch buffers");
    size_t need = 0;
    for (size_t i = 0; i < p.scratch.size(); ++i) {
        owned[i] = p.scratch[i].ptr;
        offset[i] = need;
        const size_t bytes = (size_t)p.scratch[i].count * (size_t)p.scratch[i].elem_bytes;
        need += (bytes + 255) / 256 * 256;
    }
    if (need > kStaticScratchBytes)
        fail(SPMV_ERR_UNSUPPORTED, "spmv_run_noalloc: the plan needs " + std::to_string(need) + " bytes of scratch, the static buffer holds " +
                                       std::to_string(kStaticScratchBytes));
    void *base = nullptr;
    if (need > 0) {
        const int err = static_scratch(&base);
        if (err) fail(SPMV_ERR_HIP, std::string("spmv_run_noalloc: static scratch unavailable: ") + hip_error_text(err));
    }
    auto placed = [&](const void *own) -> void * {
        if (!own) return nullptr;
        size_t i = 0;
        while (i < p.scratch.size() && owned[i] != own) ++i;
        if (i == p.scratch.size()) fail(SPMV_ERR_INTERNAL, "spmv_run_noalloc: a launch refers to an unknown scratch buffer");
        return (unsigned char *)base + offset[i];
    };
    for (const Part &part : p.parts) {
        const int err = launch_part(part, p.dtype, p.nrows, p.ncols, x_dev, y_dev, stream, placed(part.scratch), placed(part.scratch2));
        if (err) fail(SPMV_ERR_HIP, std::string("launch of ") + part.name + " failed: " + hip_error_text(err));
    }
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_run_multi(const spmv_plan_t *plan, const void *x_dev, int64_t ldx, void *y_dev, int64_t ldy,
                             int k, void *stream) {
    API_BEGIN
    if (!plan || !plan->impl) fail(SPMV_ERR_INVALID_ARG, "plan is NULL");
    const Plan &p = *plan->impl;
    if (p.mem.host_only) fail(SPMV_ERR_UNSUPPORTED, "the plan was built host-only and cannot run");
    if (k < 0 || k > 4096) fail(SPMV_ERR_INVALID_ARG, "spmv_run_multi: k must be in [0, 4096]");
    if (k == 0) return SPMV_OK;
    if ((!x_dev && p.ncols > 0) || (!y_dev && p.nrows > 0)) fail(SPMV_ERR_INVALID_ARG, "X or Y is NULL");
    if (x_dev && x_dev == y_dev) fail(SPMV_ERR_INVALID_ARG, "X and Y must not alias");
    if (k > 1 && (ldx < p.ncols || ldy < p.nrows)) fail(SPMV_ERR_INVALID_ARG, "spmv_run_multi: ldx < ncols or ldy < nrows");
    const size_t v = p.vsize();
    auto xv = [&](int i) { return (const void *)((const char *)x_dev + (size_t)i * (size_t)ldx * v); };
    auto yv = [&](int i) { return (void *)((char *)y_dev + (size_t)i * (size_t)ldy * v); };
    auto fused = [](const Part &q) { return (q.kind == K_DIA && q.ndiag >= 1 && q.ndiag <= 8) || q.kind == K_SELL || q.kind == K_CSRV; };
    auto one = [&](const Part &q, int i) {
        const int err = launch_part(q, p.dtype, p.nrows, p.ncols, xv(i), yv(i), stream);
        if (err) fail(SPMV_ERR_HIP, std::string("launch of ") + q.name + " failed: " + hip_error_text(err));
    };
    size_t i = 0;
    while (i < p.parts.size()) {
        if (fused(p.parts[i])) {
            // the matrix stream is read once for 8, 4 or 2 vectors at a time
            int done = 0;
            while (done < k) {
                const int left = k - done;
                const int kk = left >= 8 ? 8 : (left >= 4 ? 4 : (left >= 2 ? 2 : 1));
                int err = -1;
                if (kk > 1) err = launch_part_multi(p.parts[i], p.dtype, p.nrows, p.ncols, xv(done), ldx, yv(done), ldy, kk, stream);
                if (err > 0) fail(SPMV_ERR_HIP, std::string("launch of ") + p.parts[i].name + " failed: " + hip_error_text(err));
                if (err < 0)
                    for (int u = 0; u < kk; ++u) one(p.parts[i], done + u);
                done += kk;
            }
            ++i;
            continue;
        }
        // launches that hand partial sums to each other through the plan's scratch run vector by vector
        size_t j = i;
        while (j < p.parts.size() && !fused(p.parts[j])) ++j;
        for (int u = 0; u < k; ++u)
            for (size_t q = i; q < j; ++q) one(p.parts[q], u);
        i = j;
    }
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_cost_predict(const spmv_plan_t *plan, const char *corpus_path, const char *spec, double *pred_us,
                                int64_t *samples) {
    API_BEGIN
    if (!plan || !plan->impl || !corpus_path || !spec || !pred_us) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    const PlanSpec ps = parse_spec(spec);
    CostModel model;
    const int used = model.load(corpus_path);
    model.train();
    if (samples) *samples = used;
    *pred_us = model.predict_us(cost_census(plan->impl->census, plan->impl->dtype), ps);
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_fit_array(const void *data, int elem_bytes, int64_t count, char *buf, size_t cap) {
    API_BEGIN
    if ((!data && count > 0) || !buf || cap == 0) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    if ((elem_bytes != 4 && elem_bytes != 8) || count < 0) fail(SPMV_ERR_INVALID_ARG, "spmv_fit_array: 4- or 8-byte integers, count >= 0");
    const std::string t = fit_array(data, elem_bytes, count).text();
    const size_t n = std::min(cap - 1, t.size());
    std::memcpy(buf, t.data(), n);
    buf[n] = 0;
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_jit_check(const spmv_plan_t *plan, int *compiled, char *log, size_t cap) {
    API_BEGIN
    if (!plan || !plan->impl || !compiled) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    std::string text;
    *compiled = jit_check_plan(*plan->impl, text);
    if (log && cap > 0) {
        const size_t n = std::min(cap - 1, text.size());
        std::memcpy(log, text.data(), n);
        log[n] = 0;
    }
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_save(const spmv_plan_t *plan, const char *path) {
    API_BEGIN
    if (!plan || !plan->impl || !path) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    save_plan(*plan->impl, path);
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_load(spmv_plan_t **out, const char *path, const spmv_options_t *opts) {
    if (out) *out = nullptr;
    API_BEGIN
    if (!out || !path) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    spmv_options_t o;
    std::memset(&o, 0, sizeof o);
    if (opts) o = *opts;
    if ((o.dev_alloc == nullptr) != (o.dev_free == nullptr))
        fail(SPMV_ERR_INVALID_ARG, "dev_alloc and dev_free must be given together");
    Allocator mem;
    mem.alloc = o.dev_alloc ? o.dev_alloc : default_alloc;
    mem.free = o.dev_free ? o.dev_free : default_free;
    mem.user = o.user;
    if (o.host_only) {
        mem.alloc = host_alloc;
        mem.free = host_free;
        mem.user = nullptr;
        mem.host_only = true;
    } else {
        int ndev = 0;
        if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) {
            (void)hipGetLastError();
            fail(SPMV_ERR_HIP, "no HIP device available");
        }
        const int err = prepare_device();
        if (err) fail(SPMV_ERR_HIP, std::string("device set-up failed: ") + hip_error_text(err));
    }
    std::unique_ptr<Plan> plan = load_plan(path, mem);
    if (!o.host_only && hipDeviceSynchronize() != hipSuccess) fail(SPMV_ERR_HIP, "device error after loading the plan");
    plan->describe_cache = describe_json(*plan);
    *out = new spmv_plan{std::move(plan)};
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_run_timed(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream,
                             float *launch_ms) {
    API_BEGIN
    if (!plan || !plan->impl || !launch_ms) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    const Plan &p = *plan->impl;
    if (p.mem.host_only) fail(SPMV_ERR_UNSUPPORTED, "the plan was built host-only and cannot run");
    if ((!x_dev && p.ncols > 0) || (!y_dev && p.nrows > 0)) fail(SPMV_ERR_INVALID_ARG, "x or y is NULL");
    if (x_dev && x_dev == y_dev) fail(SPMV_ERR_INVALID_ARG, "x and y must not alias");
    const size_t n = p.parts.size();
    std::vector<hipEvent_t> ev(n + 1, nullptr);
    auto drop = [&]() {
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
    };
    for (size_t i = 0; i <= n; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            drop();
            fail(SPMV_ERR_HIP, "hipEventCreate failed");
        }
    (void)hipEventRecord(ev[0], (hipStream_t)stream);
    for (size_t i = 0; i < n; ++i) {
        const int err = launch_part(p.parts[i], p.dtype, p.nrows, p.ncols, x_dev, y_dev, stream);
        if (err) {
            drop();
            fail(SPMV_ERR_HIP, std::string("launch of ") + p.parts[i].name + " failed: " + hip_error_text(err));
        }
        (void)hipEventRecord(ev[i + 1], (hipStream_t)stream);
    }
    if (hipEventSynchronize(ev[n]) != hipSuccess) {
        drop();
        fail(SPMV_ERR_HIP, "a kernel failed");
    }
    for (size_t i = 0; i < n; ++i) (void)hipEventElapsedTime(&launch_ms[i], ev[i], ev[i + 1]);
    drop();
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_time_launches(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream,
                                      int repeats, float *launch_us) {
    API_BEGIN
    if (!plan || !plan->impl || !launch_us) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    const Plan &p = *plan->impl;
    if (p.mem.host_only) fail(SPMV_ERR_UNSUPPORTED, "the plan was built host-only and cannot run");
    if ((!x_dev && p.ncols > 0) || (!y_dev && p.nrows > 0)) fail(SPMV_ERR_INVALID_ARG, "x or y is NULL");
    if (x_dev && x_dev == y_dev) fail(SPMV_ERR_INVALID_ARG, "x and y must not alias");
    if (repeats < 1 || repeats > 10000) fail(SPMV_ERR_INVALID_ARG, "repeats out of range");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        fail(SPMV_ERR_HIP, "hipEventCreate failed");
    }
    auto drop = [&]() {
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
    };
    for (size_t i = 0; i < p.parts.size(); ++i) {
        // launch i of one ordinary run has the inputs it expects: everything before it ran once
        for (int r = 0; r < repeats + 1; ++r) {
            if (r == 1) (void)hipEventRecord(e0, (hipStream_t)stream);   // the first launch warms up
            const int err = launch_part(p.parts[i], p.dtype, p.nrows, p.ncols, x_dev, y_dev, stream);
            if (err) {
                drop();
                fail(SPMV_ERR_HIP, std::string("launch of ") + p.parts[i].name + " failed: " + hip_error_text(err));
            }
        }
        (void)hipEventRecord(e1, (hipStream_t)stream);
        if (hipEventSynchronize(e1) != hipSuccess) {
            drop();
            fail(SPMV_ERR_HIP, "a kernel failed");
        }
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        launch_us[i] = ms * 1000.0f / (float)repeats;
    }
    drop();
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_time(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream,
                             int repeats, double *median_us) {
    API_BEGIN
    if (!plan || !plan->impl || !median_us) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    const Plan &p = *plan->impl;
    if (p.mem.host_only) fail(SPMV_ERR_UNSUPPORTED, "the plan was built host-only and cannot run");
    if ((!x_dev && p.ncols > 0) || (!y_dev && p.nrows > 0)) fail(SPMV_ERR_INVALID_ARG, "x or y is NULL");
    if (x_dev && x_dev == y_dev) fail(SPMV_ERR_INVALID_ARG, "x and y must not alias");
    if (repeats < 1 || repeats > 100000) fail(SPMV_ERR_INVALID_ARG, "repeats out of range");
    *median_us = time_plan(p, x_dev, y_dev, repeats, stream);
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_destroy(spmv_plan_t *plan) {
    API_BEGIN
    delete plan;
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_describe(const spmv_plan_t *plan, char *buf, size_t cap, size_t *needed) {
    API_BEGIN
    if (!plan || !plan->impl) fail(SPMV_ERR_INVALID_ARG, "plan is NULL");
    const std::string &s = plan->impl->describe_cache;
    if (needed) *needed = s.size() + 1;
    if (buf && cap > 0) {
        const size_t n = std::min(cap - 1, s.size());
        std::memcpy(buf, s.data(), n);
        buf[n] = 0;
    }
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_array_count(const spmv_plan_t *plan, int *n) {
    API_BEGIN
    if (!plan || !plan->impl || !n) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    *n = (int)plan->impl->arrays.size();
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_array_info(const spmv_plan_t *plan, int i, const char **name,
                                   int *elem_bytes, int64_t *count) {
    API_BEGIN
    if (!plan || !plan->impl) fail(SPMV_ERR_INVALID_ARG, "plan is NULL");
    if (i < 0 || i >= (int)plan->impl->arrays.size()) fail(SPMV_ERR_INVALID_ARG, "array index out of range");
    const DevArray &a = plan->impl->arrays[(size_t)i];
    if (name) *name = a.name.c_str();
    if (elem_bytes) *elem_bytes = a.elem_bytes;
    if (count) *count = a.count;
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_array_copy(const spmv_plan_t *plan, int i, void *host_dst) {
    API_BEGIN
    if (!plan || !plan->impl || !host_dst) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    if (i < 0 || i >= (int)plan->impl->arrays.size()) fail(SPMV_ERR_INVALID_ARG, "array index out of range");
    const DevArray &a = plan->impl->arrays[(size_t)i];
    if (a.count > 0 && plan->impl->mem.host_only) {
        std::memcpy(host_dst, a.ptr, (size_t)a.count * (size_t)a.elem_bytes);
    } else if (a.count > 0) {
        hipError_t err = hipMemcpy(host_dst, a.ptr, (size_t)a.count * (size_t)a.elem_bytes, hipMemcpyDeviceToHost);
        if (err != hipSuccess) fail(SPMV_ERR_HIP, std::string("hipMemcpy D2H: ") + hipGetErrorString(err));
    }
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_bytes(const spmv_plan_t *plan, int64_t *b_plan, int64_t *b_csr) {
    API_BEGIN
    if (!plan || !plan->impl) fail(SPMV_ERR_INVALID_ARG, "plan is NULL");
    if (b_plan) *b_plan = plan->impl->bytes_plan();
    if (b_csr) *b_csr = plan->impl->bytes_csr();
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_launch_count(const spmv_plan_t *plan, int *n) {
    API_BEGIN
    if (!plan || !plan->impl || !n) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    *n = (int)plan->impl->parts.size();
    return SPMV_OK;
    API_END
}

spmv_status_t spmv_plan_launch_name(const spmv_plan_t *plan, int i, const char **name) {
    API_BEGIN
    if (!plan || !plan->impl || !name) fail(SPMV_ERR_INVALID_ARG, "NULL argument");
    if (i < 0 || i >= (int)plan->impl->parts.size()) fail(SPMV_ERR_INVALID_ARG, "launch index out of range");
    *name = plan->impl->parts[(size_t)i].name.c_str();
    return SPMV_OK;
    API_END
}

}  // extern "C"
