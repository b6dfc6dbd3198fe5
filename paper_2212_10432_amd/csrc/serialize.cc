// Plan files: a built plan written to disk and read back, so that neither the search nor the host
// format construction has to be repeated for a matrix that was planned before.  The paper's tool
// persists its result as generated source plus the format arrays it reads (Section III, "generated
// codes can be directly called"; artifact description); here the kernels are part of the library,
// so the file holds the plan spec, the census, the launch list and every format array.
//
// Layout (little endian): magic "SPMVPLN3", u64 payload size, u64 FNV-1a hash of the payload, then
// the payload: scalars and strings in the order written by save_plan below, every array as
// (name, element size, count, flag, raw bytes).  Pointers inside a launch record are stored as
// indices into the array list (-1: none); scratch buffers are stored as sizes only.
#include <hip/hip_runtime_api.h>

#include <cstdio>

#include "internal.h"

namespace spmv {
namespace {

constexpr char kMagic[8] = {'S', 'P', 'M', 'V', 'P', 'L', 'N', '3'};

uint64_t fnv1a(const unsigned char *p, size_t n) {
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) {
        h ^= p[i];
        h *= 1099511628211ull;
    }
    return h;
}

struct Writer {
    std::vector<unsigned char> buf;
    void raw(const void *p, size_t n) {
        const unsigned char *b = (const unsigned char *)p;
        buf.insert(buf.end(), b, b + n);
    }
    void i64(int64_t v) { raw(&v, 8); }
    void f64(double v) { raw(&v, 8); }
    void str(const std::string &s) {
        i64((int64_t)s.size());
        raw(s.data(), s.size());
    }
};

struct Reader {
    const unsigned char *p, *end;
    void need(size_t n) const {
        if ((size_t)(end - p) < n) fail(SPMV_ERR_INVALID_ARG, "plan file: truncated payload");
    }
    void raw(void *dst, size_t n) {
        need(n);
        std::memcpy(dst, p, n);
        p += n;
    }
    int64_t i64() {
        int64_t v;
        raw(&v, 8);
        return v;
    }
    double f64() {
        double v;
        raw(&v, 8);
        return v;
    }
    int64_t count(int64_t most) {   // a non-negative size that the rest of the file can hold
        const int64_t v = i64();
        if (v < 0 || v > most) fail(SPMV_ERR_INVALID_ARG, "plan file: implausible size field");
        return v;
    }
    std::string str() {
        const int64_t n = count(end - p);
        std::string s((const char *)p, (size_t)n);
        p += n;
        return s;
    }
};

// One launch record, field by field; the same list drives writing and reading.
template <typename F>
void part_scalars(Part &q, F &&f) {
    int64_t kind = (int64_t)q.kind, acc = q.accumulate, has = q.has_rows;
    f(kind); f(q.nrows); f(q.nnz); f(q.stored); f(q.units); f(acc); f(has);
    int64_t lanes = q.lanes, block = q.block, ndiag = q.ndiag, tile = q.tile, remap = q.remap, uw = q.uniform_w, delta = q.delta;
    f(lanes); f(block); f(ndiag); f(tile); f(remap); f(q.ld); f(q.nslices); f(q.ngroups); f(q.per_group); f(uw); f(delta);
    f(q.lds_bytes); f(q.bytes);
    for (int d = 0; d < 8; ++d) {
        int64_t o = q.dia_offsets[d];
        f(o);
        q.dia_offsets[d] = (int32_t)o;
    }
    q.kind = (PartKind)kind;
    q.accumulate = acc != 0;
    q.has_rows = has != 0;
    q.lanes = (int)lanes; q.block = (int)block; q.ndiag = (int)ndiag; q.tile = (int)tile; q.remap = (int)remap;
    q.uniform_w = (int)uw; q.delta = (int)delta;
}

}  // namespace

void save_plan(const Plan &plan, const char *path) {
    Writer w;
    w.i64((int64_t)plan.dtype);
    w.i64(plan.nrows);
    w.i64(plan.ncols);
    w.i64(plan.nnz);
    w.str(print_spec(plan.spec));
    const Census &c = plan.census;
    w.i64(c.nrows); w.i64(c.ncols); w.i64(c.nnz); w.i64(c.min_len); w.i64(c.max_len); w.i64(c.empty_rows);
    w.f64(c.mean_len); w.f64(c.var_len);
    for (int k = 0; k <= 20; ++k) { w.i64(c.rows_over[k]); w.i64(c.nnz_over[k]); }
    w.i64((int64_t)c.diag_offsets.size());
    for (int32_t o : c.diag_offsets) w.i64(o);
    w.i64(c.diag_nnz);
    for (int b = 0; b < 5; ++b) { w.i64(c.blocks[b]); w.f64(c.block_fill[b]); }
    w.i64(c.cols_sorted);
    // arrays
    w.i64((int64_t)plan.arrays.size());
    std::vector<unsigned char> tmp;
    for (const DevArray &a : plan.arrays) {
        w.str(a.name);
        w.i64(a.elem_bytes);
        w.i64(a.count);
        w.i64(a.read_per_run);
        const size_t bytes = (size_t)a.count * (size_t)a.elem_bytes;
        if (bytes == 0) continue;
        if (plan.mem.host_only) {
            w.raw(a.ptr, bytes);
        } else {
            tmp.resize(bytes);
            hipError_t err = hipMemcpy(tmp.data(), a.ptr, bytes, hipMemcpyDeviceToHost);
            if (err != hipSuccess) fail(SPMV_ERR_HIP, std::string("plan save: hipMemcpy D2H (") + a.name + "): " + hipGetErrorString(err));
            w.raw(tmp.data(), bytes);
        }
    }
    w.i64((int64_t)plan.scratch.size());
    for (const DevArray &a : plan.scratch) {
        w.str(a.name);
        w.i64(a.elem_bytes);
        w.i64(a.count);
    }
    auto array_index = [&](const void *p) -> int64_t {
        if (!p) return -1;
        for (size_t i = 0; i < plan.arrays.size(); ++i)
            if (plan.arrays[i].ptr == p) return (int64_t)i;
        fail(SPMV_ERR_INTERNAL, "plan save: a launch refers to memory outside the plan's arrays");
    };
    auto scratch_index = [&](const void *p) -> int64_t {
        if (!p) return -1;
        for (size_t i = 0; i < plan.scratch.size(); ++i)
            if (plan.scratch[i].ptr == p) return (int64_t)i;
        fail(SPMV_ERR_INTERNAL, "plan save: a launch refers to an unknown scratch buffer");
    };
    w.i64((int64_t)plan.parts.size());
    for (const Part &p : plan.parts) {
        Part q = p;
        w.str(q.name);
        part_scalars(q, [&](int64_t &v) { w.i64(v); });
        w.i64(array_index(p.p0)); w.i64(array_index(p.p1)); w.i64(array_index(p.p2));
        w.i64(array_index(p.p3)); w.i64(array_index(p.p4)); w.i64(array_index(p.p5));
        w.i64(scratch_index(p.scratch));
        w.i64(scratch_index(p.scratch2));
    }
    w.i64((int64_t)plan.log.size());
    for (const CandidateLog &l : plan.log) {
        w.str(l.spec);
        w.f64(l.build_ms);
        w.f64(l.run_us);
        w.f64(l.pred_us);
        w.f64(l.playoff_us);
        w.str(l.note);
    }
    FILE *f = std::fopen(path, "wb");
    if (!f) fail(SPMV_ERR_INVALID_ARG, std::string("plan save: cannot open ") + path + " for writing");
    const uint64_t size = w.buf.size(), hash = fnv1a(w.buf.data(), w.buf.size());
    bool ok = std::fwrite(kMagic, 1, 8, f) == 8 && std::fwrite(&size, 8, 1, f) == 1 && std::fwrite(&hash, 8, 1, f) == 1;
    ok = ok && (size == 0 || std::fwrite(w.buf.data(), 1, w.buf.size(), f) == w.buf.size());
    ok = (std::fclose(f) == 0) && ok;
    if (!ok) fail(SPMV_ERR_INVALID_ARG, std::string("plan save: writing ") + path + " failed");
}

std::unique_ptr<Plan> load_plan(const char *path, const Allocator &mem) {
    FILE *f = std::fopen(path, "rb");
    if (!f) fail(SPMV_ERR_INVALID_ARG, std::string("plan load: cannot open ") + path);
    std::vector<unsigned char> buf;
    {
        unsigned char head[24];
        const bool got = std::fread(head, 1, 24, f) == 24;
        uint64_t size = 0;
        if (got) std::memcpy(&size, head + 8, 8);
        if (!got || std::memcmp(head, kMagic, 8) != 0 || size > ((uint64_t)1 << 40)) {
            std::fclose(f);
            fail(SPMV_ERR_INVALID_ARG, "plan load: not a plan file of this library version");
        }
        std::fseek(f, 0, SEEK_END);
        const long total = std::ftell(f);
        if (total < 0 || (uint64_t)total != size + 24) {
            std::fclose(f);
            fail(SPMV_ERR_INVALID_ARG, "plan load: the file's length does not match its header");
        }
        std::fseek(f, 24, SEEK_SET);
        buf.resize((size_t)size);
        const bool all = size == 0 || std::fread(buf.data(), 1, (size_t)size, f) == (size_t)size;
        std::fclose(f);
        uint64_t hash = 0;
        std::memcpy(&hash, head + 16, 8);
        if (!all || fnv1a(buf.data(), buf.size()) != hash) fail(SPMV_ERR_INVALID_ARG, "plan load: the file is damaged (hash mismatch)");
    }
    Reader r{buf.data(), buf.data() + buf.size()};
    std::unique_ptr<Plan> plan(new Plan);
    plan->mem = mem;
    const int64_t dt = r.i64();
    if (dt != SPMV_F32 && dt != SPMV_F64) fail(SPMV_ERR_INVALID_ARG, "plan load: unknown dtype");
    plan->dtype = (spmv_dtype_t)dt;
    plan->nrows = r.count((int64_t)1 << 31);
    plan->ncols = r.count((int64_t)1 << 31);
    plan->nnz = r.count((int64_t)1 << 31);
    plan->spec = parse_spec(r.str());
    Census &c = plan->census;
    c.nrows = r.i64(); c.ncols = r.i64(); c.nnz = r.i64(); c.min_len = r.i64(); c.max_len = r.i64(); c.empty_rows = r.i64();
    c.mean_len = r.f64(); c.var_len = r.f64();
    for (int k = 0; k <= 20; ++k) { c.rows_over[k] = r.i64(); c.nnz_over[k] = r.i64(); }
    const int64_t nd = r.count(1 << 20);
    for (int64_t d = 0; d < nd; ++d) c.diag_offsets.push_back((int32_t)r.i64());
    c.diag_nnz = r.i64();
    for (int b = 0; b < 5; ++b) { c.blocks[b] = r.i64(); c.block_fill[b] = r.f64(); }
    c.cols_sorted = r.i64() != 0;
    const int64_t narr = r.count(1 << 16);
    for (int64_t i = 0; i < narr; ++i) {
        DevArray a;
        a.name = r.str();
        a.elem_bytes = (int)r.count(16);
        a.count = r.count(r.end - r.p);
        a.read_per_run = r.i64() != 0;
        if (a.elem_bytes != 1 && a.elem_bytes != 2 && a.elem_bytes != 4 && a.elem_bytes != 8)
            fail(SPMV_ERR_INVALID_ARG, "plan load: bad element size");
        const size_t bytes = (size_t)a.count * (size_t)a.elem_bytes;
        r.need(bytes);
        a.ptr = mem.alloc(std::max<size_t>(bytes, (size_t)a.elem_bytes), mem.user);
        if (!a.ptr) fail(SPMV_ERR_ALLOC, "plan load: device allocation of " + std::to_string(bytes) + " bytes failed (" + a.name + ")");
        if (a.count >= 2 && is_metadata_array(a.name)) {
            std::vector<int64_t> aligned((bytes + 7) / 8);   // the payload is not aligned for 4- or 8-byte reads
            std::memcpy(aligned.data(), r.p, bytes);
            a.model = fit_array(aligned.data(), a.elem_bytes, a.count);
        }
        plan->arrays.push_back(a);   // owned from here on
        if (bytes) {
            if (mem.host_only) {
                std::memcpy(a.ptr, r.p, bytes);
            } else {
                hipError_t err = hipMemcpy(a.ptr, r.p, bytes, hipMemcpyHostToDevice);
                if (err != hipSuccess) fail(SPMV_ERR_HIP, std::string("plan load: hipMemcpy H2D (") + a.name + "): " + hipGetErrorString(err));
            }
            r.p += bytes;
        }
    }
    const int64_t nscr = r.count(1 << 16);
    for (int64_t i = 0; i < nscr; ++i) {
        DevArray a;
        a.name = r.str();
        a.elem_bytes = (int)r.count(16);
        a.count = r.count((int64_t)1 << 40);
        const size_t bytes = (size_t)a.count * (size_t)a.elem_bytes;
        a.ptr = mem.alloc(std::max<size_t>(bytes, 16), mem.user);
        if (!a.ptr) fail(SPMV_ERR_ALLOC, "plan load: device allocation of the scratch buffer " + a.name + " failed");
        plan->scratch.push_back(a);
    }
    auto array_ptr = [&](int64_t i) -> const void * {
        if (i == -1) return nullptr;
        if (i < 0 || i >= (int64_t)plan->arrays.size()) fail(SPMV_ERR_INVALID_ARG, "plan load: array index out of range");
        return plan->arrays[(size_t)i].ptr;
    };
    const int64_t nparts = r.count(1 << 16);
    for (int64_t i = 0; i < nparts; ++i) {
        Part q;
        q.name = r.str();
        part_scalars(q, [&](int64_t &v) { v = r.i64(); });
        if ((int)q.kind < 0 || (int)q.kind > (int)K_LAST) fail(SPMV_ERR_INVALID_ARG, "plan load: unknown launch kind");
        q.p0 = array_ptr(r.i64()); q.p1 = array_ptr(r.i64()); q.p2 = array_ptr(r.i64());
        q.p3 = array_ptr(r.i64()); q.p4 = array_ptr(r.i64()); q.p5 = array_ptr(r.i64());
        for (void **dst : {&q.scratch, &q.scratch2}) {
            const int64_t si = r.i64();
            if (si == -1) continue;
            if (si < 0 || si >= (int64_t)plan->scratch.size()) fail(SPMV_ERR_INVALID_ARG, "plan load: scratch index out of range");
            *dst = plan->scratch[(size_t)si].ptr;
        }
        plan->parts.push_back(q);
    }
    const int64_t nlog = r.count(1 << 20);
    for (int64_t i = 0; i < nlog; ++i) {
        CandidateLog l;
        l.spec = r.str();
        l.build_ms = r.f64();
        l.run_us = r.f64();
        l.pred_us = r.f64();
        l.playoff_us = r.f64();
        l.note = r.str();
        plan->log.push_back(l);
    }
    if (r.p != r.end) fail(SPMV_ERR_INVALID_ARG, "plan load: trailing bytes after the plan");
    if (plan_wants_jit(plan->spec)) jit_compile_plan(*plan);
    return plan;
}

}  // namespace spmv
