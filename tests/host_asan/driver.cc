// Sanitizer driver for the host side of the library (format builder, census, plan-spec parser,
// Matrix Market reader, C ABI), built with -fsanitize=address,undefined by tests/test_host_sanitizers.py.
// Builds host-only plans for a list of plan specs over seeded random matrices (ragged rows, empty
// rows, repeated and unsorted columns, a long row, rectangular shapes), copies every format array
// out, and feeds well-formed and malformed Matrix Market text to the reader.  Prints "OK <n plans>".
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/spmv.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
}

struct Csr {
    int64_t nrows, ncols;
    std::vector<int32_t> rp, ci;
    std::vector<double> va;
    std::vector<float> vf;
};

static Csr make(int64_t nrows, int64_t ncols, int maxlen, bool sorted, int64_t long_row, int block) {
    Csr m;
    m.nrows = nrows;
    m.ncols = ncols;
    m.rp.push_back(0);
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t L = (rnd() % 5 == 0) ? 0 : (int64_t)(rnd() % (uint64_t)(maxlen + 1));
        if (r == long_row) L = 3000;
        if (block) L = 0;
        std::vector<int32_t> cols;
        if (block) {   // dense block x block structure: the rows of a block row share their block columns
            const int64_t br = r / block;
            uint64_t keep = state;
            state = 0xABCDEFull + (uint64_t)br * 7919;
            const int nb = 1 + (int)(rnd() % 6);
            for (int k = 0; k < nb; ++k) {
                const int64_t bc = (int64_t)(rnd() % (uint64_t)(ncols / block));
                for (int q = 0; q < block; ++q) cols.push_back((int32_t)(bc * block + q));
            }
            state = keep;
        } else {
            for (int64_t k = 0; k < L; ++k) cols.push_back((int32_t)(rnd() % (uint64_t)ncols));
        }
        if (sorted || block) {
            for (size_t i = 1; i < cols.size(); ++i)
                for (size_t j = i; j > 0 && cols[j] < cols[j - 1]; --j) std::swap(cols[j], cols[j - 1]);
        }
        for (int32_t c : cols) {
            m.ci.push_back(c);
            const double v = (double)((int)(rnd() % 7) - 3);
            m.va.push_back(v);
            m.vf.push_back((float)v);
        }
        m.rp.push_back((int32_t)m.ci.size());
    }
    return m;
}

static int plans = 0;
static const char *g_dir = "/tmp";

// save the plan, read it back host-only, then feed every kind of damaged copy to the reader
static void files(spmv_plan_t *p) {
    const std::string path = std::string(g_dir) + "/plan.bin", bad = std::string(g_dir) + "/bad.bin";
    if (spmv_plan_save(p, path.c_str()) != SPMV_OK) std::exit(6);
    spmv_options_t o;
    std::memset(&o, 0, sizeof o);
    o.host_only = 1;
    spmv_plan_t *q = nullptr;
    if (spmv_plan_load(&q, path.c_str(), &o) != SPMV_OK) std::exit(7);
    spmv_plan_destroy(q);
    FILE *f = std::fopen(path.c_str(), "rb");
    std::vector<unsigned char> data;
    unsigned char chunk[4096];
    size_t n;
    while ((n = std::fread(chunk, 1, sizeof chunk, f)) > 0) data.insert(data.end(), chunk, chunk + n);
    std::fclose(f);
    for (int variant = 0; variant < 6; ++variant) {
        std::vector<unsigned char> d = data;
        if (variant == 0) d.resize(d.size() / 2);
        if (variant == 1) d.resize(17);
        if (variant == 2) d[d.size() / 3] ^= 0x40;
        if (variant == 3) d[9] ^= 0x7f;          // the size field
        if (variant == 4) d.push_back(1);
        if (variant == 5) d.clear();
        f = std::fopen(bad.c_str(), "wb");
        if (!d.empty()) std::fwrite(d.data(), 1, d.size(), f);
        std::fclose(f);
        q = nullptr;
        if (spmv_plan_load(&q, bad.c_str(), &o) == SPMV_OK || q) std::exit(8);
    }
}

static void one(const Csr &m, const char *spec, spmv_dtype_t dt, bool must_build) {
    spmv_options_t o;
    std::memset(&o, 0, sizeof o);
    o.force_plan = spec;
    o.host_only = 1;
    o.host_threads = 3;
    spmv_plan_t *p = nullptr;
    const void *vals = dt == SPMV_F64 ? (const void *)m.va.data() : (const void *)m.vf.data();
    const spmv_status_t st = spmv_plan_create(&p, m.nrows, m.ncols, (int64_t)m.ci.size(), m.rp.data(), m.ci.data(), vals, dt, &o);
    if (st != SPMV_OK) {
        if (must_build || (st != SPMV_ERR_UNSUPPORTED && st != SPMV_ERR_INVALID_ARG)) {
            std::fprintf(stderr, "spec %s: status %d: %s\n", spec, (int)st, spmv_last_error());
            std::exit(2);
        }
        return;
    }
    ++plans;
    int n = 0;
    spmv_plan_array_count(p, &n);
    for (int i = 0; i < n; ++i) {
        const char *name = nullptr;
        int eb = 0;
        int64_t cnt = 0;
        spmv_plan_array_info(p, i, &name, &eb, &cnt);
        std::vector<char> buf((size_t)(cnt * eb) + 1);
        if (spmv_plan_array_copy(p, i, buf.data()) != SPMV_OK) std::exit(3);
    }
    size_t need = 0;
    spmv_plan_describe(p, nullptr, 0, &need);
    std::vector<char> d(need);
    spmv_plan_describe(p, d.data(), need, nullptr);
    if (spmv_run(p, m.va.data(), (void *)m.va.data(), nullptr) == SPMV_OK) std::exit(4);   // host-only plans refuse to run
    if (plans % 7 == 0) files(p);
    spmv_plan_destroy(p);
}

static void mm(const char *dir, const char *text, bool ok) {
    const std::string path = std::string(dir) + "/t.mtx";
    FILE *f = std::fopen(path.c_str(), "wb");
    std::fwrite(text, 1, std::strlen(text), f);
    std::fclose(f);
    int64_t nr, nc, nz;
    int32_t *rp, *ci;
    void *va;
    const spmv_status_t st = spmv_mm_read(path.c_str(), SPMV_F64, &nr, &nc, &nz, &rp, &ci, &va);
    if ((st == SPMV_OK) != ok) {
        std::fprintf(stderr, "matrix market case gave status %d\n%s\n", (int)st, text);
        std::exit(5);
    }
    spmv_mm_free(rp, ci, va);
}

int main(int argc, char **argv) {
    const char *dir = argc > 1 ? argv[1] : "/tmp";
    g_dir = dir;
    const char *specs[] = {
        "light=csrv", "light=csrv,lpr=8,sigma=64", "light=csrv,chunk=256", "light=sell", "light=sell,sigma=128,remap=1",
        "light=sell,sigma=-1", "light=bin,smax=4,sigma=128,chunk=512", "light=coo", "light=nnzb,r=4", "light=nnzb,r=16",
        "light=xs,k=8,sigma=256", "light=xnb,k=16,r=8", "light=xl,w=256,rb=128,chunk=512", "light=xl",
        "heavy=100,tile=512,light=sell,sigma=64", "heavy=100,tile=512,hd=1,light=xl,w=128,rb=64", "heavy=100,tile=256,light=xnb,k=8,r=4",
        "dia=1,light=sell", "dia=1,dia_fill=0.9,light=csrv,lpr=2",
        "light=bsell,block=2,sigma=128", "light=bsell,block=3,sigma=0", "light=bsell,block=3,sigma=2048,xwin=1,remap=1",
        "light=bsell,block=4,sigma=64,remap=1", "light=wbm", "light=csrv,lpr=256,chunk=512", "light=bin,smax=4,sigma=128,chunk=512,wg=1",
        "rows(4:32){light=sell,sigma=64}{light=csrv,lpr=8}{heavy=32,tile=256,light=csrv}", "bin2(5){light=sell}{light=wbm}",
        "cut(4:16){light=sell,sigma=0}", "cols(3){rows(8){light=xl,w=128,rb=64}{light=nnzb,r=4}}", "light=sell,sigma=64,jit=1",
        "heavy=100,tile=512,light=xl,w=128,rb=64,jit=1", "heavy=100,tile=512,piece=8,light=xl,w=128,rb=64",
        "heavy=100,tile=256,hd=1,piece=16,light=csrv", "heavy=40,tile=4096,piece=4,light=sell,sigma=64",
    };
    const Csr mats[] = {
        make(777, 1234, 40, false, 5, 0), make(1500, 900, 12, true, -1, 0), make(64, 64, 64, true, -1, 0),
        make(1, 5000, 10, false, 0, 0),   make(4099, 4099, 6, true, 17, 0), make(0, 0, 0, true, -1, 0),
        make(600, 600, 0, true, -1, 2),   make(603, 603, 0, true, -1, 3),   make(600, 600, 0, true, -1, 4),
    };
    for (const Csr &m : mats)
        for (const char *s : specs) {
            one(m, s, SPMV_F64, false);
            one(m, s, SPMV_F32, false);
        }
    // a tridiagonal matrix for the diagonal part
    {
        Csr t;
        t.nrows = t.ncols = 999;
        t.rp.push_back(0);
        for (int64_t r = 0; r < 999; ++r) {
            for (int64_t c = r - 1; c <= r + 1; ++c)
                if (c >= 0 && c < 999) {
                    t.ci.push_back((int32_t)c);
                    t.va.push_back(1.0 + (double)(c - r));
                    t.vf.push_back(1.0f);
                }
            t.rp.push_back((int32_t)t.ci.size());
        }
        one(t, "dia=1,light=sell", SPMV_F64, true);
        one(t, "dia=1,dia_fill=0.99,light=xl,w=64,rb=64", SPMV_F32, true);
    }
    // plan-spec strings that must be refused cleanly
    const char *bad[] = {"rows(4){light=sell", "rows(4:2){light=sell}", "cols(99){light=sell}", "rows(4){dia=1,light=sell}{light=sell}", "bin2(3){light=sell}",
                         "light=", "light=nope", "tile=7", "heavy=-1", "hd=1", "light=bsell,dia=1", "k=9", "sigma", "rb=1", "=,=", ",,,"};
    for (const char *s : bad) one(mats[0], s, SPMV_F64, false);
    mm(dir, "%%MatrixMarket matrix coordinate real general\n3 3 3\n1 1 1.5\n3 2 -2\n2 3 4e1\n", true);
    mm(dir, "%%MatrixMarket matrix coordinate pattern symmetric\n3 3 2\n2 1\n3 3\n", true);
    mm(dir, "%%MatrixMarket matrix coordinate integer skew-symmetric\r\n% comment\r\n\r\n3 3 1\r\n3 1 7\r\n", true);
    mm(dir, "%%MatrixMarket matrix coordinate real general\n3 3 2\n1\n2 3 5.0\n", false);
    mm(dir, "%%MatrixMarket matrix coordinate real general\n3 3 2\n1 2", false);
    mm(dir, "%%MatrixMarket matrix coordinate real general\n3 3 2000000000\n1 1 1.0\n", false);
    mm(dir, "%%MatrixMarket matrix coordinate real general\n3 3", false);
    mm(dir, "", false);
    std::printf("OK %d plans\n", plans);
    return 0;
}
