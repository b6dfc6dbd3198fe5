/*
 * Seeded synthetic sparse-matrix generators for the SpMV workloads.
 *
 * This file only produces INPUTS (CSR arrays and dense vectors).  It holds none
 * of the SpMV method's arithmetic and is shared by the test oracle and by the
 * GPU library's tests/bench purely as a data source.
 *
 * Every random quantity is a pure function of (seed, stream, row, counter), so
 * the output does not depend on the number of OpenMP threads.
 *
 * The five matrix families stand in for the paper's SuiteSparse test set
 * (Section VII-A: rows > 9K, 50K..60M non-zeros, "irregular" = row-length
 * variance > 100), which is not available offline:
 *   1 uniform      fixed k non-zeros per row, uniform distinct columns
 *   2 laplace2d    5-point stencil on a g x g grid (+ small perturbation)
 *   3 powerlaw     shifted-Pareto row lengths, uniform distinct columns
 *   4 fem3         dense 3x3 blocks clustered around the diagonal
 *   5 hybrid       a few very long rows + many very short rows (the pattern
 *                  of the paper's Limitation case, Section VII-F)
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC gen.c -o libspmvgen.so -lm
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

/* ---- counter-based random numbers (splitmix64 finaliser, chained) -------- */
static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
enum { ST_LEN = 1, ST_COL = 2, ST_VAL = 3, ST_VEC = 4, ST_HEAVY = 5 };

static inline uint64_t rnd(uint64_t seed, uint64_t stream, uint64_t a, uint64_t b) {
    return mix64(mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) + a) + b);
}
/* uniform in [0,1) with 53 bits */
static inline double u01(uint64_t r) { return (double)(r >> 11) * (1.0 / 9007199254740992.0); }
/* uniform integer in [0,m) */
static inline uint64_t below(uint64_t r, uint64_t m) { return (uint64_t)(((__uint128_t)r * m) >> 64); }

/* value modes: 0 = uniform real in [-1,1); 1 = non-zero integer in [-vmax,vmax] */
static inline double draw_value(uint64_t r, int vmode, int vmax) {
    if (vmode == 0) return 2.0 * u01(r) - 1.0;
    int64_t v = (int64_t)below(r, (uint64_t)(2 * vmax)) - vmax; /* [-vmax, vmax-1] */
    if (v >= 0) v += 1;                                          /* skip zero */
    return (double)v;
}

void gen_vector(int64_t n, uint64_t seed, int vmode, int vmax, double *x) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) x[i] = draw_value(rnd(seed, ST_VEC, (uint64_t)i, 0), vmode, vmax);
}

/* ---- k distinct sorted integers from [lo, lo+m) --------------------------- */
typedef struct { uint64_t *bits; int64_t nwords; int32_t *tmp; int64_t tmpcap; } scratch_t;

static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

static void scratch_need(scratch_t *s, int64_t m) {
    int64_t nw = (m + 63) / 64;
    if (nw > s->nwords) {
        free(s->bits);
        s->bits = (uint64_t *)calloc((size_t)nw, 8);
        s->nwords = nw;
    }
}

/* draws use rnd(seed, ST_COL, row, j) for j = 0,1,2,... (rejected draws included) */
static void distinct_sorted(uint64_t seed, uint64_t row, int64_t lo, int64_t m, int64_t k,
                            int32_t *out, scratch_t *s) {
    uint64_t j = 0;
    if (k <= 0) return;
    if (k >= m) { for (int64_t i = 0; i < m; ++i) out[i] = (int32_t)(lo + i); return; }
    if (k <= 32) {
        int64_t cnt = 0;
        while (cnt < k) {
            int32_t c = (int32_t)below(rnd(seed, ST_COL, row, j++), (uint64_t)m);
            int dup = 0;
            for (int64_t t = 0; t < cnt; ++t) if (out[t] == c) { dup = 1; break; }
            if (dup) continue;
            int64_t p = cnt++;                       /* insertion keeps it sorted */
            while (p > 0 && out[p - 1] > c) { out[p] = out[p - 1]; --p; }
            out[p] = c;
        }
        for (int64_t t = 0; t < k; ++t) out[t] += (int32_t)lo;
        return;
    }
    scratch_need(s, m);
    int64_t cnt = 0;
    while (cnt < k) {
        int64_t c = (int64_t)below(rnd(seed, ST_COL, row, j++), (uint64_t)m);
        uint64_t bit = 1ull << (c & 63);
        if (s->bits[c >> 6] & bit) continue;
        s->bits[c >> 6] |= bit;
        out[cnt++] = (int32_t)c;
    }
    for (int64_t t = 0; t < k; ++t) s->bits[out[t] >> 6] = 0;   /* clear touched words */
    qsort(out, (size_t)k, sizeof(int32_t), cmp_i32);
    for (int64_t t = 0; t < k; ++t) out[t] += (int32_t)lo;
}

/* ---- row-length laws ------------------------------------------------------ */
typedef struct {
    int kind;
    int64_t n;        /* rows (= cols); for fem3: scalar rows = 3 * block rows */
    int64_t p0, p1, p2, p3;
    double d0, d1;
    uint64_t seed;
    int vmode, vmax;
} cfg_t;

/* hybrid: the sorted ids of the heavy rows (n_heavy distinct rows, uniform) */
void gen_hybrid_heavy_rows(int64_t n, int64_t n_heavy, uint64_t seed, int32_t *ids) {
    scratch_t s = {0};
    /* reuse the distinct sampler on its own stream: row key = all-ones */
    uint64_t j = 0; int64_t cnt = 0;
    scratch_need(&s, n);
    while (cnt < n_heavy) {
        int64_t c = (int64_t)below(rnd(seed, ST_HEAVY, 0, j++), (uint64_t)n);
        uint64_t bit = 1ull << (c & 63);
        if (s.bits[c >> 6] & bit) continue;
        s.bits[c >> 6] |= bit;
        ids[cnt++] = (int32_t)c;
    }
    qsort(ids, (size_t)n_heavy, sizeof(int32_t), cmp_i32);
    free(s.bits);
}

static int64_t row_len(const cfg_t *c, int64_t r, const uint8_t *heavy) {
    switch (c->kind) {
    case 1: return c->p0;                                         /* k per row */
    case 2: {                                                     /* 5-point stencil */
        int64_t g = c->p0, i = r / g, j = r % g;
        return 1 + (i > 0) + (i < g - 1) + (j > 0) + (j < g - 1);
    }
    case 3: {                                                     /* shifted Pareto */
        double u = 1.0 - u01(rnd(c->seed, ST_LEN, (uint64_t)r, 0));      /* (0,1] */
        double L = floor(c->d0 * (pow(u, -1.0 / (c->d1 - 1.0)) - 1.0)) + 1.0;
        int64_t cap = c->p0 < c->n ? c->p0 : c->n;
        if (!(L >= 1.0)) L = 1.0;
        if (L > (double)cap) L = (double)cap;
        return (int64_t)L;
    }
    case 4: {                                                     /* 3 * (#blocks) */
        int64_t br = r / 3, nb = c->n / 3;
        int64_t kmin = c->p0, kmax = c->p1, w = c->p2;
        int64_t lo = br - w < 0 ? 0 : br - w, hi = br + w > nb - 1 ? nb - 1 : br + w;
        int64_t k = kmin + (int64_t)below(rnd(c->seed, ST_LEN, (uint64_t)br, 0), (uint64_t)(kmax - kmin + 1));
        if (k > hi - lo + 1) k = hi - lo + 1;
        return 3 * k;
    }
    case 5: {
        if (heavy[r]) return c->p1 < c->n ? c->p1 : c->n;
        int64_t lo = c->p2, hi = c->p3;
        int64_t k = lo + (int64_t)below(rnd(c->seed, ST_LEN, (uint64_t)r, 0), (uint64_t)(hi - lo + 1));
        return k < c->n ? k : c->n;
    }
    }
    return 0;
}

static void fill_row(const cfg_t *c, int64_t r, int64_t len, int32_t *col, double *val, scratch_t *s) {
    switch (c->kind) {
    case 1: case 3: case 5:
        distinct_sorted(c->seed, (uint64_t)r, 0, c->n, len, col, s);
        for (int64_t k = 0; k < len; ++k)
            val[k] = draw_value(rnd(c->seed, ST_VAL, (uint64_t)r, (uint64_t)k), c->vmode, c->vmax);
        break;
    case 2: {
        int64_t g = c->p0, i = r / g, j = r % g, k = 0;
        double amp = c->d0;
        int64_t cc[5]; double base[5];
        if (i > 0)     { cc[k] = r - g; base[k++] = -1.0; }
        if (j > 0)     { cc[k] = r - 1; base[k++] = -1.0; }
        cc[k] = r; base[k++] = 4.0;
        if (j < g - 1) { cc[k] = r + 1; base[k++] = -1.0; }
        if (i < g - 1) { cc[k] = r + g; base[k++] = -1.0; }
        for (int64_t t = 0; t < k; ++t) {
            col[t] = (int32_t)cc[t];
            double p = (c->vmode == 0) ? amp * (2.0 * u01(rnd(c->seed, ST_VAL, (uint64_t)r, (uint64_t)t)) - 1.0) : 0.0;
            val[t] = base[t] + p;
        }
        break;
    }
    case 4: {
        /* the three scalar rows of a block row share the block pattern */
        int64_t br = r / 3, nb = c->n / 3, w = c->p2, k = len / 3;
        int64_t lo = br - w < 0 ? 0 : br - w, hi = br + w > nb - 1 ? nb - 1 : br + w;
        int64_t m = hi - lo + 1;
        /* k-1 distinct off-diagonal block columns: sample from the window with the
           diagonal removed (positions >= br-lo shift by one), then add the diagonal */
        int32_t *bc = col + 2 * k;                    /* build at the tail, expand forward */
        distinct_sorted(c->seed, (uint64_t)br, 0, m - 1, k - 1, bc, s);
        int64_t dpos = br - lo, ins = 0;
        for (int64_t t = 0; t < k - 1; ++t) { if (bc[t] >= dpos) bc[t] += 1; }
        /* insert the diagonal, keeping order */
        while (ins < k - 1 && bc[ins] < dpos) ++ins;
        for (int64_t t = k - 1; t > ins; --t) bc[t] = bc[t - 1];
        bc[ins] = (int32_t)dpos;
        for (int64_t t = 0; t < k; ++t) {
            int64_t b = lo + bc[t];
            col[3 * t + 0] = (int32_t)(3 * b);
            col[3 * t + 1] = (int32_t)(3 * b + 1);
            col[3 * t + 2] = (int32_t)(3 * b + 2);
        }
        for (int64_t t = 0; t < len; ++t)
            val[t] = draw_value(rnd(c->seed, ST_VAL, (uint64_t)r, (uint64_t)t), c->vmode, c->vmax);
        break;
    }
    }
}

/*
 * Two-phase interface.
 *   gen_row_ptr : fills row_ptr[0..n] (int64).  Returns nnz, or -1 on bad arguments.
 *   gen_fill    : fills col_idx / values for the same parameters (row_ptr from phase one).
 * kind / parameters:
 *   1 uniform   p0 = non-zeros per row
 *   2 laplace2d p0 = grid side g (n must equal g*g), d0 = perturbation amplitude
 *   3 powerlaw  p0 = cap on row length, d0 = scale s, d1 = exponent (2.1)
 *   4 fem3      n = 3 * block rows, p0 = kmin, p1 = kmax blocks per block row, p2 = half window
 *   5 hybrid    p0 = number of heavy rows, p1 = heavy row length, p2..p3 = light length range
 */
static uint8_t *heavy_mask(const cfg_t *c) {
    if (c->kind != 5) return NULL;
    uint8_t *m = (uint8_t *)calloc((size_t)c->n, 1);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(c->p0 > 0 ? c->p0 : 1));
    gen_hybrid_heavy_rows(c->n, c->p0, c->seed, ids);
    for (int64_t t = 0; t < c->p0; ++t) m[ids[t]] = 1;
    free(ids);
    return m;
}

static int cfg_ok(const cfg_t *c) {
    if (c->n <= 0 || c->n > 2147483647LL) return 0;
    switch (c->kind) {
    case 1: return c->p0 >= 0 && c->p0 <= c->n;
    case 2: return c->p0 > 0 && c->p0 * c->p0 == c->n;
    case 3: return c->p0 >= 1 && c->d0 > 0 && c->d1 > 1.0;
    case 4: return c->n % 3 == 0 && c->p0 >= 1 && c->p1 >= c->p0 && c->p2 >= 0;
    case 5: return c->p0 >= 0 && c->p0 <= c->n && c->p1 >= 0 && c->p2 >= 0 && c->p3 >= c->p2;
    }
    return 0;
}

int64_t gen_row_ptr(int kind, int64_t n, int64_t p0, int64_t p1, int64_t p2, int64_t p3,
                    double d0, double d1, uint64_t seed, int64_t *row_ptr) {
    cfg_t c = {kind, n, p0, p1, p2, p3, d0, d1, seed, 0, 1};
    if (!cfg_ok(&c)) return -1;
    uint8_t *hm = heavy_mask(&c);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) row_ptr[r + 1] = row_len(&c, r, hm);
    row_ptr[0] = 0;
    for (int64_t r = 0; r < n; ++r) row_ptr[r + 1] += row_ptr[r];
    free(hm);
    return row_ptr[n];
}

int gen_fill(int kind, int64_t n, int64_t p0, int64_t p1, int64_t p2, int64_t p3,
             double d0, double d1, uint64_t seed, int vmode, int vmax,
             const int64_t *row_ptr, int32_t *col_idx, double *values) {
    cfg_t c = {kind, n, p0, p1, p2, p3, d0, d1, seed, vmode, vmax};
    if (!cfg_ok(&c)) return -1;
#pragma omp parallel
    {
        scratch_t s = {0};
#pragma omp for schedule(dynamic, 256)
        for (int64_t r = 0; r < n; ++r) {
            int64_t b = row_ptr[r], len = row_ptr[r + 1] - b;
            fill_row(&c, r, len, col_idx + b, values + b, &s);
        }
        free(s.bits);
    }
    return 0;
}
