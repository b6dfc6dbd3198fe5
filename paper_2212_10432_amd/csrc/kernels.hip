// Hand-written gfx950 SpMV kernels: the "implementing" stage of the paper (Table II; Section V-C
// "Distribution" reads the block metadata, "Reduction" multiplies and reduces by row).
//
// Mapping of the paper's parallelism levels (Section IV-A, CUDA terms) to CDNA4:
//   BMTB (thread block) -> workgroup, BMW (warp, 32 lanes) -> wavefront (64 lanes), BMT -> lane.
//
// Every kernel streams the matrix arrays exactly once with non-temporal loads (they are never
// reused, and must not evict x from the L2), gathers x through the ordinary cached path, and
// writes each y element once.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace spmv {
namespace {

constexpr int kWG = 256;   // workgroup size of the streaming kernels: 4 wavefronts

template <typename T>
__device__ __forceinline__ T ldnt(const T *p) {
    return __builtin_nontemporal_load(p);
}

// Workgroup ids are dealt round-robin to the 8 XCDs, each with a private L2.  With remap on, XCD
// k works on the k-th contiguous eighth of the blocks, so neighbouring rows (which share their
// window of x in banded matrices) meet in one L2.
__device__ __forceinline__ int64_t logical_block(int64_t bid, int64_t nblk, int remap) {
    if (!remap) return bid;
    const int64_t per = nblk >> 3;
    if (bid >= (per << 3)) return bid;
    return (bid & 7) * per + (bid >> 3);
}

template <typename T>
__device__ __forceinline__ void atomic_add(T *p, T v) {
    unsafeAtomicAdd(p, v);   // hardware floating-point atomic in the L2 (GMEM_ATOM_RED)
}

// Sum over aligned groups of LANES lanes; every lane of the wavefront must call it.
template <int LANES, typename T>
__device__ __forceinline__ T group_sum(T v) {
#pragma unroll
    for (int o = LANES >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// ---- y[rows[i]] = 0 : rows that are later accumulated with atomics --------------------------
template <typename T>
__global__ __launch_bounds__(kWG) void k_zero_rows(const int32_t *__restrict__ rows, int64_t n,
                                                   T *__restrict__ y) {
    int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i < n) y[rows[i]] = T(0);
}

// ---- DIA: one lane per row, diagonals stored column-major (d * ld + row) --------------------
// THREAD_TOTAL_RED over the ndiag slots of a row; the column index is arithmetic (row + offset),
// i.e. the index array is replaced by a linear model (Section V-D).
template <typename T, bool ACC>
__global__ __launch_bounds__(kWG) void k_dia(const int32_t *__restrict__ offs, int ndiag,
                                             const T *__restrict__ vals, int64_t ld,
                                             const T *__restrict__ x, T *__restrict__ y,
                                             int64_t nrows, int64_t ncols) {
    int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i >= nrows) return;
    T acc = T(0);
    for (int d = 0; d < ndiag; ++d) {
        int64_t c = i + offs[d];
        T v = ldnt(vals + (int64_t)d * ld + i);
        if (c >= 0 && c < ncols) acc += v * x[c];
    }
    y[i] = ACC ? y[i] + acc : acc;
}

// ---- SELL: one wavefront per slice of 64 rows, one lane per row -----------------------------
// BMW_ROW_BLOCK(64) + BMT_ROW_BLOCK(1) + BMW_PAD + THREAD_TOTAL_RED.  Entry j of the row held by
// `lane` sits at slice_ptr[s] + 64*j + lane, so every load of a wavefront is one contiguous run.
template <typename T, bool ROWS, bool ACC>
__global__ __launch_bounds__(kWG) void k_sell(const int64_t *__restrict__ slice_ptr,
                                              const int32_t *__restrict__ cols,
                                              const T *__restrict__ vals,
                                              const int32_t *__restrict__ rows,
                                              const T *__restrict__ x, T *__restrict__ y,
                                              int64_t nslices, int64_t nrows_part, int remap) {
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t s = blk * (kWG / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= nslices) return;
    const int64_t b = slice_ptr[s];
    const int w = (int)((slice_ptr[s + 1] - b) >> 6);
    const int32_t *c = cols + b + lane;
    const T *v = vals + b + lane;
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    int j = 0;
    for (; j + 4 <= w; j += 4) {
        const int32_t c0 = ldnt(c + (j + 0) * 64), c1 = ldnt(c + (j + 1) * 64);
        const int32_t c2 = ldnt(c + (j + 2) * 64), c3 = ldnt(c + (j + 3) * 64);
        const T v0 = ldnt(v + (j + 0) * 64), v1 = ldnt(v + (j + 1) * 64);
        const T v2 = ldnt(v + (j + 2) * 64), v3 = ldnt(v + (j + 3) * 64);
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
        a2 += v2 * x[c2];
        a3 += v3 * x[c3];
    }
    for (; j < w; ++j) a0 += ldnt(v + j * 64) * x[ldnt(c + j * 64)];
    const T acc = (a0 + a1) + (a2 + a3);
    const int64_t r = s * 64 + lane;
    if (r < nrows_part) {
        const int64_t row = ROWS ? (int64_t)rows[r] : r;
        y[row] = ACC ? y[row] + acc : acc;
    }
}

// ---- CSR segments: LPR lanes per row segment ------------------------------------------------
// BMT_COL_BLOCK inside a row + WARP_TOTAL_RED over the LPR lanes of the group.  A row longer
// than the plan's chunk is cut into several segments (BMW_COL_BLOCK); those carry ~row in
// seg_row and add their partial sum atomically (GMEM_ATOM_RED) into a y element zeroed before.
template <typename T, int LPR, bool ROWS, bool ACC>
__global__ __launch_bounds__(kWG) void k_csrv(const int32_t *__restrict__ seg_ptr,
                                              const int32_t *__restrict__ seg_row,
                                              const int32_t *__restrict__ cols,
                                              const T *__restrict__ vals,
                                              const T *__restrict__ x, T *__restrict__ y,
                                              int64_t nseg, int remap) {
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t g = (blk * kWG + threadIdx.x) / LPR;
    const int t = threadIdx.x % LPR;
    const bool live = g < nseg;
    int32_t b = 0, e = 0;
    if (live) {
        b = seg_ptr[g];
        e = seg_ptr[g + 1];
    }
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    int32_t k = b + t;
    for (; k + 3 * LPR < e; k += 4 * LPR) {
        const int32_t c0 = ldnt(cols + k), c1 = ldnt(cols + k + LPR);
        const int32_t c2 = ldnt(cols + k + 2 * LPR), c3 = ldnt(cols + k + 3 * LPR);
        const T v0 = ldnt(vals + k), v1 = ldnt(vals + k + LPR);
        const T v2 = ldnt(vals + k + 2 * LPR), v3 = ldnt(vals + k + 3 * LPR);
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
        a2 += v2 * x[c2];
        a3 += v3 * x[c3];
    }
    for (; k < e; k += LPR) a0 += ldnt(vals + k) * x[ldnt(cols + k)];
    const T acc = group_sum<LPR>((a0 + a1) + (a2 + a3));
    if (live && t == 0) {
        if (ROWS) {
            const int32_t r = seg_row[g];
            if (r < 0)
                atomic_add(y + (int64_t)(~r), acc);
            else
                y[r] = ACC ? y[r] + acc : acc;
        } else {
            y[g] = ACC ? y[g] + acc : acc;
        }
    }
}

// ---- blocked SELL: dense B x B blocks, one lane per block row -------------------------------
// The SELL design applied to block rows; one column index per block (the per-entry indices of a
// block follow a periodic linear model, Section V-D), B accumulators per lane in registers.
// Value (ri, ci) of block j of the block row held by `lane` sits at
// B*B*slice_ptr[s] + 64*(B*B*j + B*ri + ci) + lane.
template <typename T, int B, bool ROWS>
__global__ __launch_bounds__(kWG) void k_bsell(const int64_t *__restrict__ slice_ptr,
                                               const int32_t *__restrict__ bcols,
                                               const T *__restrict__ vals,
                                               const int32_t *__restrict__ brows,
                                               const T *__restrict__ x, T *__restrict__ y,
                                               int64_t nslices, int64_t nbrows_part, int remap) {
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t s = blk * (kWG / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= nslices) return;
    const int64_t b = slice_ptr[s];
    const int w = (int)((slice_ptr[s + 1] - b) >> 6);
    const int32_t *c = bcols + b + lane;
    const T *v = vals + b * (B * B) + lane;
    T acc[B];
#pragma unroll
    for (int ri = 0; ri < B; ++ri) acc[ri] = T(0);
    for (int j = 0; j < w; ++j) {
        const int64_t xc = (int64_t)ldnt(c + j * 64) * B;
        T av[B * B];
#pragma unroll
        for (int q = 0; q < B * B; ++q) av[q] = ldnt(v + ((int64_t)j * (B * B) + q) * 64);
        T xv[B];
#pragma unroll
        for (int ci = 0; ci < B; ++ci) xv[ci] = x[xc + ci];
#pragma unroll
        for (int ri = 0; ri < B; ++ri)
#pragma unroll
            for (int ci = 0; ci < B; ++ci) acc[ri] += av[ri * B + ci] * xv[ci];
    }
    const int64_t r = s * 64 + lane;
    if (r < nbrows_part) {
        const int64_t br = ROWS ? (int64_t)brows[r] : r;
#pragma unroll
        for (int ri = 0; ri < B; ++ri) y[br * B + ri] = acc[ri];
    }
}

// ---- heavy rows, column stripes: x tile in LDS ----------------------------------------------
// ROW_DIV (rows longer than a threshold) then COL_DIV (stripes of `tile` columns).  A workgroup
// copies its stripe of x into LDS with coalesced loads, then walks the (row, stripe) segments:
// LPS lanes per segment gather from LDS with 16-bit local columns, WARP_TOTAL_RED over the
// group, GMEM_ATOM_RED into y (zeroed by k_zero_rows).  x is read once per row group instead of
// once per non-zero cache line.
template <typename T, int LPS>
__global__ __launch_bounds__(512) void k_stripe(const int32_t *__restrict__ seg_ptr,
                                                const uint16_t *__restrict__ lcol,
                                                const T *__restrict__ vals,
                                                const int32_t *__restrict__ hrows,
                                                const T *__restrict__ x, T *__restrict__ y,
                                                int nh, int tile, int64_t ncols, int rows_per_y) {
    extern __shared__ __align__(16) unsigned char smem[];
    T *xs = reinterpret_cast<T *>(smem);
    const int s = blockIdx.x;
    const int64_t c0 = (int64_t)s * tile;
    const int w = (int)((ncols - c0) < (int64_t)tile ? (ncols - c0) : (int64_t)tile);
    for (int i = threadIdx.x; i < w; i += blockDim.x) xs[i] = x[c0 + i];
    __syncthreads();
    const int ngroups = blockDim.x / LPS;
    const int g = threadIdx.x / LPS, t = threadIdx.x % LPS;
    const int32_t *sp = seg_ptr + (int64_t)s * nh;
    const int hbeg = blockIdx.y * rows_per_y;
    const int hend = (hbeg + rows_per_y < nh) ? hbeg + rows_per_y : nh;
    for (int h0 = hbeg; h0 < hend; h0 += ngroups) {   // same trip count for every lane of the group
        const int h = h0 + g;
        int32_t b = 0, e = 0;
        if (h < hend) {
            b = sp[h];
            e = sp[h + 1];
        }
        T a0 = T(0), a1 = T(0);
        int32_t k = b + t;
        for (; k + LPS < e; k += 2 * LPS) {
            const uint16_t c0l = ldnt(lcol + k), c1l = ldnt(lcol + k + LPS);
            const T v0 = ldnt(vals + k), v1 = ldnt(vals + k + LPS);
            a0 += v0 * xs[c0l];
            a1 += v1 * xs[c1l];
        }
        for (; k < e; k += LPS) a0 += ldnt(vals + k) * xs[ldnt(lcol + k)];
        const T acc = group_sum<LPS>(a0 + a1);
        if (t == 0 && e > b) atomic_add(y + hrows[h], acc);
    }
}

// -------------------------------------------------------------------------------------------
template <typename T>
int launch_typed(const Part &p, int64_t nrows, int64_t ncols, const T *x, T *y, hipStream_t st) {
    auto blocks = [](int64_t items, int64_t per) { return (unsigned)((items + per - 1) / per); };
    switch (p.kind) {
    case K_ZERO: {
        if (p.nrows == 0) return 0;
        k_zero_rows<T><<<blocks(p.nrows, kWG), kWG, 0, st>>>((const int32_t *)p.p0, p.nrows, y);
        break;
    }
    case K_DIA: {
        if (nrows == 0) return 0;
        auto *offs = (const int32_t *)p.p0;
        auto *vals = (const T *)p.p1;
        if (p.accumulate)
            k_dia<T, true><<<blocks(nrows, kWG), kWG, 0, st>>>(offs, p.ndiag, vals, p.ld, x, y, nrows, ncols);
        else
            k_dia<T, false><<<blocks(nrows, kWG), kWG, 0, st>>>(offs, p.ndiag, vals, p.ld, x, y, nrows, ncols);
        break;
    }
    case K_SELL: {
        if (p.units == 0) return 0;
        const unsigned grid = blocks(p.units, kWG / kWave);
#define SELL_GO(R, A)                                                                              \
    k_sell<T, R, A><<<grid, kWG, 0, st>>>((const int64_t *)p.p0, (const int32_t *)p.p1,           \
                                           (const T *)p.p2, (const int32_t *)p.p3, x, y, p.units, \
                                           p.nrows, p.remap)
        if (p.has_rows) { if (p.accumulate) SELL_GO(true, true); else SELL_GO(true, false); }
        else            { if (p.accumulate) SELL_GO(false, true); else SELL_GO(false, false); }
#undef SELL_GO
        break;
    }
    case K_CSRV: {
        if (p.units == 0) return 0;
#define CSRV_GO(L, R, A)                                                                           \
    k_csrv<T, L, R, A><<<blocks(p.units * L, kWG), kWG, 0, st>>>(                                  \
        (const int32_t *)p.p0, (const int32_t *)p.p1, (const int32_t *)p.p2, (const T *)p.p3, x,   \
        y, p.units, p.remap)
#define CSRV_L(L)                                                                                  \
    case L:                                                                                        \
        if (p.has_rows) { if (p.accumulate) CSRV_GO(L, true, true); else CSRV_GO(L, true, false); } \
        else            { if (p.accumulate) CSRV_GO(L, false, true); else CSRV_GO(L, false, false); } \
        break;
        switch (p.lanes) {
            CSRV_L(1) CSRV_L(2) CSRV_L(4) CSRV_L(8) CSRV_L(16) CSRV_L(32) CSRV_L(64)
        default: return (int)hipErrorInvalidValue;
        }
#undef CSRV_L
#undef CSRV_GO
        break;
    }
    case K_BSELL: {
        if (p.units == 0) return 0;
        const unsigned grid = blocks(p.units, kWG / kWave);
#define BSELL_GO(B, R)                                                                             \
    k_bsell<T, B, R><<<grid, kWG, 0, st>>>((const int64_t *)p.p0, (const int32_t *)p.p1,          \
                                            (const T *)p.p2, (const int32_t *)p.p3, x, y, p.units, \
                                            p.nrows, p.remap)
#define BSELL_B(B)                                                                                 \
    case B:                                                                                        \
        if (p.has_rows) BSELL_GO(B, true); else BSELL_GO(B, false);                                \
        break;
        switch (p.block) {
            BSELL_B(2) BSELL_B(3) BSELL_B(4)
        default: return (int)hipErrorInvalidValue;
        }
#undef BSELL_B
#undef BSELL_GO
        break;
    }
    case K_STRIPE: {
        if (p.units == 0 || p.nrows == 0) return 0;
        const int nh = (int)p.nrows;
        const int threads = 512;
        const int ngroups = threads / p.lanes;
        // enough workgroups to fill 256 CUs: split the heavy rows over blockIdx.y when there
        // are few stripes
        int64_t ysplit = (1024 + p.units - 1) / p.units;
        const int64_t max_split = (nh + ngroups - 1) / ngroups;
        if (ysplit > max_split) ysplit = max_split;
        if (ysplit < 1) ysplit = 1;
        const int rows_per_y = (int)((nh + ysplit - 1) / ysplit);
        const dim3 grid((unsigned)p.units, (unsigned)((nh + rows_per_y - 1) / rows_per_y));
        const size_t lds = (size_t)p.tile * sizeof(T);
#define STRIPE_L(L)                                                                                \
    case L:                                                                                        \
        k_stripe<T, L><<<grid, threads, lds, st>>>((const int32_t *)p.p0, (const uint16_t *)p.p1,  \
                                                   (const T *)p.p2, (const int32_t *)p.p3, x, y,   \
                                                   nh, p.tile, ncols, rows_per_y);                 \
        break;
        switch (p.lanes) {
            STRIPE_L(4) STRIPE_L(8) STRIPE_L(16) STRIPE_L(32) STRIPE_L(64)
        default: return (int)hipErrorInvalidValue;
        }
#undef STRIPE_L
        break;
    }
    }
    return (int)hipGetLastError();
}

}  // namespace

int launch_part(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x,
                void *y, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (dtype == SPMV_F64) return launch_typed<double>(p, nrows, ncols, (const double *)x, (double *)y, st);
    return launch_typed<float>(p, nrows, ncols, (const float *)x, (float *)y, st);
}

const char *hip_error_text(int err) { return hipGetErrorString((hipError_t)err); }

}  // namespace spmv
