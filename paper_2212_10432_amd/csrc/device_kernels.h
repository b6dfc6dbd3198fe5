// Hand-written gfx950 SpMV kernels: the "implementing" stage of the paper (Table II; Section V-C
// "Distribution" reads the block metadata, "Reduction" multiplies and reduces by row).
//
// Device code only.  This file is compiled twice: ahead of time as part of kernels.hip, and at run
// time by hipRTC when a plan asks for kernels specialised to its own constants (Section V-C, the
// Kernel Builder; Section V-D, model-driven compression: an index array that follows a fitted
// model is replaced by arithmetic).  The specialisation points are the SPMV_JIT_* macros: left
// undefined they read the run-time argument or the array; the run-time compile defines them as
// literals or closed-form expressions.
//
// Mapping of the paper's parallelism levels (Section IV-A, CUDA terms) to CDNA4:
//   BMTB (thread block) -> workgroup, BMW (warp, 32 lanes) -> wavefront (64 lanes), BMT -> lane.
//
// Every kernel streams the matrix arrays exactly once with non-temporal loads (they are never
// reused, and must not evict x from the L2) and writes each y element once.  x is gathered through
// the ordinary cached path, or from a copy of a window of x in LDS (heavy stripes, blocked SELL
// with a window, the two-pass part).
#pragma once

#ifdef __HIPCC_RTC__
typedef signed char int8_t;
typedef unsigned char uint8_t;
typedef short int16_t;
typedef unsigned short uint16_t;
typedef int int32_t;
typedef unsigned int uint32_t;
typedef long long int64_t;
typedef unsigned long long uint64_t;
typedef unsigned long long uintptr_t;
#else
#include <hip/hip_runtime.h>
#include <cstdint>
#endif

#include "constants.h"

namespace spmv {
namespace dev {

// ---- specialisation points -----------------------------------------------------------------------
// JIT_<point>(a): the run-time argument `a`, or the literal SPMV_JIT_<point> when the run-time compile
// defines it.  JIT_<array>(p, i): element i of an offset array, or the closed form fitted to it.
#ifdef SPMV_JIT_DIA_LD
#define JIT_DIA_LD(a) (SPMV_JIT_DIA_LD)
#else
#define JIT_DIA_LD(a) (a)
#endif
#ifdef SPMV_JIT_DIA_NROWS
#define JIT_DIA_NROWS(a) (SPMV_JIT_DIA_NROWS)
#else
#define JIT_DIA_NROWS(a) (a)
#endif
#ifdef SPMV_JIT_DIA_NCOLS
#define JIT_DIA_NCOLS(a) (SPMV_JIT_DIA_NCOLS)
#else
#define JIT_DIA_NCOLS(a) (a)
#endif
#ifdef SPMV_JIT_CSRV_NSEG
#define JIT_CSRV_NSEG(a) (SPMV_JIT_CSRV_NSEG)
#else
#define JIT_CSRV_NSEG(a) (a)
#endif
#ifdef SPMV_JIT_CSRV_ULEN
#define JIT_CSRV_ULEN(a) (SPMV_JIT_CSRV_ULEN)
#else
#define JIT_CSRV_ULEN(a) (a)
#endif
#ifdef SPMV_JIT_CSRV_REMAP
#define JIT_CSRV_REMAP(a) (SPMV_JIT_CSRV_REMAP)
#else
#define JIT_CSRV_REMAP(a) (a)
#endif
#ifdef SPMV_JIT_SELL_NSLICES
#define JIT_SELL_NSLICES(a) (SPMV_JIT_SELL_NSLICES)
#else
#define JIT_SELL_NSLICES(a) (a)
#endif
#ifdef SPMV_JIT_SELL_NROWS
#define JIT_SELL_NROWS(a) (SPMV_JIT_SELL_NROWS)
#else
#define JIT_SELL_NROWS(a) (a)
#endif
#ifdef SPMV_JIT_SELL_REMAP
#define JIT_SELL_REMAP(a) (SPMV_JIT_SELL_REMAP)
#else
#define JIT_SELL_REMAP(a) (a)
#endif
#ifdef SPMV_JIT_SELL_UW
#define JIT_SELL_UW(a) (SPMV_JIT_SELL_UW)
#else
#define JIT_SELL_UW(a) (a)
#endif
#ifdef SPMV_JIT_BSELL_NSLICES
#define JIT_BSELL_NSLICES(a) (SPMV_JIT_BSELL_NSLICES)
#else
#define JIT_BSELL_NSLICES(a) (a)
#endif
#ifdef SPMV_JIT_BSELL_NBROWS
#define JIT_BSELL_NBROWS(a) (SPMV_JIT_BSELL_NBROWS)
#else
#define JIT_BSELL_NBROWS(a) (a)
#endif
#ifdef SPMV_JIT_BSELL_REMAP
#define JIT_BSELL_REMAP(a) (SPMV_JIT_BSELL_REMAP)
#else
#define JIT_BSELL_REMAP(a) (a)
#endif
#ifdef SPMV_JIT_HS_NSL
#define JIT_HS_NSL(a) (SPMV_JIT_HS_NSL)
#else
#define JIT_HS_NSL(a) (a)
#endif
#ifdef SPMV_JIT_HS_NH
#define JIT_HS_NH(a) (SPMV_JIT_HS_NH)
#else
#define JIT_HS_NH(a) (a)
#endif
#ifdef SPMV_JIT_HS_TILE
#define JIT_HS_TILE(a) (SPMV_JIT_HS_TILE)
#else
#define JIT_HS_TILE(a) (a)
#endif
#ifdef SPMV_JIT_HS_NCOLS
#define JIT_HS_NCOLS(a) (SPMV_JIT_HS_NCOLS)
#else
#define JIT_HS_NCOLS(a) (a)
#endif
#ifdef SPMV_JIT_HS_NS
#define JIT_HS_NS(a) (SPMV_JIT_HS_NS)
#else
#define JIT_HS_NS(a) (a)
#endif
#ifdef SPMV_JIT_HS_SPW
#define JIT_HS_SPW(a) (SPMV_JIT_HS_SPW)
#else
#define JIT_HS_SPW(a) (a)
#endif
#ifdef SPMV_JIT_RW_NP
#define JIT_RW_NP(a) (SPMV_JIT_RW_NP)
#else
#define JIT_RW_NP(a) (a)
#endif
#ifdef SPMV_JIT_RW_N
#define JIT_RW_N(a) (SPMV_JIT_RW_N)
#else
#define JIT_RW_N(a) (a)
#endif
#ifdef SPMV_JIT_XL_W
#define JIT_XL_W(a) (SPMV_JIT_XL_W)
#else
#define JIT_XL_W(a) (a)
#endif
#ifdef SPMV_JIT_XL_NCOLS
#define JIT_XL_NCOLS(a) (SPMV_JIT_XL_NCOLS)
#else
#define JIT_XL_NCOLS(a) (a)
#endif
#ifdef SPMV_JIT_XLR_RB
#define JIT_XLR_RB(a) (SPMV_JIT_XLR_RB)
#else
#define JIT_XLR_RB(a) (a)
#endif
#ifdef SPMV_JIT_XLR_N
#define JIT_XLR_N(a) (SPMV_JIT_XLR_N)
#else
#define JIT_XLR_N(a) (a)
#endif
#ifdef SPMV_JIT_SEG_PTR
#define JIT_SEG_PTR(p, i) (SPMV_JIT_SEG_PTR(i))
#else
#define JIT_SEG_PTR(p, i) ((p)[i])
#endif
#ifdef SPMV_JIT_SLICE_PTR
#define JIT_SLICE_PTR(p, i) (SPMV_JIT_SLICE_PTR(i))
#else
#define JIT_SLICE_PTR(p, i) ((p)[i])
#endif
#ifdef SPMV_JIT_GPTR
#define JIT_GPTR(p, i) (SPMV_JIT_GPTR(i))
#else
#define JIT_GPTR(p, i) ((p)[i])
#endif
#ifdef SPMV_JIT_DIA_OFFS
#define JIT_DIA_OFF(offsets, d) (spmv::dev::kJitDiaOffs[d])
#else
#define JIT_DIA_OFF(offsets, d) ((offsets).o[d])
#endif


constexpr int kWG = 256;   // workgroup size of the streaming kernels: 4 wavefronts
constexpr int kMaxLds = 160 * 1024;   // LDS of one CDNA4 compute unit

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

// Sum of one lane of a SELL slice: entries at c[64*j], v[64*j], j < w (w is uniform over the
// wavefront).  Four independent loads and gathers are in flight per step; the last 1-3 entries
// are issued together as well instead of one dependent load-gather chain per entry.
// WIDE adds front loops with sixteen and eight entries in flight (long slices of narrow entries).
template <typename T, typename CI, bool WIDE = false>
__device__ __forceinline__ T sell_lane_sum(const CI *__restrict__ c, const T *__restrict__ v, int w,
                                           const T *__restrict__ xsrc) {
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    int j = 0;
    if (WIDE) {
        for (; j + 16 <= w; j += 16) {
            CI cc[16];
            T vv[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                cc[u] = ldnt(c + (j + u) * 64);
                vv[u] = ldnt(v + (j + u) * 64);
            }
#pragma unroll
            for (int u = 0; u < 16; u += 4) {
                a0 += vv[u + 0] * xsrc[cc[u + 0]];
                a1 += vv[u + 1] * xsrc[cc[u + 1]];
                a2 += vv[u + 2] * xsrc[cc[u + 2]];
                a3 += vv[u + 3] * xsrc[cc[u + 3]];
            }
        }
        for (; j + 8 <= w; j += 8) {
            CI cc[8];
            T vv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                cc[u] = ldnt(c + (j + u) * 64);
                vv[u] = ldnt(v + (j + u) * 64);
            }
#pragma unroll
            for (int u = 0; u < 8; u += 4) {
                a0 += vv[u + 0] * xsrc[cc[u + 0]];
                a1 += vv[u + 1] * xsrc[cc[u + 1]];
                a2 += vv[u + 2] * xsrc[cc[u + 2]];
                a3 += vv[u + 3] * xsrc[cc[u + 3]];
            }
        }
    }
    for (; j + 4 <= w; j += 4) {
        const CI c0 = ldnt(c + (j + 0) * 64), c1 = ldnt(c + (j + 1) * 64);
        const CI c2 = ldnt(c + (j + 2) * 64), c3 = ldnt(c + (j + 3) * 64);
        const T v0 = ldnt(v + (j + 0) * 64), v1 = ldnt(v + (j + 1) * 64);
        const T v2 = ldnt(v + (j + 2) * 64), v3 = ldnt(v + (j + 3) * 64);
        a0 += v0 * xsrc[c0];
        a1 += v1 * xsrc[c1];
        a2 += v2 * xsrc[c2];
        a3 += v3 * xsrc[c3];
    }
    switch (w - j) {
    case 3: {
        const CI c0 = ldnt(c + (j + 0) * 64), c1 = ldnt(c + (j + 1) * 64), c2 = ldnt(c + (j + 2) * 64);
        const T v0 = ldnt(v + (j + 0) * 64), v1 = ldnt(v + (j + 1) * 64), v2 = ldnt(v + (j + 2) * 64);
        a0 += v0 * xsrc[c0];
        a1 += v1 * xsrc[c1];
        a2 += v2 * xsrc[c2];
        break;
    }
    case 2: {
        const CI c0 = ldnt(c + (j + 0) * 64), c1 = ldnt(c + (j + 1) * 64);
        const T v0 = ldnt(v + (j + 0) * 64), v1 = ldnt(v + (j + 1) * 64);
        a0 += v0 * xsrc[c0];
        a1 += v1 * xsrc[c1];
        break;
    }
    case 1:
        a0 += ldnt(v + j * 64) * xsrc[ldnt(c + j * 64)];
        break;
    default: break;
    }
    return (a0 + a1) + (a2 + a3);
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
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i >= nrows) return;
    T acc = T(0);
    for (int d = 0; d < ndiag; ++d) {
        const int64_t c = i + offs[d];
        const T v = ldnt(vals + (int64_t)d * ld + i);
        if (c >= 0 && c < ncols) acc += v * x[c];
    }
    y[i] = ACC ? y[i] + acc : acc;
}

// Up to 8 diagonals: the offsets travel as kernel arguments and the loop is unrolled, so all
// 2*ND loads of a lane are issued before the first is used.
struct DiaOffsets {
    int32_t o[8];
};
#ifdef SPMV_JIT_DIA_OFFS
constexpr int32_t kJitDiaOffs[8] = {SPMV_JIT_DIA_OFFS};
#endif
template <typename T, int ND, bool ACC>
__global__ __launch_bounds__(kWG) void k_dia_fixed(DiaOffsets offs, const T *__restrict__ vals,
                                                   int64_t ld, const T *__restrict__ x,
                                                   T *__restrict__ y, int64_t nrows_arg, int64_t ncols_arg) {
    const int64_t nrows = JIT_DIA_NROWS(nrows_arg), ncols = JIT_DIA_NCOLS(ncols_arg);
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i >= nrows) return;
    T v[ND], xv[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) {
        const int64_t c = i + JIT_DIA_OFF(offs, d);
        v[d] = ldnt(vals + (int64_t)d * JIT_DIA_LD(ld) + i);
        xv[d] = (c >= 0 && c < ncols) ? x[c] : T(0);
    }
    T acc = T(0);
#pragma unroll
    for (int d = 0; d < ND; ++d) acc += v[d] * xv[d];
    if (ACC) y[i] += acc;
    else __builtin_nontemporal_store(acc, y + i);
}

// BMT_ROW_BLOCK(RPL): a lane owns RPL consecutive rows, so that the values of a diagonal arrive as
// one RPL-wide vector load per lane and a quarter (half) as many workgroups have to start: at a few
// microseconds per launch the ramp of the grid is a visible part of the run.
template <typename T, int ND, int RPL, bool ACC>
__global__ __launch_bounds__(kWG) void k_dia_rows(DiaOffsets offs, const T *__restrict__ vals,
                                                  int64_t ld, const T *__restrict__ x,
                                                  T *__restrict__ y, int64_t nrows_arg, int64_t ncols_arg) {
    const int64_t nrows = JIT_DIA_NROWS(nrows_arg), ncols = JIT_DIA_NCOLS(ncols_arg);
    typedef T VT __attribute__((ext_vector_type(RPL)));
    const int64_t i0 = ((int64_t)blockIdx.x * kWG + threadIdx.x) * RPL;
    if (i0 >= nrows) return;   // ld is a multiple of 64 >= nrows: the vector loads below stay inside a diagonal
    VT v[ND];
    T xv[ND][RPL];
#pragma unroll
    for (int d = 0; d < ND; ++d) {
        v[d] = ldnt(reinterpret_cast<const VT *>(vals + (int64_t)d * JIT_DIA_LD(ld) + i0));
        const int64_t c0 = i0 + JIT_DIA_OFF(offs, d);
#pragma unroll
        for (int r = 0; r < RPL; ++r) {
            const int64_t c = c0 + r;
            xv[d][r] = (c >= 0 && c < ncols) ? x[c] : T(0);
        }
    }
    VT acc;
#pragma unroll
    for (int r = 0; r < RPL; ++r) {
        T a = T(0);
#pragma unroll
        for (int d = 0; d < ND; ++d) a += v[d][r] * xv[d][r];
        acc[r] = a;
    }
    if (i0 + RPL <= nrows && (reinterpret_cast<uintptr_t>(y + i0) % sizeof(VT)) == 0) {
        VT *dst = reinterpret_cast<VT *>(y + i0);
        if (ACC) acc += *dst;
        __builtin_nontemporal_store(acc, dst);
    } else {
#pragma unroll
        for (int r = 0; r < RPL; ++r)
            if (i0 + r < nrows) y[i0 + r] = ACC ? y[i0 + r] + acc[r] : acc[r];
    }
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
                                              int64_t nslices_arg, int64_t nrows_part_arg, int remap_arg,
                                              int uniform_w_arg) {
    const int64_t nslices = JIT_SELL_NSLICES(nslices_arg), nrows_part = JIT_SELL_NROWS(nrows_part_arg);
    const int remap = JIT_SELL_REMAP(remap_arg), uniform_w = JIT_SELL_UW(uniform_w_arg);
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t s = blk * (kWG / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= nslices) return;
    // every slice equally wide: the offset array follows a linear model and is not read (Section V-D)
    const int64_t b = uniform_w >= 0 ? s * 64 * (int64_t)uniform_w : JIT_SLICE_PTR(slice_ptr, s);
    const int w = uniform_w >= 0 ? uniform_w : (int)((JIT_SLICE_PTR(slice_ptr, s + 1) - b) >> 6);
    const T acc = sell_lane_sum<T, int32_t>(cols + b + lane, vals + b + lane, w, x);
    const int64_t r = s * 64 + lane;
    if (r < nrows_part) {
        const int64_t row = ROWS ? (int64_t)rows[r] : r;
        y[row] = ACC ? y[row] + acc : acc;
    }
}

// ---- XCD-striped SELL -----------------------------------------------------------------------
// COL_DIV into K = 8*P column stripes, stripe s being worked on by XCD s mod 8 only (workgroup
// ids are dealt round-robin to the 8 XCDs, so workgroup b serves XCD b & 7).  The piece of x a
// stripe touches is ncols/K elements; sized to fit the 4 MB L2 of one XCD, the gathers of random
// columns hit that L2 instead of each pulling a 128-byte line across the fabric.  Inside a stripe
// the rows that have entries there are sorted by that count in windows (SORT_SUB) and stored as
// SELL slices (BMW_ROW_BLOCK(64) + BMT_ROW_BLOCK(1) + BMW_PAD + THREAD_TOTAL_RED).  A lane's sum is
// one of the partial sums of its row; lane l of unit u stores it to scratch[64*u + l] (one
// contiguous 512-byte store per wavefront: scattered 8-byte stores cost a 64-byte write each) and
// k_reduce_rows gathers the partial sums of every row.  The units (slices) of XCD k are
// contiguous: [xbase[k], xbase[k+1]), phase by phase, so all XCDs move from their first stripe to
// their second together.
template <typename T>
__global__ __launch_bounds__(kWG) void k_xs(const int64_t *__restrict__ unit_ptr,
                                            const int32_t *__restrict__ cols,
                                            const T *__restrict__ vals,
                                            const int64_t *__restrict__ xbase,
                                            const T *__restrict__ x, T *__restrict__ partial) {
    const int k = blockIdx.x & 7;
    const int64_t u = xbase[k] + (int64_t)(blockIdx.x >> 3) * (kWG / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (u >= xbase[k + 1]) return;
    const int64_t b = unit_ptr[u];
    const int w = (int)((unit_ptr[u + 1] - b) >> 6);
    const T acc = sell_lane_sum<T, int32_t>(cols + b + lane, vals + b + lane, w, x);
    partial[u * 64 + lane] = acc;   // lanes without a row hold only padding and store 0
}

// y[rows[i]] (+)= sum of the partial sums of row i: scratch[pslot[q]], pptr[i] <= q < pptr[i+1].
// With remap on, an XCD reduces a contiguous range of rows, so a scratch line (16 partial sums of
// neighbouring rows of one window) is fetched into one L2 only.
template <typename T, bool ROWS, bool ACC>
__global__ __launch_bounds__(kWG) void k_reduce_rows(const int32_t *__restrict__ pptr,
                                                     const int32_t *__restrict__ pslot,
                                                     const T *__restrict__ partial,
                                                     const int32_t *__restrict__ rows,
                                                     T *__restrict__ y, int64_t n, int remap) {
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t i = blk * kWG + threadIdx.x;
    if (i >= n) return;
    const int32_t b = pptr[i], e = pptr[i + 1];
    T a0 = T(0), a1 = T(0);
    int32_t q = b;
    for (; q + 1 < e; q += 2) {
        const int32_t s0 = ldnt(pslot + q), s1 = ldnt(pslot + q + 1);
        a0 += partial[s0];
        a1 += partial[s1];
    }
    if (q < e) a0 += partial[ldnt(pslot + q)];
    const int64_t r = ROWS ? (int64_t)rows[i] : i;
    y[r] = ACC ? y[r] + (a0 + a1) : (a0 + a1);
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
                                              int64_t nseg_arg, int remap_arg, int uniform_len_arg) {
    const int64_t nseg = JIT_CSRV_NSEG(nseg_arg);
    const int remap = JIT_CSRV_REMAP(remap_arg), uniform_len = JIT_CSRV_ULEN(uniform_len_arg);
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t g = (blk * kWG + threadIdx.x) / LPR;
    const int t = threadIdx.x % LPR;
    const bool live = g < nseg;
    int32_t b = 0, e = 0;
    if (live) {
        if (uniform_len >= 0) {   // every segment equally long: the offsets follow a linear model
            b = (int32_t)g * uniform_len;
            e = b + uniform_len;
        } else {
            b = (int32_t)JIT_SEG_PTR(seg_ptr, g);
            e = (int32_t)JIT_SEG_PTR(seg_ptr, g + 1);
        }
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
    // the lane's last 1-3 entries are loaded together, not one dependent chain after the other
    const int left = k < e ? (e - k + LPR - 1) / LPR : 0;
    if (left == 3) {
        const int32_t c0 = ldnt(cols + k), c1 = ldnt(cols + k + LPR), c2 = ldnt(cols + k + 2 * LPR);
        const T v0 = ldnt(vals + k), v1 = ldnt(vals + k + LPR), v2 = ldnt(vals + k + 2 * LPR);
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
        a2 += v2 * x[c2];
    } else if (left == 2) {
        const int32_t c0 = ldnt(cols + k), c1 = ldnt(cols + k + LPR);
        const T v0 = ldnt(vals + k), v1 = ldnt(vals + k + LPR);
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
    } else if (left == 1) {
        a0 += ldnt(vals + k) * x[ldnt(cols + k)];
    }
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

// ---- CSR segments, one workgroup per segment ------------------------------------------------------
// BMTB_ROW_BLOCK(1) + BMT_COL_BLOCK(256 lanes) + WARP_TOTAL_RED inside each wavefront + SHMEM_TOTAL_RED:
// the whole workgroup reduces into one row through shared memory.  Same arrays as k_csrv.
template <typename T, bool ROWS, bool ACC>
__global__ __launch_bounds__(kWG) void k_csr_wg_row(const int32_t *__restrict__ seg_ptr,
                                                    const int32_t *__restrict__ seg_row,
                                                    const int32_t *__restrict__ cols,
                                                    const T *__restrict__ vals,
                                                    const T *__restrict__ x, T *__restrict__ y,
                                                    int remap, int uniform_len) {
    __shared__ T red[kWG / kWave];
    const int64_t g = logical_block(blockIdx.x, gridDim.x, remap);
    int32_t b, e;
    if (uniform_len >= 0) {
        b = (int32_t)g * uniform_len;
        e = b + uniform_len;
    } else {
        b = seg_ptr[g];
        e = seg_ptr[g + 1];
    }
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    int32_t k = b + (int32_t)threadIdx.x;
    for (; k + 3 * kWG < e; k += 4 * kWG) {
        const int32_t c0 = ldnt(cols + k), c1 = ldnt(cols + k + kWG);
        const int32_t c2 = ldnt(cols + k + 2 * kWG), c3 = ldnt(cols + k + 3 * kWG);
        const T v0 = ldnt(vals + k), v1 = ldnt(vals + k + kWG);
        const T v2 = ldnt(vals + k + 2 * kWG), v3 = ldnt(vals + k + 3 * kWG);
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
        a2 += v2 * x[c2];
        a3 += v3 * x[c3];
    }
    for (; k < e; k += kWG) a0 += ldnt(vals + k) * x[ldnt(cols + k)];
    const T wsum = group_sum<kWave>((a0 + a1) + (a2 + a3));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = wsum;
    __syncthreads();
    if (threadIdx.x == 0) {
        T acc = T(0);
#pragma unroll
        for (int w = 0; w < kWG / kWave; ++w) acc += red[w];
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

// ---- COO: one lane per stored entry ---------------------------------------------------------
// BMT_NNZ_BLOCK(1) + GMEM_ATOM_RED: every product is added atomically into a y element zeroed by
// an earlier launch.  The root format the paper starts from (Section I); kept as the fallback that
// needs no structure at all.
template <typename T>
__global__ __launch_bounds__(kWG) void k_coo(const int32_t *__restrict__ rows,
                                             const int32_t *__restrict__ cols,
                                             const T *__restrict__ vals, const T *__restrict__ x,
                                             T *__restrict__ y, int64_t nnz) {
    const int64_t k = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (k < nnz) atomic_add(y + ldnt(rows + k), ldnt(vals + k) * x[ldnt(cols + k)]);
}

// ---- nnz-balanced segmented kernel ----------------------------------------------------------
// BMT_NNZ_BLOCK(R): every lane owns R consecutive non-zeros of the part's CSR stream, whatever
// rows they belong to (perfect balance, no padding except the stream's tail).  A wavefront's tile
// of 64*R entries is stored transposed (entry t of lane l at 64*R*tile + 64*t + l) so that loads
// stay contiguous.  THREAD_BITMAP_RED: bit t of the lane's bitmap marks an entry that starts a
// row; the lane adds its entries up serially and closes a row at each mark.  Rows that lie inside
// one lane are stored directly.  WARP_SEG_RED: the open pieces (the lane's sum before its first
// mark, after its last mark, or everything if it has no mark) are combined by a segmented scan
// over the 64 lanes.  A row that starts in the wavefront and ends in it is stored by the lane that
// sees its end; what enters the wavefront from an earlier tile and what is still open at its end
// is added atomically (GMEM_ATOM_RED) to y elements zeroed by an earlier launch.
// tile_row[i] = number of row starts before tile i = index (into rows[]) of the first row that
// starts in it.
// One tile of the nnz-balanced stream.  ROWS: row r of the stream is y element rows[r]; otherwise
// the stream's rows are consecutive elements of `y` (the scratch slots of a striped part).
// STAGE (only with !ROWS): the sums of the rows that start and end inside the tile are consecutive
// elements of `y`; they are collected in the wavefront's LDS buffer `stage` and written out as
// contiguous runs instead of one scattered 8-byte store each.
template <typename T, int R, typename BM, bool ACC, bool ROWS, bool STAGE>
__device__ __forceinline__ void nnzb_tile(int64_t tile, int lane, const int32_t *__restrict__ cols,
                                          const T *__restrict__ vals, const BM *__restrict__ bits,
                                          const int32_t *__restrict__ tile_row,
                                          const int32_t *__restrict__ rows,
                                          const T *__restrict__ x, T *__restrict__ y, T *stage) {
    const int64_t base = tile * 64 * R + lane;
    int32_t c[R];
    T v[R], xv[R];
#pragma unroll
    for (int t = 0; t < R; ++t) {
        c[t] = ldnt(cols + base + t * 64);
        v[t] = ldnt(vals + base + t * 64);
    }
    const uint32_t bm = (uint32_t)ldnt(bits + tile * 64 + lane);
#pragma unroll
    for (int t = 0; t < R; ++t) xv[t] = x[c[t]];
    // index of the first row starting in this lane: row starts in earlier lanes of the tile
    const int nstart = __popc(bm);
    int pre = nstart;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(pre, o, kWave);
        if (lane >= o) pre += up;
    }
    const int32_t tile_first = tile_row[tile];
    const int32_t first_row = tile_first + (pre - nstart);   // row of the lane's first mark
    int32_t row = first_row;
    // serial pass over the lane's entries
    T acc = T(0), head = T(0);
    bool seen = false;
#pragma unroll
    for (int t = 0; t < R; ++t) {
        if ((bm >> t) & 1u) {
            if (seen) {
                if (STAGE) {
                    stage[row - tile_first] = acc;   // a row inside this lane
                } else {
                    const int64_t r = ROWS ? (int64_t)rows[row] : (int64_t)row;
                    y[r] = ACC ? y[r] + acc : acc;
                }
                ++row;
            } else {
                head = acc;           // belongs to a row that started earlier
                seen = true;
            }
            acc = T(0);
        }
        acc += v[t] * xv[t];
    }
    // now: seen ? (head = sum before the first mark, acc = sum after the last mark) : (acc = sum of
    // the whole lane, which lies inside one open row)
    // segmented scan: carry entering lane k = seen_{k-1} ? tail_{k-1} : carry_{k-1} + all_{k-1}
    T val = acc;
    int flag = seen ? 1 : 0;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const T uv = __shfl_up(val, o, kWave);
        const int uf = __shfl_up(flag, o, kWave);
        if (lane >= o) {
            if (!flag) val += uv;
            flag |= uf;
        }
    }
    // val/flag are inclusive; the carry entering this lane is the inclusive result of lane - 1
    T carry = __shfl_up(val, 1, kWave);
    int started = __shfl_up(flag, 1, kWave);   // a row start exists in an earlier lane of the tile
    if (lane == 0) {
        carry = T(0);
        started = 0;
    }
    if (seen) {
        // close the row that ends at this lane's first mark (unless nothing precedes the mark)
        const bool empty = (lane == 0) && (bm & 1u);
        if (!empty) {
            const T total = carry + head;
            const int64_t r = ROWS ? (int64_t)rows[first_row - 1] : (int64_t)(first_row - 1);
            if (started) {
                if (STAGE) stage[first_row - 1 - tile_first] = total;
                else y[r] = ACC ? y[r] + total : total;
            } else {
                atomic_add(y + r, total);
            }
        }
    }
    if (lane == 63) {
        // what is still open at the end of the tile: the row of the last mark at or before it
        const int32_t last_row = tile_row[tile + 1] - 1;
        const int64_t r = ROWS ? (int64_t)rows[last_row] : (int64_t)last_row;
        atomic_add(y + r, val);
    }
    if (STAGE) {
        // rows tile_first .. tile_row[tile+1]-2 started and ended in this tile; each was staged once
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        const int ndone = tile_row[tile + 1] - 1 - tile_first;
        for (int j = lane; j < ndone; j += kWave) y[(int64_t)tile_first + j] = stage[j];
    }
}

// ---- one entry per lane, one row-start bitmap per wavefront step --------------------------------
// BMW_NNZ_BLOCK(64*kWbmSteps) + BMT_NNZ_BLOCK(1) + WARP_BITMAP_RED: the part's entries form one stream
// in row order, stored as it is; a wavefront owns kWbmSteps consecutive groups of 64 entries (a tile)
// and in every step each lane multiplies one entry.  mask[tile*kWbmSteps + t] has bit l set when entry
// l of that step starts a row: the wavefront's 64 products are summed by row with a segmented scan
// steered by that one 64-bit word (the paper's 32-bit warp bitmap, widened to the 64-lane wavefront).
// The lane at the end of a segment stores the row's sum; what is still open after lane 63 is carried
// into the next step in a register; what enters a tile from the tile before, and what is open at its
// end, is added atomically to y elements zeroed by an earlier launch (GMEM_ATOM_RED).
constexpr int kWbmSteps = kWbmTileSteps;
template <typename T, bool ACC>
__global__ __launch_bounds__(kWG) void k_wbm(const int32_t *__restrict__ cols, const T *__restrict__ vals,
                                             const uint64_t *__restrict__ mask,
                                             const int32_t *__restrict__ tile_row,
                                             const int32_t *__restrict__ rows, const T *__restrict__ x,
                                             T *__restrict__ y, int64_t ntiles) {
    const int64_t tile = (int64_t)blockIdx.x * (kWG / kWave) + (threadIdx.x >> 6);
    if (tile >= ntiles) return;
    const int lane = threadIdx.x & 63;
    const int64_t base = tile * (64 * kWbmSteps) + lane;
    int32_t c[kWbmSteps];
    T p[kWbmSteps];
#pragma unroll
    for (int t = 0; t < kWbmSteps; ++t) {
        c[t] = ldnt(cols + base + t * 64);
        p[t] = ldnt(vals + base + t * 64);
    }
    uint64_t m[kWbmSteps];
#pragma unroll
    for (int t = 0; t < kWbmSteps; ++t) m[t] = mask[tile * kWbmSteps + t];   // uniform over the wavefront
#pragma unroll
    for (int t = 0; t < kWbmSteps; ++t) p[t] *= x[c[t]];
    const int32_t first = tile_row[tile];   // row starts before this tile
    int32_t cnt = 0;                        // row starts seen in this tile so far
    T carry = T(0);                         // sum of the segment still open after the previous step
    const uint64_t upto = lane == 63 ? ~0ull : ((2ull << lane) - 1);   // bits 0 .. lane
#pragma unroll
    for (int t = 0; t < kWbmSteps; ++t) {
        const uint64_t mk = m[t];
        // a row start at lane 0 closes what the previous steps left open
        if ((mk & 1ull) && lane == 0 && (t > 0)) {
            const int32_t k = cnt;   // starts before this step: the open row is number first + k - 1
            const int64_t r = rows[first + k - 1];
            if (k == 0) atomic_add(y + r, carry);
            else y[r] = ACC ? y[r] + carry : carry;
        }
        // head = first lane of this lane's segment: the highest row start at or below the lane, else 0
        const uint64_t below = mk & upto;
        const int head = below ? 63 - __builtin_clzll(below) : 0;
        T val = p[t];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const T up = __shfl_up(val, o, kWave);
            if (lane - o >= head) val += up;
        }
        if (head == 0 && !(mk & 1ull)) val += carry;   // the segment continues the open one
        const bool ends = lane < 63 && ((mk >> (lane + 1)) & 1ull);
        const int32_t k = cnt + (int32_t)__popcll(below);   // row starts at or before this entry, in the tile
        if (ends) {
            const int64_t r = rows[first + k - 1];
            if (k == 0) atomic_add(y + r, val);
            else y[r] = ACC ? y[r] + val : val;
        }
        carry = __shfl(val, 63, kWave);
        cnt += (int32_t)__popcll(mk);
    }
    if (lane == 0) atomic_add(y + rows[first + cnt - 1], carry);   // open at the end of the tile
}

template <typename T, int R, typename BM, bool ACC>
__global__ __launch_bounds__(kWG) void k_nnzb(const int32_t *__restrict__ cols,
                                              const T *__restrict__ vals,
                                              const BM *__restrict__ bits,
                                              const int32_t *__restrict__ tile_row,
                                              const int32_t *__restrict__ rows,
                                              const T *__restrict__ x, T *__restrict__ y,
                                              int64_t ntiles) {
    const int64_t tile = (int64_t)blockIdx.x * (kWG / kWave) + (threadIdx.x >> 6);
    if (tile >= ntiles) return;
    nnzb_tile<T, R, BM, ACC, true, false>(tile, threadIdx.x & 63, cols, vals, bits, tile_row, rows, x, y, nullptr);
}

// ---- XCD-striped nnz-balanced tiles -----------------------------------------------------------
// COL_DIV into K = 8*P stripes as in k_xs (stripe s only on XCD s mod 8, so that the stripe of x
// stays in that XCD's L2), but inside a stripe the (row, stripe) segments simply follow each other
// in row order as one nnz-balanced stream (BMT_NNZ_BLOCK + THREAD_BITMAP_RED + WARP_SEG_RED): no
// sorting, no padding, and the partial sum of segment number q (counted stripe by stripe, in row
// order) lands in scratch[q].  k_reduce_bitmap then finds the partial sums of a row by arithmetic.
// Tiles never straddle stripes; the tiles of XCD k are [xbase[k], xbase[k+1]).
template <typename T, int R, typename BM>
__global__ __launch_bounds__(kWG) void k_xnb(const int32_t *__restrict__ cols,
                                             const T *__restrict__ vals,
                                             const BM *__restrict__ bits,
                                             const int32_t *__restrict__ tile_row,
                                             const int64_t *__restrict__ xbase,
                                             const T *__restrict__ x, T *__restrict__ partial) {
    __shared__ T stage[kWG / kWave][kWave * R];
    const int k = blockIdx.x & 7;
    const int wave = threadIdx.x >> 6;
    const int64_t tile = xbase[k] + (int64_t)(blockIdx.x >> 3) * (kWG / kWave) + wave;
    if (tile >= xbase[k + 1]) return;
    nnzb_tile<T, R, BM, false, false, true>(tile, threadIdx.x & 63, cols, vals, bits, tile_row, nullptr, x,
                                            partial, stage[wave]);
}

// Row reduce of the striped nnz-balanced part.  A workgroup owns kRedRows consecutive rows of the
// part.  In every stripe the segments of those rows are consecutive scratch slots
// [bbase[blk*K + s], bbase[(blk+1)*K + s]); seg_row[q] is the row (within the block) segment q
// belongs to.  The slots are read with contiguous loads and added into one LDS accumulator per row
// (SHMEM_OFFSET_RED: a shared-memory reduction by row offset); then y is written contiguously.
constexpr int kRedRows = kReduceBlockRows;   // the builder cuts the part into blocks of this many rows
template <typename T, bool ROWS, bool ACC>
__global__ __launch_bounds__(kWG) void k_reduce_lds(const uint16_t *__restrict__ seg_row,
                                                    const int32_t *__restrict__ bbase,
                                                    const T *__restrict__ partial,
                                                    const int32_t *__restrict__ rows,
                                                    T *__restrict__ y, int64_t n, int K) {
    // the accumulators are double for both value types: LDS adds of doubles are the faster ones here
    __shared__ double acc[kRedRows];
    for (int t = threadIdx.x; t < kRedRows; t += kWG) acc[t] = 0.0;
    __syncthreads();
    const int64_t blk = blockIdx.x;
    const int32_t *b0 = bbase + blk * K, *b1 = b0 + K;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // every wavefront walks its own stripes (two at a time, so their loads overlap)
    for (int s0 = 2 * wave; s0 < K; s0 += 2 * (kWG / kWave)) {   // K is a multiple of 8
        int32_t q0 = b0[s0] + lane, q1 = b0[s0 + 1] + lane;
        const int32_t e0 = b1[s0], e1 = b1[s0 + 1];
        while (__any(q0 < e0 || q1 < e1)) {
            T v0 = T(0), v1 = T(0);
            uint16_t r0 = 0, r1 = 0;
            const bool a0 = q0 < e0, a1 = q1 < e1;
            if (a0) {
                v0 = ldnt(partial + q0);
                r0 = ldnt(seg_row + q0);
            }
            if (a1) {
                v1 = ldnt(partial + q1);
                r1 = ldnt(seg_row + q1);
            }
            if (a0) atomic_add(&acc[r0], (double)v0);
            if (a1) atomic_add(&acc[r1], (double)v1);
            q0 += kWave;
            q1 += kWave;
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kRedRows; t += kWG) {
        const int64_t i = blk * kRedRows + t;
        if (i < n) {
            const int64_t r = ROWS ? (int64_t)rows[i] : i;
            y[r] = ACC ? y[r] + (T)acc[t] : (T)acc[t];
        }
    }
}

// ---- blocked SELL: dense B x B blocks, one lane per block row -------------------------------
// The SELL design applied to block rows; one column index per block (the per-entry indices of a
// block follow a periodic linear model, Section V-D), B accumulators per lane in registers
// (THREAD_TOTAL_RED).  The B*B values of block j of the block row held by `lane` form a record
// of 64*B*B values starting at B*B*(slice_ptr[s] + 64*j); inside the record the first
// NV*V values of a lane are packed for 16-byte loads (vector p of the lane at V*(64*p + lane)),
// the remaining B*B - NV*V values follow one per lane (at V*NV*64 + 64*r + lane).
template <typename T, int B>
struct BlockLoad {
    static constexpr int BB = B * B;
    static constexpr int V = 16 / (int)sizeof(T);
    static constexpr int NV = BB / V;
    static constexpr int NR = BB % V;
    typedef T VT __attribute__((ext_vector_type(V)));
    // values of one block into av[q], q = B*ri + ci
    static __device__ __forceinline__ void load(const T *rec, int lane, T *av) {
        VT pv[NV];
#pragma unroll
        for (int p = 0; p < NV; ++p) pv[p] = ldnt(reinterpret_cast<const VT *>(rec) + p * 64 + lane);
#pragma unroll
        for (int p = 0; p < NV; ++p)
#pragma unroll
            for (int e = 0; e < V; ++e) av[p * V + e] = pv[p][e];
#pragma unroll
        for (int r = 0; r < NR; ++r) av[NV * V + r] = ldnt(rec + NV * V * 64 + r * 64 + lane);
    }
};

// One slice: the gathers of block j are issued before the loads of block j + 1, so waiting for
// x leaves the next block's stream in flight.  XS = true gathers from the LDS copy of x.
template <typename T, int B, bool XS>
__device__ __forceinline__ void bsell_slice(const int32_t *__restrict__ c, const T *__restrict__ v,
                                            int w, int lane, const T *__restrict__ xsrc,
                                            int64_t xbase, T *acc) {
    constexpr int BB = B * B;
    if (w <= 0) return;
    int64_t xc = (int64_t)ldnt(c) * B - xbase;
    T av[BB];
    BlockLoad<T, B>::load(v, lane, av);
    for (int j = 0; j < w; ++j) {
        T xv[B];
#pragma unroll
        for (int ci = 0; ci < B; ++ci) xv[ci] = xsrc[xc + ci];
        int64_t xcn = xc;
        T an[BB];
#pragma unroll
        for (int q = 0; q < BB; ++q) an[q] = av[q];
        if (j + 1 < w) {   // uniform over the wavefront
            xcn = (int64_t)ldnt(c + (j + 1) * 64) * B - xbase;
            BlockLoad<T, B>::load(v + (int64_t)(j + 1) * 64 * BB, lane, an);
        }
#pragma unroll
        for (int ri = 0; ri < B; ++ri)
#pragma unroll
            for (int ci = 0; ci < B; ++ci) acc[ri] += av[ri * B + ci] * xv[ci];
#pragma unroll
        for (int q = 0; q < BB; ++q) av[q] = an[q];
        xc = xcn;
    }
}

// The same slice for the LDS-window kernel: two value buffers take turns and a buffer is refilled
// with the block two ahead as soon as its block has been multiplied, so one to two blocks are in
// flight.  A block's column is kept as loaded and turned into an LDS offset only when the block is
// used.  No test stands between an issue and a use in the steady state: the compiler counts
// outstanding loads per path, and a skipped issue on one path would turn the next wait into a drain.
template <typename T, int B, typename CT>
__device__ __forceinline__ void bsell_slice2(const CT *__restrict__ c, const T *__restrict__ v,
                                             int w, int lane, const T *__restrict__ xs, int xbase,
                                             T *acc) {
    constexpr int BB = B * B;
    if (w <= 0) return;
    int32_t ca = 0, cb = 0;
    T a[BB], b[BB];
    auto issue = [&](int j, int32_t &craw, T *buf) {
        craw = (int32_t)ldnt(c + j * 64);
        BlockLoad<T, B>::load(v + (int64_t)j * 64 * BB, lane, buf);
    };
    auto use = [&](int32_t craw, const T *buf) {
        const int xc = craw * B - xbase;
        T xv[B];
#pragma unroll
        for (int ci = 0; ci < B; ++ci) xv[ci] = xs[xc + ci];
#pragma unroll
        for (int ri = 0; ri < B; ++ri)
#pragma unroll
            for (int ci = 0; ci < B; ++ci) acc[ri] += buf[ri * B + ci] * xv[ci];
    };
    issue(0, ca, a);
    if (w > 1) issue(1, cb, b);
    int j = 0;
    for (; j + 4 <= w; j += 2) {   // a holds block j, b block j + 1; blocks j + 2 and j + 3 exist
        use(ca, a);
        issue(j + 2, ca, a);
        use(cb, b);
        issue(j + 3, cb, b);
    }
    if (j < w) {   // the last one to three blocks (w is uniform over the wavefront)
        use(ca, a);
        if (j + 2 < w) issue(j + 2, ca, a);
    }
    if (j + 1 < w) use(cb, b);
    if (j + 2 < w) use(ca, a);
}

template <typename T, int B, bool ROWS>
__global__ __launch_bounds__(kWG) void k_bsell(const int64_t *__restrict__ slice_ptr,
                                               const int32_t *__restrict__ bcols,
                                               const T *__restrict__ vals,
                                               const int32_t *__restrict__ brows,
                                               const T *__restrict__ x, T *__restrict__ y,
                                               int64_t nslices_arg, int64_t nbrows_part_arg, int remap_arg) {
    const int64_t nslices = JIT_BSELL_NSLICES(nslices_arg), nbrows_part = JIT_BSELL_NBROWS(nbrows_part_arg);
    const int remap = JIT_BSELL_REMAP(remap_arg);
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t s = blk * (kWG / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= nslices) return;
    const int64_t b = JIT_SLICE_PTR(slice_ptr, s);
    const int w = (int)((JIT_SLICE_PTR(slice_ptr, s + 1) - b) >> 6);
    T acc[B];
#pragma unroll
    for (int ri = 0; ri < B; ++ri) acc[ri] = T(0);
    bsell_slice<T, B, false>(bcols + b + lane, vals + b * (B * B), w, lane, x, 0, acc);
    const int64_t r = s * 64 + lane;
    if (r < nbrows_part) {
        const int64_t br = ROWS ? (int64_t)brows[r] : r;
#pragma unroll
        for (int ri = 0; ri < B; ++ri) y[br * B + ri] = acc[ri];
    }
}

// Blocked SELL with the x window of the workgroup staged in LDS.  A workgroup of 16 wavefronts
// owns 32 consecutive slices (one SORT_SUB window of 2048 block rows when sigma = 2048); the
// columns its blocks touch lie in [win[2g], win[2g] + win[2g+1]), copied once with coalesced
// loads; all gathers then go to LDS and leave the vector-memory path to the matrix stream.
// Wavefront w takes slices w and 31 - w: inside a sorted window that pairs the longest slice with
// the shortest, so the 16 wavefronts finish together.
constexpr int kXwinWaves = 16;
constexpr int kXwinSlices = 2 * kXwinWaves;
// The block columns are stored as 16-bit offsets from the window's first block column (index
// compression: 2 bytes per block instead of 4).
// LOCALY: every block row of the group lies in the group's own range of 64 * 32 block rows (no sort,
// or sort windows that are whole groups).  The results are then collected in LDS, in the space of the
// x window once every wavefront is done with it, and written to y as one contiguous piece: stores
// scattered by the sort permutation, mixed into the stream one slice at a time, cost 14 % of the run.
template <typename T, int B, bool ROWS, bool LOCALY>
__global__ __launch_bounds__(kXwinWaves * kWave) void k_bsell_xwin(
    const int64_t *__restrict__ slice_ptr, const uint16_t *__restrict__ bcols,
    const T *__restrict__ vals, const int32_t *__restrict__ brows, const int32_t *__restrict__ win,
    const T *__restrict__ x, T *__restrict__ y, int64_t nslices_arg, int64_t nbrows_part_arg, int remap_arg) {
    const int64_t nslices = JIT_BSELL_NSLICES(nslices_arg), nbrows_part = JIT_BSELL_NBROWS(nbrows_part_arg);
    const int remap = JIT_BSELL_REMAP(remap_arg);
    extern __shared__ __align__(16) unsigned char smem[];
    T *xs = reinterpret_cast<T *>(smem);
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int lo = win[2 * blk], n = win[2 * blk + 1];
    for (int i = threadIdx.x; i < n; i += kXwinWaves * kWave) xs[i] = x[lo + i];
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    T res[2][B];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int64_t s = blk * kXwinSlices + (half ? kXwinSlices - 1 - wave : wave);
        T acc[B];
#pragma unroll
        for (int ri = 0; ri < B; ++ri) acc[ri] = T(0);
        if (s < nslices) {
            const int64_t b = JIT_SLICE_PTR(slice_ptr, s);
            const int w = (int)((JIT_SLICE_PTR(slice_ptr, s + 1) - b) >> 6);
            bsell_slice2<T, B, uint16_t>(bcols + b + lane, vals + b * (B * B), w, lane, xs, 0, acc);
            const int64_t r = s * 64 + lane;
            if (!LOCALY && r < nbrows_part) {
                const int64_t br = ROWS ? (int64_t)brows[r] : r;
#pragma unroll
                for (int ri = 0; ri < B; ++ri) y[br * B + ri] = acc[ri];
            }
        }
#pragma unroll
        for (int ri = 0; ri < B; ++ri) res[half][ri] = acc[ri];
    }
    if (LOCALY) {
        const int64_t row0 = blk * (kXwinSlices * 64);   // first block row of the group
        __syncthreads();                                  // nobody reads the x window any more
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int64_t s = blk * kXwinSlices + (half ? kXwinSlices - 1 - wave : wave);
            const int64_t r = s * 64 + lane;
            if (s < nslices && r < nbrows_part) {
                const int loc = (int)((ROWS ? (int64_t)brows[r] : r) - row0);
#pragma unroll
                for (int ri = 0; ri < B; ++ri) xs[loc * B + ri] = res[half][ri];
            }
        }
        __syncthreads();
        const int64_t left = nbrows_part - row0;
        const int cnt = (int)(left < kXwinSlices * 64 ? left : kXwinSlices * 64) * B;
        T *yg = y + row0 * B;
        for (int i = threadIdx.x; i < cnt; i += kXwinWaves * kWave) __builtin_nontemporal_store(xs[i], yg + i);
    }
}

// ---- heavy rows, column stripes: x tile in LDS ----------------------------------------------
// ROW_DIV (rows longer than a threshold), then COL_DIV (stripes of `tile` columns): one workgroup
// (BMTB) owns a few consecutive stripes and copies each stripe's piece of x into LDS with coalesced
// loads.  Inside a stripe the heavy rows are sorted by the number of entries they have in it
// (SORT_BMTB) and cut into slices of 64 (BMW_ROW_BLOCK), each padded to its longest row (BMW_PAD):
// a lane owns one (row, stripe) segment, gathers x from LDS through 16-bit local columns and keeps
// its sum in a register (THREAD_TOTAL_RED).  The sums of a workgroup meet in an LDS accumulator per
// heavy row (the shared-memory reduction by row of SHMEM_OFFSET_RED, the "offset" being the lane's
// row id); a row occurs once per stripe, so no two lanes touch an accumulator between barriers
// (PIECES: a segment is cut into several lanes of bounded length, a row may occur in many lanes of a
// stripe and the sums are added with LDS atomics; sunits[s] is then the stripe's first unit).
// The workgroup then writes its nh partial sums to scratch and k_reduce_wide adds them up: global
// atomics (GMEM_ATOM_RED) would be several times slower here, since hundreds of workgroups would
// hit the same few thousand y elements.
// Entry j of lane `lane` of unit u = stripe * nsl + slice sits at unit_ptr[u] + 64*j + lane.
// Lanes per workgroup: 512 when two workgroups (x tile + row accumulators each) fit the LDS of a compute
// unit, else 1024, so that the compute unit still holds sixteen wavefronts (chosen by the builder).
constexpr int kHeavyWG = 512;
constexpr int kHeavyWGBig = 1024;
// Four consecutive units of the same width W <= 4 (4 * 64 * W entries starting at entry p0, lane
// rows starting at lr0): every load is issued before the first product.
// PIECES: several lanes of a stripe may hold pieces of the same heavy row, so the lane sums meet in the
// row's LDS accumulator through an atomic add.
template <typename T, bool PIECES>
__device__ __forceinline__ void heavy_add(T *ys, unsigned lr, T acc) {
    if (PIECES) atomic_add(ys + lr, acc);
    else ys[lr] += acc;
}

template <typename T, int W, bool PIECES>
__device__ __forceinline__ void narrow_quad(const uint16_t *__restrict__ lcol, const T *__restrict__ vals,
                                            const uint16_t *__restrict__ lane_row, int32_t p0, int64_t lr0,
                                            int lane, const T *__restrict__ xs, T *__restrict__ ys) {
    uint16_t c[4 * W], lr[4];
    T v[4 * W];
#pragma unroll
    for (int t = 0; t < 4 * W; ++t) {   // entry j of unit k is row k * W + j of the 4 * W rows of 64
        c[t] = ldnt(lcol + p0 + t * 64 + lane);
        v[t] = ldnt(vals + p0 + t * 64 + lane);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) lr[k] = ldnt(lane_row + lr0 + k * 64 + lane);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        T acc = T(0);
#pragma unroll
        for (int j = 0; j < W; ++j) acc += v[k * W + j] * xs[c[k * W + j]];
        if (lr[k] != 0xFFFFu) heavy_add<T, PIECES>(ys, lr[k], acc);
    }
}

template <typename T, bool PIECES, int WG>
__global__ __launch_bounds__(WG) void k_hsell(const int32_t *__restrict__ unit_ptr,
                                                    const uint16_t *__restrict__ lcol,
                                                    const T *__restrict__ vals,
                                                    const uint16_t *__restrict__ lane_row,
                                                    const int32_t *__restrict__ sunits,
                                                    const T *__restrict__ x, T *__restrict__ partial,
                                                    int nsl_arg, int nh_arg, int tile_arg, int64_t ncols_arg, int ns_arg,
                                                    int stripes_per_wg_arg) {
    const int nsl_all = JIT_HS_NSL(nsl_arg), nh = JIT_HS_NH(nh_arg), tile = JIT_HS_TILE(tile_arg), ns = JIT_HS_NS(ns_arg);
    const int stripes_per_wg = JIT_HS_SPW(stripes_per_wg_arg);
    const int64_t ncols = JIT_HS_NCOLS(ncols_arg);
    extern __shared__ __align__(16) unsigned char smem[];
    T *xs = reinterpret_cast<T *>(smem);
    T *ys = xs + tile;
    for (int i = threadIdx.x; i < nh; i += WG) ys[i] = T(0);
    const int lane = threadIdx.x & 63;
    const int s0 = blockIdx.x * stripes_per_wg;
    const int s1 = (s0 + stripes_per_wg < ns) ? s0 + stripes_per_wg : ns;
    for (int s = s0; s < s1; ++s) {
        __syncthreads();   // the previous stripe's gathers are done (first pass: ys is zeroed)
        const int64_t c0 = (int64_t)s * tile;
        const int w = (int)((ncols - c0) < (int64_t)tile ? (ncols - c0) : (int64_t)tile);
        for (int i = threadIdx.x; i < w; i += WG) xs[i] = x[c0 + i];
        __syncthreads();
        // units of this stripe: nsl_all everywhere, or (PIECES) the stripe's own count, at most 128
        const int64_t u0 = PIECES ? (int64_t)sunits[s] : (int64_t)s * nsl_all;
        const int nsl = PIECES ? sunits[s + 1] - sunits[s] : nsl_all;
        // The stripe's unit offsets live in lane registers (nsl <= 128: lane i holds offsets i and
        // 64 + i), so a unit costs no dependent load of its own.  Units are ordered by decreasing
        // width: the first n_wide are wider than four entries and are walked one by one; the narrow
        // ones after them are taken four at a time when the four widths agree, with all their loads
        // issued together (a narrow unit alone is one dependent round trip for a few bytes).
        const int32_t upa = (lane <= nsl) ? unit_ptr[u0 + lane] : 0;
        const int32_t upb = (64 + lane <= nsl) ? unit_ptr[u0 + 64 + lane] : 0;
        const int32_t uplast = unit_ptr[u0 + nsl];
        auto offset_of = [&](int gq) -> int32_t {   // gq uniform over the wavefront, 0 <= gq <= nsl
            const int32_t va = __shfl(upa, gq & 63, kWave), vb = __shfl(upb, gq & 63, kWave);
            return gq >= 128 ? uplast : (gq >= 64 ? vb : va);
        };
        int n_wide = 0, n_used = 0;
        {
            const int32_t na = __shfl_down(upa, 1, kWave), fb = __shfl(upb, 0, kWave);
            const int32_t wa = ((lane == 63) ? fb : na) - upa;                      // width * 64 of unit lane
            const int32_t nb2 = __shfl_down(upb, 1, kWave);
            const int32_t wb = ((lane == 63) ? uplast : nb2) - upb;                 // unit 64 + lane
            const bool ina = lane < nsl, inb = 64 + lane < nsl;
            n_wide = __popcll(__ballot(ina && wa > 4 * 64)) + __popcll(__ballot(inb && wb > 4 * 64));
            n_used = __popcll(__ballot(ina && wa > 0)) + __popcll(__ballot(inb && wb > 0));
        }
        const int wave = threadIdx.x >> 6;
        for (int g = wave; g < n_wide; g += WG / kWave) {
            const int32_t b = offset_of(g), e = offset_of(g + 1);
            const uint16_t lr = lane_row[(u0 + g) * 64 + lane];
            const T acc = sell_lane_sum<T, uint16_t, true>(lcol + b + lane, vals + b + lane, (e - b) >> 6, xs);
            if (lr != 0xFFFFu) heavy_add<T, PIECES>(ys, lr, acc);
        }
        for (int g0 = n_wide + 4 * wave; g0 < n_used; g0 += 4 * (WG / kWave)) {
            const int32_t p0 = offset_of(g0), p1 = offset_of(g0 + 1);
            const int wq = (p1 - p0) >> 6;                                          // 1 .. 4
            bool quad = g0 + 4 <= n_used;
            int32_t p2 = p1, p3 = p1, p4 = p1;
            if (quad) {
                p2 = offset_of(g0 + 2);
                p3 = offset_of(g0 + 3);
                p4 = offset_of(g0 + 4);
                quad = (p2 - p1) >> 6 == wq && (p3 - p2) >> 6 == wq && (p4 - p3) >> 6 == wq;
            }
            if (quad) {
                switch (wq) {
                case 1: narrow_quad<T, 1, PIECES>(lcol, vals, lane_row, p0, (u0 + g0) * 64, lane, xs, ys); break;
                case 2: narrow_quad<T, 2, PIECES>(lcol, vals, lane_row, p0, (u0 + g0) * 64, lane, xs, ys); break;
                case 3: narrow_quad<T, 3, PIECES>(lcol, vals, lane_row, p0, (u0 + g0) * 64, lane, xs, ys); break;
                default: narrow_quad<T, 4, PIECES>(lcol, vals, lane_row, p0, (u0 + g0) * 64, lane, xs, ys); break;
                }
            } else {
                const int cnt = n_used - g0 < 4 ? n_used - g0 : 4;
                for (int k = 0; k < cnt; ++k) {
                    const int32_t b = offset_of(g0 + k), e = offset_of(g0 + k + 1);
                    const uint16_t lr = lane_row[(u0 + g0 + k) * 64 + lane];
                    const T acc = sell_lane_sum<T, uint16_t, false>(lcol + b + lane, vals + b + lane, (e - b) >> 6, xs);
                    if (lr != 0xFFFFu) heavy_add<T, PIECES>(ys, lr, acc);
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nh; i += WG) __builtin_nontemporal_store(ys[i], partial + (int64_t)blockIdx.x * nh + i);
}

// The same part with 8-bit column differences (index compression): a lane starts at the first
// local column of its segment (upper half of lane_meta) and adds one byte per entry; four entries
// share a 32-bit word.  Bridging entries (difference 255, value 0) and padding (0, 0) multiply an
// in-range x element by zero.
template <typename T, int NW>
__device__ __forceinline__ void hdelta_step(const uint32_t *__restrict__ dw, const T *__restrict__ vv,
                                            int j, uint32_t &c, const T *__restrict__ xs, T &a0, T &a1,
                                            T &a2, T &a3) {
    uint32_t w[NW];
    T v[4 * NW];
#pragma unroll
    for (int q = 0; q < NW; ++q) w[q] = ldnt(dw + ((j >> 2) + q) * 64);
#pragma unroll
    for (int t = 0; t < 4 * NW; ++t) v[t] = ldnt(vv + (j + t) * 64);
#pragma unroll
    for (int q = 0; q < NW; ++q) {
        c += w[q] & 255u;
        a0 += v[4 * q + 0] * xs[c];
        c += (w[q] >> 8) & 255u;
        a1 += v[4 * q + 1] * xs[c];
        c += (w[q] >> 16) & 255u;
        a2 += v[4 * q + 2] * xs[c];
        c += w[q] >> 24;
        a3 += v[4 * q + 3] * xs[c];
    }
}

template <typename T, bool PIECES, int WG>
__global__ __launch_bounds__(WG) void k_hsell_delta(const int32_t *__restrict__ unit_ptr,
                                                          const uint32_t *__restrict__ dcols,
                                                          const T *__restrict__ vals,
                                                          const uint32_t *__restrict__ lane_meta,
                                                          const int32_t *__restrict__ sunits,
                                                          const T *__restrict__ x, T *__restrict__ partial,
                                                          int nsl_arg, int nh_arg, int tile_arg, int64_t ncols_arg, int ns_arg,
                                                          int stripes_per_wg_arg) {
    const int nsl_all = JIT_HS_NSL(nsl_arg), nh = JIT_HS_NH(nh_arg), tile = JIT_HS_TILE(tile_arg), ns = JIT_HS_NS(ns_arg);
    const int stripes_per_wg = JIT_HS_SPW(stripes_per_wg_arg);
    const int64_t ncols = JIT_HS_NCOLS(ncols_arg);
    extern __shared__ __align__(16) unsigned char smem[];
    T *xs = reinterpret_cast<T *>(smem);
    T *ys = xs + tile;
    for (int i = threadIdx.x; i < nh; i += WG) ys[i] = T(0);
    const int lane = threadIdx.x & 63;
    const int s0 = blockIdx.x * stripes_per_wg;
    const int s1 = (s0 + stripes_per_wg < ns) ? s0 + stripes_per_wg : ns;
    for (int s = s0; s < s1; ++s) {
        __syncthreads();   // the previous stripe's gathers are done (first pass: ys is zeroed)
        const int64_t c0 = (int64_t)s * tile;
        const int w = (int)((ncols - c0) < (int64_t)tile ? (ncols - c0) : (int64_t)tile);
        for (int i = threadIdx.x; i < w; i += WG) xs[i] = x[c0 + i];
        __syncthreads();
        const int64_t u0 = PIECES ? (int64_t)sunits[s] : (int64_t)s * nsl_all;
        const int nsl = PIECES ? sunits[s + 1] - sunits[s] : nsl_all;
        for (int g = threadIdx.x >> 6; g < nsl; g += WG / kWave) {
            const int64_t u = u0 + g;
            const int32_t b = unit_ptr[u];
            const int wd = (unit_ptr[u + 1] - b) >> 6;   // a multiple of 4
            if (wd == 0) continue;
            const uint32_t meta = lane_meta[u * 64 + lane];
            uint32_t c = meta >> 16;
            const uint32_t *dw = dcols + (b >> 2) + lane;
            const T *vv = vals + b + lane;
            T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
            int j = 0;
            for (; j + 16 <= wd; j += 16) hdelta_step<T, 4>(dw, vv, j, c, xs, a0, a1, a2, a3);
            for (; j + 8 <= wd; j += 8) hdelta_step<T, 2>(dw, vv, j, c, xs, a0, a1, a2, a3);
            for (; j < wd; j += 4) hdelta_step<T, 1>(dw, vv, j, c, xs, a0, a1, a2, a3);
            const uint32_t lr = meta & 0xFFFFu;
            if (lr != 0xFFFFu) heavy_add<T, PIECES>(ys, lr, (a0 + a1) + (a2 + a3));
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nh; i += WG) __builtin_nontemporal_store(ys[i], partial + (int64_t)blockIdx.x * nh + i);
}

// y[rows[i]] (+)= sum over g < np of partial[g * n + i]: many partials (one per workgroup of the
// heavy kernel), few rows.  16 wavefronts split the partials, LDS combines them.
constexpr int kReduceWaves = 16;
constexpr int kReduceRows = 32;   // rows per workgroup: the two halves of a wavefront take alternate partials
template <typename T, bool ACC>
__global__ __launch_bounds__(kReduceWaves * kWave) void k_reduce_wide(const T *__restrict__ partial,
                                                                      int np_arg, int64_t n_arg,
                                                                      const int32_t *__restrict__ rows,
                                                                      T *__restrict__ y) {
    const int np = JIT_RW_NP(np_arg);
    const int64_t n = JIT_RW_N(n_arg);
    __shared__ T red[kReduceWaves][kWave];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
    const int64_t i = (int64_t)blockIdx.x * kReduceRows + (lane & 31);
    // The launch has few workgroups and lives on latency: a lane issues sixteen loads before it adds
    // the first (partials 2*wave + half + 32*u), which covers 512 partials in a single round trip.
    T acc = T(0);
    if (i < n) {
        for (int g0 = 2 * wave + half; g0 < np; g0 += 32 * 16) {
            T a[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int g = g0 + 32 * u;
                a[u] = g < np ? ldnt(partial + (int64_t)g * n + i) : T(0);
            }
#pragma unroll
            for (int u = 0; u < 16; u += 4) acc += (a[u] + a[u + 1]) + (a[u + 2] + a[u + 3]);
        }
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && half == 0 && i < n) {
        T sum = T(0);
#pragma unroll
        for (int k = 0; k < kReduceWaves; ++k) sum += red[k][lane] + red[k][lane + 32];
        const int64_t r = rows[i];
        y[r] = ACC ? y[r] + sum : sum;
    }
}

// ---- two passes with x windows in LDS ---------------------------------------------------------
// For rows too short and too scattered for any tile of x to be reused from a cache: COL_DIV cuts
// the columns into windows small enough for LDS, and the part's entries are stored window by
// window (inside a window by row block, then by row).  The first launch stages a window of x in
// LDS and writes one product per stored entry to scratch, at the entry's own index; everything it
// touches in memory is streamed.  The second launch owns one block of rows per workgroup, keeps a
// double accumulator per row in LDS and adds the block's products, which it finds through a list
// of 16-entry groups (SHMEM_OFFSET_RED).  Runs of one (window, row block) pair are padded to whole
// groups with (value 0, local column 0, local row 0).
typedef double xl_d2 __attribute__((ext_vector_type(2)));
typedef float xl_f4 __attribute__((ext_vector_type(4)));
typedef unsigned short xl_u2 __attribute__((ext_vector_type(2)));
typedef unsigned short xl_u4 __attribute__((ext_vector_type(4)));
template <typename T> struct XlVec;
template <> struct XlVec<double> { typedef xl_d2 V; typedef xl_u2 I; static constexpr int N = 2; };
template <> struct XlVec<float> { typedef xl_f4 V; typedef xl_u4 I; static constexpr int N = 4; };

constexpr int kXlWG = 1024;
// item i = (window, first entry, end entry); both entry numbers are multiples of 16.  One workgroup
// per item, each staging its window of x: workgroups that walk several items of a window and stage it
// once were measured to be slower (many short workgroups overlap one workgroup's staging with
// another's streaming, and the end of the launch is less ragged).  The items of a window follow each
// other on one XCD (item number mod 8), so all but the first stage from that XCD's L2; issuing the
// first loads of the stream before the staging, or keeping two steps in flight, was measured to
// change nothing.
template <typename T>
__global__ __launch_bounds__(kXlWG) void k_xl_mul(const int32_t *__restrict__ item,
                                                  const T *__restrict__ vals,
                                                  const uint16_t *__restrict__ lcol,
                                                  const T *__restrict__ x, T *__restrict__ prod, int W_arg,
                                                  int64_t ncols_arg) {
    const int W = JIT_XL_W(W_arg);
    const int64_t ncols = JIT_XL_NCOLS(ncols_arg);
    typedef typename XlVec<T>::V V;
    typedef typename XlVec<T>::I I;
    constexpr int N = XlVec<T>::N;
    extern __shared__ __align__(16) unsigned char smem[];
    T *xs = reinterpret_cast<T *>(smem);
    const int s = item[3 * blockIdx.x];
    const int64_t b = item[3 * blockIdx.x + 1], e = item[3 * blockIdx.x + 2];
    if (b >= e) return;   // a filler item (uniform over the workgroup)
    const int64_t c0 = (int64_t)s * W;
    const int w = (int)((ncols - c0) < (int64_t)W ? (ncols - c0) : (int64_t)W);
    for (int i = threadIdx.x; i < w; i += kXlWG) xs[i] = x[c0 + i];
    __syncthreads();
    const V *vv = reinterpret_cast<const V *>(vals + b);
    const I *cc = reinterpret_cast<const I *>(lcol + b);
    V *pp = reinterpret_cast<V *>(prod + b);
    const int64_t nv = (e - b) / N;
    // one 16-byte load of values per lane and step: two workgroups of 16 wavefronts per CU keep
    // enough of them in flight (unrolling this loop was measured to be no faster)
    for (int64_t i = threadIdx.x; i < nv; i += kXlWG) {
        const V v = ldnt(vv + i);
        const I c = ldnt(cc + i);
        V r;
#pragma unroll
        for (int k = 0; k < N; ++k) r[k] = v[k] * xs[c[k]];
        __builtin_nontemporal_store(r, pp + i);
    }
}

// Block blk adds the groups glist[gptr[blk]] .. glist[gptr[blk + 1] - 1].  A lane reads 16 bytes of
// products, so 16 / N lanes share a group and one load instruction of a wavefront covers 64 * N
// entries; a wavefront takes 64 list entries at a time and fetches the next 64 while it adds.
// A group is up to 16 consecutive entries of one run, starting at any multiple of N entries.
// lrow is stored in list order, 16 slots per listed group: lrow[16*p + t] is the local row of entry
// N*(glist[p] >> 3) + t.
//
// HEAVY: the leaf also has a heavy part whose rows this part owns as rows without entries.  Block blk
// then adds, for its heavy rows hptr[blk] .. hptr[blk + 1] - 1 (local row hloc[h]), the np partial
// sums hpartial[g * nh + h] that the heavy launch's workgroups left, so that no launch of its own is
// needed for them (a launch that lives on latency: 8 to 10 us for a few megabytes).  A lane loads two
// of them with every step's products and adds them with those, so their latency costs nothing; what
// the steps do not cover is added at the end.
template <typename T, bool ROWS, bool ACC, bool HEAVY>
__global__ __launch_bounds__(kXlWG) void k_xl_reduce(const int32_t *__restrict__ gptr,
                                                     const int32_t *__restrict__ glist,
                                                     const T *__restrict__ prod,
                                                     const uint16_t *__restrict__ lrow,
                                                     const int32_t *__restrict__ rows,
                                                     T *__restrict__ y, int RB_arg, int64_t n_arg,
                                                     const int32_t *__restrict__ hptr,
                                                     const uint16_t *__restrict__ hloc,
                                                     const T *__restrict__ hpartial, int np, int nh) {
    const int RB = JIT_XLR_RB(RB_arg);
    const int64_t n = JIT_XLR_N(n_arg);
    typedef typename XlVec<T>::V V;
    typedef typename XlVec<T>::I I;
    constexpr int N = XlVec<T>::N, LPG = kXlGroup / N, GPI = kWave / LPG, IT = kWave / GPI;
    extern __shared__ __align__(16) unsigned char smem[];
    double *acc = reinterpret_cast<double *>(smem);
    for (int i = threadIdx.x; i < RB; i += kXlWG) acc[i] = 0.0;
    __syncthreads();
    // Neighbouring blocks run on one XCD (workgroup i is on XCD i mod 8): the runs of blocks b and b + 1
    // of a window are adjacent in memory and share a cache line where they meet, and two workgroups
    // that started together reach it at about the same time (C5: 95 -> 89 us).
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, 1);
    const int32_t g0 = (int32_t)JIT_GPTR(gptr, blk), g1 = (int32_t)JIT_GPTR(gptr, blk + 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane / LPG, l = lane % LPG;
    // partial sum i of the block: workgroup i / nhb of the heavy launch, heavy row h0 + i % nhb;
    // lane t takes the partial sums t, t + 1024, ...: the q-th of them is number hq
    constexpr int HK = 2;
    int h0 = 0, nhb = 0, htot = 0, hq = 0;
    if (HEAVY) {
        h0 = hptr[blk];
        nhb = hptr[blk + 1] - h0;
        htot = nhb * np;
    }
    const V *pv = reinterpret_cast<const V *>(prod);
    const I *pr = reinterpret_cast<const I *>(lrow);
    int32_t base = g0 + wave * kWave;
    int32_t mine = (base + lane < g1) ? ldnt(glist + base + lane) : -1;
    while (base < g1) {   // uniform over the wavefront
        const int32_t nbase = base + (kXlWG / kWave) * kWave;
        const int32_t next = (nbase + lane < g1) ? ldnt(glist + nbase + lane) : -1;
        V v[IT];
        I r[IT];
        bool ok[IT];
        T hv[HK];
        int hl[HK];
        if (HEAVY) {
#pragma unroll
            for (int u = 0; u < HK; ++u) {
                const int i = (hq + u) * kXlWG + (int)threadIdx.x;
                hl[u] = -1;
                if (i < htot) {
                    const int g = i / nhb, j = i - g * nhb;
                    hl[u] = hloc[h0 + j];
                    hv[u] = ldnt(hpartial + (int64_t)g * nh + h0 + j);
                }
            }
            hq += HK;
        }
#pragma unroll
        for (int u = 0; u < IT; ++u) {
            const int32_t gid = __shfl(mine, u * GPI + sub, kWave);
            // a list entry is (first 16-byte vector of the group) * 8 + (vectors in the group - 1): the last
            // group of a run may be short, and the lanes past its end stay out
            ok[u] = gid >= 0 && l <= (gid & 7);
            if (ok[u]) {
                // an ordinary load: the line where two runs meet is wanted again by the neighbouring block on
                // this XCD, and a non-temporal load would not leave it in the L2 (C5: 91 -> 89 us)
                v[u] = pv[(int64_t)(gid >> 3) + l];
                r[u] = ldnt(pr + (int64_t)(base + u * GPI + sub) * LPG + l);   // rows are in list order
            }
        }
#pragma unroll
        for (int u = 0; u < IT; ++u)
            if (ok[u]) {
#pragma unroll
                for (int k = 0; k < N; ++k) atomic_add(&acc[r[u][k]], (double)v[u][k]);
            }
        if (HEAVY) {
#pragma unroll
            for (int u = 0; u < HK; ++u)
                if (hl[u] >= 0) atomic_add(&acc[hl[u]], (double)hv[u]);
        }
        base = nbase;
        mine = next;
    }
    if (HEAVY) {
        for (int i = hq * kXlWG + (int)threadIdx.x; i < htot; i += kXlWG) {
            const int g = i / nhb, j = i - g * nhb;
            atomic_add(&acc[hloc[h0 + j]], (double)ldnt(hpartial + (int64_t)g * nh + h0 + j));
        }
    }
    __syncthreads();
    if (!ROWS && (reinterpret_cast<uintptr_t>(y) & 15) == 0) {
        // the block's rows are consecutive y elements: 16-byte stores (RB is a multiple of 64)
        for (int i = threadIdx.x * N; i < RB; i += kXlWG * N) {
            const int64_t pos = blk * RB + i;
            if (pos + N <= n) {
                V out;
#pragma unroll
                for (int k = 0; k < N; ++k) out[k] = (T)acc[i + k];
                V *dst = reinterpret_cast<V *>(y + pos);
                if (ACC) out += *dst;
                __builtin_nontemporal_store(out, dst);
            } else {
                for (int k = 0; k < N && pos + k < n; ++k) y[pos + k] = ACC ? y[pos + k] + (T)acc[i + k] : (T)acc[i + k];
            }
        }
        return;
    }
    for (int i = threadIdx.x; i < RB; i += kXlWG) {
        const int64_t pos = blk * RB + i;
        if (pos < n) {
            const int64_t row = ROWS ? (int64_t)rows[pos] : pos;
            y[row] = ACC ? y[row] + (T)acc[i] : (T)acc[i];
        }
    }
}

// ---- several right-hand sides at once (SpMM with a few vectors) -------------------------------
// Y[:, v] = A * X[:, v] for K vectors stored one after the other (vector v of X at x + v*ldx, of Y at
// y + v*ldy).  The matrix stream is read once for all K vectors, which is what pays for matrices
// whose single-vector run is bound by launch latency or by the matrix stream.  Same layouts and the
// same lane-to-entry mapping as the single-vector kernels; K accumulators per lane.
template <typename T, int K>
__global__ __launch_bounds__(kWG) void k_dia_multi(DiaOffsets offs, int nd, const T *__restrict__ vals,
                                                   int64_t ld, const T *__restrict__ x, int64_t ldx,
                                                   T *__restrict__ y, int64_t ldy, int64_t nrows,
                                                   int64_t ncols, int acc_flag) {
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i >= nrows) return;
    T acc[K];
#pragma unroll
    for (int k = 0; k < K; ++k) acc[k] = T(0);
#pragma unroll 2
    for (int d = 0; d < nd; ++d) {
        const int64_t c = i + offs.o[d];
        const T v = ldnt(vals + (int64_t)d * ld + i);
        if (c >= 0 && c < ncols) {
#pragma unroll
            for (int k = 0; k < K; ++k) acc[k] += v * x[c + k * ldx];
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        T *dst = y + i + k * ldy;
        *dst = acc_flag ? *dst + acc[k] : acc[k];
    }
}

template <typename T, int K>
__global__ __launch_bounds__(kWG) void k_sell_multi(const int64_t *__restrict__ slice_ptr,
                                                    const int32_t *__restrict__ cols,
                                                    const T *__restrict__ vals,
                                                    const int32_t *__restrict__ rows,
                                                    const T *__restrict__ x, int64_t ldx,
                                                    T *__restrict__ y, int64_t ldy, int64_t nslices,
                                                    int64_t nrows_part, int remap, int uniform_w,
                                                    int acc_flag) {
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t s = blk * (kWG / kWave) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= nslices) return;
    const int64_t b = uniform_w >= 0 ? s * 64 * (int64_t)uniform_w : slice_ptr[s];
    const int w = uniform_w >= 0 ? uniform_w : (int)((slice_ptr[s + 1] - b) >> 6);
    const int32_t *c = cols + b + lane;
    const T *v = vals + b + lane;
    T acc[K];
#pragma unroll
    for (int k = 0; k < K; ++k) acc[k] = T(0);
    int j = 0;
    for (; j + 2 <= w; j += 2) {
        const int32_t c0 = ldnt(c + j * 64), c1 = ldnt(c + (j + 1) * 64);
        const T v0 = ldnt(v + j * 64), v1 = ldnt(v + (j + 1) * 64);
#pragma unroll
        for (int k = 0; k < K; ++k) acc[k] += v0 * x[c0 + k * ldx];
#pragma unroll
        for (int k = 0; k < K; ++k) acc[k] += v1 * x[c1 + k * ldx];
    }
    if (j < w) {
        const int32_t c0 = ldnt(c + j * 64);
        const T v0 = ldnt(v + j * 64);
#pragma unroll
        for (int k = 0; k < K; ++k) acc[k] += v0 * x[c0 + k * ldx];
    }
    const int64_t r = s * 64 + lane;
    if (r < nrows_part) {
        const int64_t row = rows ? (int64_t)rows[r] : r;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            T *dst = y + row + k * ldy;
            *dst = acc_flag ? *dst + acc[k] : acc[k];
        }
    }
}

template <typename T, int LPR, int K>
__global__ __launch_bounds__(kWG) void k_csrv_multi(const int32_t *__restrict__ seg_ptr,
                                                    const int32_t *__restrict__ seg_row,
                                                    const int32_t *__restrict__ cols,
                                                    const T *__restrict__ vals,
                                                    const T *__restrict__ x, int64_t ldx,
                                                    T *__restrict__ y, int64_t ldy, int64_t nseg,
                                                    int remap, int uniform_len, int acc_flag) {
    const int64_t blk = logical_block(blockIdx.x, gridDim.x, remap);
    const int64_t g = (blk * kWG + threadIdx.x) / LPR;
    const int t = threadIdx.x % LPR;
    const bool live = g < nseg;
    int32_t b = 0, e = 0;
    if (live) {
        if (uniform_len >= 0) {
            b = (int32_t)g * uniform_len;
            e = b + uniform_len;
        } else {
            b = seg_ptr[g];
            e = seg_ptr[g + 1];
        }
    }
    T acc[K];
#pragma unroll
    for (int k = 0; k < K; ++k) acc[k] = T(0);
    int32_t q = b + t;
    for (; q + LPR < e; q += 2 * LPR) {
        const int32_t c0 = ldnt(cols + q), c1 = ldnt(cols + q + LPR);
        const T v0 = ldnt(vals + q), v1 = ldnt(vals + q + LPR);
#pragma unroll
        for (int k = 0; k < K; ++k) acc[k] += v0 * x[c0 + k * ldx];
#pragma unroll
        for (int k = 0; k < K; ++k) acc[k] += v1 * x[c1 + k * ldx];
    }
    if (q < e) {
        const int32_t c0 = ldnt(cols + q);
        const T v0 = ldnt(vals + q);
#pragma unroll
        for (int k = 0; k < K; ++k) acc[k] += v0 * x[c0 + k * ldx];
    }
#pragma unroll
    for (int k = 0; k < K; ++k) acc[k] = group_sum<LPR>(acc[k]);
    if (live && t == 0) {
        int64_t row = g;
        bool atomic = false;
        if (seg_row) {
            const int32_t r = seg_row[g];
            atomic = r < 0;
            row = atomic ? (int64_t)(~r) : (int64_t)r;
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            T *dst = y + row + k * ldy;
            if (atomic) atomic_add(dst, acc[k]);
            else *dst = acc_flag ? *dst + acc[k] : acc[k];
        }
    }
}

}  // namespace dev
}  // namespace spmv
