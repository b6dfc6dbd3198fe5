// Launchers of the hand-written gfx950 SpMV kernels (device_kernels.h), the measurement kernels, the
// per-device set-up and the static scratch array.
#include <hip/hip_runtime.h>

#include <mutex>
#include <sstream>

#include "internal.h"
#include "device_kernels.h"

namespace spmv {
namespace {

using namespace dev;
// Returns -1 when the part has no fused multi-vector kernel for this K (the caller then runs the
// vectors one by one), otherwise a hipError_t as int.
template <typename T>
int launch_multi_typed(const Part &p, int64_t nrows, int64_t ncols, const T *x, int64_t ldx, T *y,
                       int64_t ldy, int K, hipStream_t st) {
    auto blocks = [](int64_t items, int64_t per) { return (unsigned)((items + per - 1) / per); };
    if (K != 2 && K != 4 && K != 8) return -1;
    switch (p.kind) {
    case K_DIA: {
        if (p.ndiag < 1 || p.ndiag > 8) return -1;
        if (nrows == 0) return 0;
        DiaOffsets o;
        for (int d = 0; d < 8; ++d) o.o[d] = d < p.ndiag ? p.dia_offsets[d] : 0;
        const unsigned grid = blocks(nrows, kWG);
#define DIAM(KK) k_dia_multi<T, KK><<<grid, kWG, 0, st>>>(o, p.ndiag, (const T *)p.p1, p.ld, x, ldx, y, ldy, nrows, ncols, (int)p.accumulate)
        if (K == 2) DIAM(2); else if (K == 4) DIAM(4); else DIAM(8);
#undef DIAM
        break;
    }
    case K_SELL: {
        if (p.units == 0) return 0;
        const unsigned grid = blocks(p.units, kWG / kWave);
#define SELLM(KK)                                                                                  \
    k_sell_multi<T, KK><<<grid, kWG, 0, st>>>((const int64_t *)p.p0, (const int32_t *)p.p1, (const T *)p.p2, \
                                              p.has_rows ? (const int32_t *)p.p3 : nullptr, x, ldx, y, ldy, \
                                              p.units, p.nrows, p.remap, p.uniform_w, (int)p.accumulate)
        if (K == 2) SELLM(2); else if (K == 4) SELLM(4); else SELLM(8);
#undef SELLM
        break;
    }
    case K_CSRV: {
        if (p.units == 0) return 0;
        if (p.lanes > kWave) return -1;
#define CSRVM(L, KK)                                                                               \
    k_csrv_multi<T, L, KK><<<blocks(p.units * L, kWG), kWG, 0, st>>>(                              \
        (const int32_t *)p.p0, p.has_rows ? (const int32_t *)p.p1 : nullptr, (const int32_t *)p.p2, \
        (const T *)p.p3, x, ldx, y, ldy, p.units, p.remap, p.uniform_w, (int)p.accumulate)
#define CSRVM_L(L)                                                                                 \
    case L:                                                                                        \
        if (K == 2) CSRVM(L, 2); else if (K == 4) CSRVM(L, 4); else CSRVM(L, 8);                   \
        break;
        switch (p.lanes) {
            CSRVM_L(1) CSRVM_L(2) CSRVM_L(4) CSRVM_L(8) CSRVM_L(16) CSRVM_L(32) CSRVM_L(64)
        default: return (int)hipErrorInvalidValue;
        }
#undef CSRVM_L
#undef CSRVM
        break;
    }
    default: return -1;
    }
    return (int)hipGetLastError();
}

// -------------------------------------------------------------------------------------------
template <typename T>
int launch_typed(const Part &p, int64_t nrows, int64_t ncols, const T *x, T *y, hipStream_t st, void *scratch, void *scratch2) {
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
        const unsigned grid = blocks(nrows, kWG);
        if (p.ndiag >= 1 && p.ndiag <= 8) {
            DiaOffsets o;
            for (int d = 0; d < 8; ++d) o.o[d] = d < p.ndiag ? p.dia_offsets[d] : 0;
#define DIA_GO(N, RPL)                                                                             \
    {                                                                                              \
        const unsigned g = blocks(nrows, (int64_t)kWG * RPL);                                      \
        if (p.accumulate) k_dia_rows<T, N, RPL, true><<<g, kWG, 0, st>>>(o, vals, p.ld, x, y, nrows, ncols); \
        else k_dia_rows<T, N, RPL, false><<<g, kWG, 0, st>>>(o, vals, p.ld, x, y, nrows, ncols);   \
    }
#define DIA_N(N)                                                                                   \
    case N:                                                                                        \
        if (p.lanes == 2) DIA_GO(N, 2)                                                             \
        else if (p.lanes == 4) DIA_GO(N, 4)                                                        \
        else if (p.accumulate) k_dia_fixed<T, N, true><<<grid, kWG, 0, st>>>(o, vals, p.ld, x, y, nrows, ncols); \
        else k_dia_fixed<T, N, false><<<grid, kWG, 0, st>>>(o, vals, p.ld, x, y, nrows, ncols);    \
        break;
            switch (p.ndiag) { DIA_N(1) DIA_N(2) DIA_N(3) DIA_N(4) DIA_N(5) DIA_N(6) DIA_N(7) DIA_N(8) }
#undef DIA_GO
#undef DIA_N
            break;
        }
        if (p.accumulate)
            k_dia<T, true><<<grid, kWG, 0, st>>>(offs, p.ndiag, vals, p.ld, x, y, nrows, ncols);
        else
            k_dia<T, false><<<grid, kWG, 0, st>>>(offs, p.ndiag, vals, p.ld, x, y, nrows, ncols);
        break;
    }
    case K_SELL: {
        if (p.units == 0) return 0;
        const unsigned grid = blocks(p.units, kWG / kWave);
#define SELL_GO(R, A)                                                                              \
    k_sell<T, R, A><<<grid, kWG, 0, st>>>((const int64_t *)p.p0, (const int32_t *)p.p1,           \
                                           (const T *)p.p2, (const int32_t *)p.p3, x, y, p.units, \
                                           p.nrows, p.remap, p.uniform_w)
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
        y, p.units, p.remap, p.uniform_w)
#define CSRV_L(L)                                                                                  \
    case L:                                                                                        \
        if (p.has_rows) { if (p.accumulate) CSRV_GO(L, true, true); else CSRV_GO(L, true, false); } \
        else            { if (p.accumulate) CSRV_GO(L, false, true); else CSRV_GO(L, false, false); } \
        break;
        if (p.lanes == kWG) {   // one workgroup per segment
#define WGROW_GO(R, A)                                                                             \
    k_csr_wg_row<T, R, A><<<(unsigned)p.units, kWG, 0, st>>>(                                      \
        (const int32_t *)p.p0, (const int32_t *)p.p1, (const int32_t *)p.p2, (const T *)p.p3, x, y, \
        p.remap, p.uniform_w)
            if (p.has_rows) { if (p.accumulate) WGROW_GO(true, true); else WGROW_GO(true, false); }
            else            { if (p.accumulate) WGROW_GO(false, true); else WGROW_GO(false, false); }
#undef WGROW_GO
            break;
        }
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
        if (p.lds_bytes > 0) {   // x window in LDS: 32 slices per workgroup of 1024 threads
            const unsigned grid = blocks(p.units, kXwinSlices);
            const int threads = kXwinWaves * kWave;
#define XWIN_GO(B, R, L)                                                                           \
    {                                                                                              \
        k_bsell_xwin<T, B, R, L><<<grid, threads, (size_t)p.lds_bytes, st>>>(                      \
            (const int64_t *)p.p0, (const uint16_t *)p.p1, (const T *)p.p2, (const int32_t *)p.p3, \
            (const int32_t *)p.p4, x, y, p.units, p.nrows, p.remap);                               \
    }
#define XWIN_B(B)                                                                                  \
    case B:                                                                                        \
        if (p.uniform_w == 1) { if (p.has_rows) XWIN_GO(B, true, true) else XWIN_GO(B, false, true) }   \
        else                  { if (p.has_rows) XWIN_GO(B, true, false) else XWIN_GO(B, false, false) } \
        break;
            switch (p.block) {
                XWIN_B(2) XWIN_B(3) XWIN_B(4)
            default: return (int)hipErrorInvalidValue;
            }
#undef XWIN_B
#undef XWIN_GO
            break;
        }
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
        if (p.units == 0 || p.nslices == 0) return 0;
        const size_t lds = ((size_t)p.tile + (size_t)p.nrows) * sizeof(T);
        const int32_t *sunits = (const int32_t *)p.p5;   // units per stripe when the rows are cut into pieces
#define HS_GO(KERNEL, CT, WGL)                                                                     \
    KERNEL<<<(unsigned)p.ngroups, WGL, lds, st>>>(                                                 \
        (const int32_t *)p.p0, (const CT *)p.p1, (const T *)p.p2, (const CT *)p.p4, sunits, x, (T *)scratch, \
        (int)p.nslices, (int)p.nrows, p.tile, ncols, (int)p.units, (int)p.per_group)
#define HS_WG(NAME, PIECES, CT)                                                                    \
    {                                                                                              \
        if (p.lanes == kHeavyWGBig) HS_GO((NAME<T, PIECES, kHeavyWGBig>), CT, kHeavyWGBig);        \
        else HS_GO((NAME<T, PIECES, kHeavyWG>), CT, kHeavyWG);                                     \
    }
        if (p.delta) {
            if (sunits) HS_WG(k_hsell_delta, true, uint32_t) else HS_WG(k_hsell_delta, false, uint32_t)
        } else {
            if (sunits) HS_WG(k_hsell, true, uint16_t) else HS_WG(k_hsell, false, uint16_t)
        }
#undef HS_WG
#undef HS_GO
        break;
    }
    case K_XS: {
        if (p.units == 0) return 0;
        k_xs<T><<<(unsigned)(8 * p.ngroups), kWG, 0, st>>>((const int64_t *)p.p0, (const int32_t *)p.p1,
                                                          (const T *)p.p2, (const int64_t *)p.p4, x,
                                                          (T *)scratch);
        break;
    }
    case K_REDUCE_ROWS: {
        if (p.nrows == 0) return 0;
        const unsigned grid = blocks(p.nrows, kWG);
#define RR_GO(R, A)                                                                               \
    k_reduce_rows<T, R, A><<<grid, kWG, 0, st>>>((const int32_t *)p.p0, (const int32_t *)p.p1,    \
                                                  (const T *)scratch, (const int32_t *)p.p3, y, \
                                                  p.nrows, 1)
        if (p.has_rows) { if (p.accumulate) RR_GO(true, true); else RR_GO(true, false); }
        else            { if (p.accumulate) RR_GO(false, true); else RR_GO(false, false); }
#undef RR_GO
        break;
    }
    case K_NNZB: {
        if (p.units == 0) return 0;
        const unsigned grid = blocks(p.units, kWG / kWave);
#define NNZB_GO(RR, BM)                                                                            \
    if (p.accumulate)                                                                              \
        k_nnzb<T, RR, BM, true><<<grid, kWG, 0, st>>>((const int32_t *)p.p0, (const T *)p.p1,     \
                                                       (const BM *)p.p2, (const int32_t *)p.p3,    \
                                                       (const int32_t *)p.p4, x, y, p.units);      \
    else                                                                                           \
        k_nnzb<T, RR, BM, false><<<grid, kWG, 0, st>>>((const int32_t *)p.p0, (const T *)p.p1,    \
                                                        (const BM *)p.p2, (const int32_t *)p.p3,   \
                                                        (const int32_t *)p.p4, x, y, p.units)
        switch (p.lanes) {
        case 4: NNZB_GO(4, uint8_t); break;
        case 8: NNZB_GO(8, uint8_t); break;
        case 16: NNZB_GO(16, uint16_t); break;
        default: return (int)hipErrorInvalidValue;
        }
#undef NNZB_GO
        break;
    }
    case K_WBM: {
        if (p.units == 0) return 0;
        const unsigned grid = blocks(p.units, kWG / kWave);
        if (p.accumulate)
            k_wbm<T, true><<<grid, kWG, 0, st>>>((const int32_t *)p.p0, (const T *)p.p1, (const uint64_t *)p.p2,
                                                 (const int32_t *)p.p3, (const int32_t *)p.p4, x, y, p.units);
        else
            k_wbm<T, false><<<grid, kWG, 0, st>>>((const int32_t *)p.p0, (const T *)p.p1, (const uint64_t *)p.p2,
                                                  (const int32_t *)p.p3, (const int32_t *)p.p4, x, y, p.units);
        break;
    }
    case K_XNB: {
        if (p.units == 0) return 0;
#define XNB_GO(RR, BM)                                                                             \
    k_xnb<T, RR, BM><<<(unsigned)(8 * p.ngroups), kWG, 0, st>>>(                                   \
        (const int32_t *)p.p0, (const T *)p.p1, (const BM *)p.p2, (const int32_t *)p.p3,           \
        (const int64_t *)p.p4, x, (T *)scratch)
        switch (p.lanes) {
        case 4: XNB_GO(4, uint8_t); break;
        case 8: XNB_GO(8, uint8_t); break;
        case 16: XNB_GO(16, uint16_t); break;
        default: return (int)hipErrorInvalidValue;
        }
#undef XNB_GO
        break;
    }
    case K_ZERO_SCRATCH: {
        if (p.nrows == 0) return 0;
        k_zero_rows<T><<<blocks(p.nrows, kWG), kWG, 0, st>>>((const int32_t *)p.p0, p.nrows, (T *)scratch);
        break;
    }
    case K_REDUCE_LDS: {
        if (p.nrows == 0) return 0;
        const unsigned grid = blocks(p.nrows, kRedRows);
#define RL_GO(Rw, A)                                                                               \
    k_reduce_lds<T, Rw, A><<<grid, kWG, 0, st>>>((const uint16_t *)p.p0, (const int32_t *)p.p1,    \
                                                 (const T *)scratch, (const int32_t *)p.p3, y,   \
                                                 p.nrows, p.lanes)
        if (p.has_rows) { if (p.accumulate) RL_GO(true, true); else RL_GO(true, false); }
        else            { if (p.accumulate) RL_GO(false, true); else RL_GO(false, false); }
#undef RL_GO
        break;
    }
    case K_COO: {
        if (p.units == 0) return 0;
        k_coo<T><<<blocks(p.units, kWG), kWG, 0, st>>>((const int32_t *)p.p0, (const int32_t *)p.p1,
                                                       (const T *)p.p2, x, y, p.units);
        break;
    }
    case K_XL_MUL: {
        if (p.units == 0) return 0;
        const size_t lds = (size_t)p.tile * sizeof(T);
        k_xl_mul<T><<<(unsigned)p.units, kXlWG, lds, st>>>((const int32_t *)p.p0, (const T *)p.p1,
                                                          (const uint16_t *)p.p2, x, (T *)scratch,
                                                          p.tile, ncols);
        break;
    }
    case K_XL_REDUCE: {
        if (p.units == 0) return 0;
        const size_t lds = (size_t)p.tile * sizeof(double);
#define XLR_GO(Rw, A, H)                                                                           \
    {                                                                                              \
        k_xl_reduce<T, Rw, A, H><<<(unsigned)p.units, kXlWG, lds, st>>>(                           \
            (const int32_t *)p.p0, (const int32_t *)p.p1, (const T *)scratch,                    \
            (const uint16_t *)p.p2, (const int32_t *)p.p3, y, p.tile, p.nrows,                     \
            (const int32_t *)p.p4, (const uint16_t *)p.p5, (const T *)scratch2, (int)p.ngroups,    \
            (int)p.nslices);                                                                       \
    }
#define XLR_H(Rw, A)                                                                               \
    {                                                                                              \
        if (p.p4) XLR_GO(Rw, A, true) else XLR_GO(Rw, A, false)                                    \
    }
        if (p.has_rows) { if (p.accumulate) XLR_H(true, true) else XLR_H(true, false) }
        else            { if (p.accumulate) XLR_H(false, true) else XLR_H(false, false) }
#undef XLR_H
#undef XLR_GO
        break;
    }
    case K_REDUCE_WIDE: {
        if (p.nrows == 0) return 0;
        if (p.accumulate)
            k_reduce_wide<T, true><<<blocks(p.nrows, kReduceRows), kReduceWaves * kWave, 0, st>>>(
                (const T *)scratch, (int)p.ngroups, p.nrows, (const int32_t *)p.p3, y);
        else
            k_reduce_wide<T, false><<<blocks(p.nrows, kReduceRows), kReduceWaves * kWave, 0, st>>>(
                (const T *)scratch, (int)p.ngroups, p.nrows, (const int32_t *)p.p3, y);
        break;
    }
    }
    return (int)hipGetLastError();
}

// ---- streaming ceiling of the device (measurement helper) --------------------------------------
typedef float ceil_f4 __attribute__((ext_vector_type(4)));
// one workgroup per 8 x 256 vectors (read) or per 256 vectors (copy): many short workgroups keep
// more requests in flight than a few persistent ones, and that is what reaches the ceiling
__global__ __launch_bounds__(kWG) void k_stream_read(const ceil_f4 *__restrict__ p, int64_t n, float *sink) {
    const int64_t i = (int64_t)blockIdx.x * (kWG * 8) + threadIdx.x;
    ceil_f4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int64_t j = i + u * kWG;
        if (j < n) a += ldnt(p + j);
    }
    if (a[0] + a[1] + a[2] + a[3] == 1.2345e30f) sink[0] = a[0];   // never true for the zero-filled buffer
}
__global__ __launch_bounds__(kWG) void k_stream_copy(const ceil_f4 *__restrict__ src, ceil_f4 *__restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kWG + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(ldnt(src + i), dst + i);
}

}  // namespace

int flush_read(void *buf, size_t bytes, void *stream) {
    const int64_t n16 = (int64_t)(bytes / 16);
    if (n16 == 0) return 0;
    const unsigned grid = (unsigned)((n16 + kWG * 8 - 1) / (kWG * 8));
    k_stream_read<<<grid, kWG, 0, (hipStream_t)stream>>>((const ceil_f4 *)buf, n16, (float *)buf);
    return (int)hipGetLastError();
}

// Reads `bytes` bytes, then copies bytes/2 to the other half of the same buffer; best of `repeats`
// timed launches each.  Returns a hipError_t as int.
int stream_ceiling(size_t bytes, int repeats, void *stream, double *read_gbps, double *copy_gbps) {
    hipStream_t st = (hipStream_t)stream;
    void *buf = nullptr;
    float *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t err = hipMalloc(&buf, bytes);
    if (err == hipSuccess) err = hipMalloc((void **)&sink, sizeof(float));
    if (err == hipSuccess) err = hipMemsetAsync(buf, 0, bytes, st);
    if (err == hipSuccess) err = hipEventCreate(&e0);
    if (err == hipSuccess) err = hipEventCreate(&e1);
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned grid_r = (unsigned)((n16 + kWG * 8 - 1) / (kWG * 8)), grid_c = (unsigned)((n16 / 2 + kWG - 1) / kWG);
    double best_r = 0, best_c = 0;
    for (int it = 0; err == hipSuccess && it < repeats + 1; ++it) {   // the first pass warms up
        float ms = 0;
        (void)hipEventRecord(e0, st);
        k_stream_read<<<grid_r, kWG, 0, st>>>((const ceil_f4 *)buf, n16, sink);
        (void)hipEventRecord(e1, st);
        err = hipEventSynchronize(e1);
        if (err != hipSuccess) break;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (it && ms > 0) best_r = std::max(best_r, (double)n16 * 16.0 / (ms * 1e-3) / 1e9);
        (void)hipEventRecord(e0, st);
        k_stream_copy<<<grid_c, kWG, 0, st>>>((const ceil_f4 *)buf, (ceil_f4 *)buf + n16 / 2, n16 / 2);
        (void)hipEventRecord(e1, st);
        err = hipEventSynchronize(e1);
        if (err != hipSuccess) break;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (it && ms > 0) best_c = std::max(best_c, (double)(n16 / 2) * 32.0 / (ms * 1e-3) / 1e9);   // read + written
    }
    if (err == hipSuccess) err = hipGetLastError();
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (buf) (void)hipFree(buf);
    *read_gbps = best_r;
    *copy_gbps = best_c;
    return (int)err;
}

namespace {

// Kernels that take more than 64 KiB of dynamic LDS need the limit raised once per device; this is
// done when a plan is created, never on the launch path (spmv_run only enqueues kernels).
template <typename T>
hipError_t raise_lds_limits() {
    const void *fns[] = {
        (const void *)k_hsell<T, false, kHeavyWG>, (const void *)k_hsell<T, true, kHeavyWG>,
        (const void *)k_hsell_delta<T, false, kHeavyWG>, (const void *)k_hsell_delta<T, true, kHeavyWG>,
        (const void *)k_hsell<T, false, kHeavyWGBig>, (const void *)k_hsell<T, true, kHeavyWGBig>,
        (const void *)k_hsell_delta<T, false, kHeavyWGBig>, (const void *)k_hsell_delta<T, true, kHeavyWGBig>, (const void *)k_xl_mul<T>,
        (const void *)k_xl_reduce<T, false, false, false>, (const void *)k_xl_reduce<T, false, true, false>,
        (const void *)k_xl_reduce<T, true, false, false>, (const void *)k_xl_reduce<T, true, true, false>,
        (const void *)k_xl_reduce<T, false, false, true>, (const void *)k_xl_reduce<T, false, true, true>,
        (const void *)k_xl_reduce<T, true, false, true>, (const void *)k_xl_reduce<T, true, true, true>,
#define XWIN_ALL(B)                                                                               \
    (const void *)k_bsell_xwin<T, B, false, false>, (const void *)k_bsell_xwin<T, B, false, true>, \
    (const void *)k_bsell_xwin<T, B, true, false>, (const void *)k_bsell_xwin<T, B, true, true>
        XWIN_ALL(2), XWIN_ALL(3), XWIN_ALL(4)
#undef XWIN_ALL
    };
    for (const void *f : fns) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Scratch shared by every spmv_run_noalloc call on a device: a file-scope device array, so that no
// allocation is ever needed for it.  Host code never uses the symbol itself as an address: the
// device address is looked up once per device (each device holds its own copy) and kept.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_dev_mutex;
bool g_dev_ready[kMaxDevices] = {false};
void *g_scratch_ptr[kMaxDevices] = {nullptr};

}  // namespace

int prepare_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (g_dev_ready[dev]) return 0;
    e = raise_lds_limits<double>();
    if (e == hipSuccess) e = raise_lds_limits<float>();
    void *ptr = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    g_scratch_ptr[dev] = ptr;
    g_dev_ready[dev] = true;
    return 0;
}

int static_scratch(void **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    {
        std::lock_guard<std::mutex> lock(g_dev_mutex);
        if (g_dev_ready[dev]) {
            *ptr = g_scratch_ptr[dev];
            return 0;
        }
    }
    const int err = prepare_device();   // first use of this device by the library
    if (err) return err;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    *ptr = g_scratch_ptr[dev];
    return 0;
}

// ---- run-time specialised kernels -----------------------------------------------------------------
// Launch of a run-time compiled kernel: the grid, workgroup, LDS size and argument list of the
// ahead-of-time launch of the same kind (launch_typed above), handed to the module launch call.
template <typename T>
int launch_jit_typed(const Part &p, int64_t nrows, int64_t ncols, const T *x, T *y, hipStream_t st, void *scratch, void *scratch2) {
    auto blocks = [](int64_t items, int64_t per) { return (unsigned)((items + per - 1) / per); };
    hipFunction_t fn = (hipFunction_t)p.jit_fn;
    unsigned grid = 0, block = kWG;
    size_t lds = 0;
    void *args[16];
    int na = 0;
    // argument storage that outlives the switch
    DiaOffsets o;
    const void *q0 = p.p0, *q1 = p.p1, *q2 = p.p2, *q3 = p.p3, *q4 = p.p4, *q5 = p.p5;
    int64_t a64[4];
    int a32[8];
    const T *xx = x;
    T *yy = y;
    void *sc = scratch, *sc2 = scratch2;
    auto P = [&](void *ptr) { args[na++] = ptr; };
    switch (p.kind) {
    case K_DIA: {
        if (nrows == 0) return 0;
        const int rpl = (p.lanes == 2 || p.lanes == 4) ? p.lanes : 1;
        grid = blocks(nrows, (int64_t)kWG * rpl);
        for (int d = 0; d < 8; ++d) o.o[d] = d < p.ndiag ? p.dia_offsets[d] : 0;
        a64[0] = p.ld; a64[1] = nrows; a64[2] = ncols;
        P(&o); P(&q1); P(&a64[0]); P(&xx); P(&yy); P(&a64[1]); P(&a64[2]);
        break;
    }
    case K_CSRV:
        if (p.units == 0) return 0;
        grid = blocks(p.units * p.lanes, kWG);
        a64[0] = p.units; a32[0] = p.remap; a32[1] = p.uniform_w;
        P(&q0); P(&q1); P(&q2); P(&q3); P(&xx); P(&yy); P(&a64[0]); P(&a32[0]); P(&a32[1]);
        break;
    case K_SELL:
        if (p.units == 0) return 0;
        grid = blocks(p.units, kWG / kWave);
        a64[0] = p.units; a64[1] = p.nrows; a32[0] = p.remap; a32[1] = p.uniform_w;
        P(&q0); P(&q1); P(&q2); P(&q3); P(&xx); P(&yy); P(&a64[0]); P(&a64[1]); P(&a32[0]); P(&a32[1]);
        break;
    case K_BSELL:
        if (p.units == 0) return 0;
        a64[0] = p.units; a64[1] = p.nrows; a32[0] = p.remap;
        if (p.lds_bytes > 0) {
            grid = blocks(p.units, kXwinSlices);
            block = kXwinWaves * kWave;
            lds = (size_t)p.lds_bytes;
            P(&q0); P(&q1); P(&q2); P(&q3); P(&q4); P(&xx); P(&yy); P(&a64[0]); P(&a64[1]); P(&a32[0]);
        } else {
            grid = blocks(p.units, kWG / kWave);
            P(&q0); P(&q1); P(&q2); P(&q3); P(&xx); P(&yy); P(&a64[0]); P(&a64[1]); P(&a32[0]);
        }
        break;
    case K_STRIPE:
        if (p.units == 0 || p.nslices == 0) return 0;
        grid = (unsigned)p.ngroups;
        block = p.lanes == kHeavyWGBig ? kHeavyWGBig : kHeavyWG;
        lds = ((size_t)p.tile + (size_t)p.nrows) * sizeof(T);
        a32[0] = (int)p.nslices; a32[1] = (int)p.nrows; a32[2] = p.tile; a64[0] = ncols; a32[3] = (int)p.units; a32[4] = (int)p.per_group;
        P(&q0); P(&q1); P(&q2); P(&q4); P(&q5); P(&xx); P(&sc); P(&a32[0]); P(&a32[1]); P(&a32[2]); P(&a64[0]); P(&a32[3]); P(&a32[4]);
        break;
    case K_REDUCE_WIDE:
        if (p.nrows == 0) return 0;
        grid = blocks(p.nrows, kReduceRows);
        block = kReduceWaves * kWave;
        a32[0] = (int)p.ngroups; a64[0] = p.nrows;
        P(&sc); P(&a32[0]); P(&a64[0]); P(&q3); P(&yy);
        break;
    case K_XL_MUL:
        if (p.units == 0) return 0;
        grid = (unsigned)p.units;
        block = kXlWG;
        lds = (size_t)p.tile * sizeof(T);
        a32[0] = p.tile; a64[0] = ncols;
        P(&q0); P(&q1); P(&q2); P(&xx); P(&sc); P(&a32[0]); P(&a64[0]);
        break;
    case K_XL_REDUCE:
        if (p.units == 0) return 0;
        grid = (unsigned)p.units;
        block = kXlWG;
        lds = (size_t)p.tile * sizeof(double);
        a32[0] = p.tile; a64[0] = p.nrows; a32[1] = (int)p.ngroups; a32[2] = (int)p.nslices;
        P(&q0); P(&q1); P(&sc); P(&q2); P(&q3); P(&yy); P(&a32[0]); P(&a64[0]); P(&q4); P(&q5); P(&sc2); P(&a32[1]); P(&a32[2]);
        break;
    default: return (int)hipErrorInvalidValue;
    }
    return (int)hipModuleLaunchKernel(fn, grid, 1, 1, block, 1, 1, (unsigned)lds, st, args, nullptr);
}

int launch_jit(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x, void *y, void *stream, void *scratch,
               void *scratch2) {
    hipStream_t st = (hipStream_t)stream;
    if (dtype == SPMV_F64) return launch_jit_typed<double>(p, nrows, ncols, (const double *)x, (double *)y, st, scratch, scratch2);
    return launch_jit_typed<float>(p, nrows, ncols, (const float *)x, (float *)y, st, scratch, scratch2);
}

int launch_part(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x,
                void *y, void *stream, void *scratch_override, void *scratch2_override) {
    hipStream_t st = (hipStream_t)stream;
    void *scratch = scratch_override ? scratch_override : p.scratch;
    void *scratch2 = scratch2_override ? scratch2_override : p.scratch2;
    if (p.jit_fn) return launch_jit(p, dtype, nrows, ncols, x, y, stream, scratch, scratch2);
    if (dtype == SPMV_F64) return launch_typed<double>(p, nrows, ncols, (const double *)x, (double *)y, st, scratch, scratch2);
    return launch_typed<float>(p, nrows, ncols, (const float *)x, (float *)y, st, scratch, scratch2);
}

int launch_part_multi(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x,
                      int64_t ldx, void *y, int64_t ldy, int k, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (dtype == SPMV_F64) return launch_multi_typed<double>(p, nrows, ncols, (const double *)x, ldx, (double *)y, ldy, k, st);
    return launch_multi_typed<float>(p, nrows, ncols, (const float *)x, ldx, (float *)y, ldy, k, st);
}

const char *hip_error_text(int err) { return hipGetErrorString((hipError_t)err); }

}  // namespace spmv
