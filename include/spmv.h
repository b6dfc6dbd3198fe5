/*
 * spmv.h -- C ABI of the MI355X (gfx950) SpMV plan/search library.
 *
 * The library computes y = A*x (paper, Section I) for a sparse matrix A given once in CSR.
 * spmv_plan_create runs the paper's pipeline on the host and the device:
 *   - a census of the sparsity pattern (row-length statistics, diagonals, dense blocks) that
 *     prunes the candidate designs (Section VI-B, "Pruning");
 *   - the converting and mapping operators of Table II (ROW_DIV / COL_DIV, SORT, SORT_SUB, BIN,
 *     *_ROW_BLOCK, *_COL_BLOCK, *_PAD), plus the three strategies the paper lists as missing in
 *     Section VII-F (HYB-like split of heavy rows, diagonal extraction, dense r x c blocks),
 *     which turn the CSR arrays into the device layout of one candidate plan (Sections IV, V-A,
 *     V-B);
 *   - the search (Section VI-A, level two): every candidate plan is run and timed on the device
 *     and the fastest is kept.
 * spmv_run executes the kept plan: one or a few hand-written HIP kernels, each using one of the
 * reduction strategies of the implementing stage (Table II: THREAD_TOTAL_RED, WARP_TOTAL_RED,
 * GMEM_ATOM_RED, ...; Section V-C "Distribution" and "Reduction").
 *
 * Conventions
 *   - Every function returns spmv_status_t; nothing throws, aborts or exits.  On failure
 *     spmv_last_error() (thread-local) holds a message.
 *   - "HOST" pointers are ordinary process memory; "DEVICE" pointers are HIP device memory on
 *     the device that was current when the plan was created.
 *   - Indices are int32; nnz must be < 2^31.  Values are float or double (spmv_dtype_t).
 *   - Empty rows and an empty matrix are legal (y_i = +0).  Within a row the column order is
 *     free and repeated columns are legal (they add).
 *   - x must be finite: padded slots multiply an explicit 0 by an x element.
 */
#ifndef SPMV_MI355_H
#define SPMV_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spmv_plan spmv_plan_t; /* opaque; owned by the library */

typedef enum { SPMV_F32 = 0, SPMV_F64 = 1 } spmv_dtype_t;

typedef enum {
    SPMV_OK = 0,
    SPMV_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad option or plan-spec string */
    SPMV_ERR_BAD_CSR = 2,     /* row_ptr not monotone / wrong ends, column out of range */
    SPMV_ERR_UNSUPPORTED = 3, /* nnz >= 2^31, unknown dtype, forced plan illegal for this matrix */
    SPMV_ERR_ALLOC = 4,       /* host or device allocation failed */
    SPMV_ERR_HIP = 5,         /* a HIP call failed; text in spmv_last_error() */
    SPMV_ERR_INTERNAL = 6
} spmv_status_t;

/* All fields optional; a NULL options pointer, or a zeroed struct, means defaults. */
typedef struct {
    /* Plan-spec string: skip the search and build exactly this plan.  NULL or "" = search.
     * spmv_plan_describe prints the spec of any plan ("spec") in this grammar (operators of Table II):
     *   leaf  = key=value,key=value,...   one design for a set of rows:
     *     dia=0|1, dia_fill=f, drows=1|2|4      well-populated diagonals first, the rest accumulates
     *     heavy=T, tile=W, hd=0|1, piece=P      rows longer than T: column stripes of W with x in LDS,
     *                                           8-bit column differences, lanes of at most P entries
     *     light=csrv|sell|bsell|bin|nnzb|wbm|xs|xnb|xl|coo   design of the remaining rows, with
     *     lpr, chunk, sigma, block, xwin, smax, wg, r, k, w, rb, remap   (its blocking parameters)
     *     jit=0|1                               kernels compiled at run time for this plan
     *   node  = rows(c1:...:cn){spec}...{spec}  ROW_DIV by row length, n+1 classes
     *         | bin2(k){spec}{spec}             BIN: lengths below / from 2^k
     *         | cut(rho:min){spec}              ROW_DIV where the sorted lengths drop by the ratio rho
     *         | cols(k){spec}...{spec}          COL_DIV into k stripes, the later ones accumulate
     * A malformed spec is SPMV_ERR_INVALID_ARG; one the matrix cannot satisfy SPMV_ERR_UNSUPPORTED. */
    const char *force_plan;
    /* Wall-clock cap for the search in milliseconds.  0 = default (8000).  Negative = no timing:
     * the first candidate of the pruned list is taken (a deterministic function of the census). */
    double search_budget_ms;
    int search_repeats; /* timed runs per candidate; 0 = default (5) */
    int host_threads;   /* threads of the host format builder; 0 = all available */
    /* Device allocator pair, e.g. backed by the caller's framework.  NULL = hipMalloc/hipFree. */
    void *(*dev_alloc)(size_t bytes, void *user);
    void (*dev_free)(void *ptr, void *user);
    void *user;
    int verbosity; /* > 0: progress of the search on stderr */
    /* Non-zero: build the format arrays in HOST memory only, touching no device, so that the
     * layout can be inspected (spmv_plan_array_copy) on a machine without a GPU.  Needs
     * force_plan or a negative search_budget_ms (nothing can be timed); spmv_run refuses such a
     * plan with SPMV_ERR_UNSUPPORTED.  dev_alloc / dev_free are ignored. */
    int host_only;
    /* Learned cost model of the search (Section VI-A, level three).  cost_model_path: a corpus of
     * earlier measurements (the lines a search appends to cost_log_path); when it holds enough of
     * them a regression tree is fitted before the search starts, candidates are tried in the order
     * of their predicted time, and those predicted more than three times slower than the best
     * prediction are skipped (the first candidate of the census is always timed).  NULL: the
     * environment variable SPMV_COST_MODEL, else no model.  cost_log_path: every timed candidate is
     * appended to this file (census features, spec, microseconds).  NULL: SPMV_COST_LOG, else none. */
    const char *cost_model_path;
    const char *cost_log_path;
    /* Non-zero (or the environment variable SPMV_SEARCH_COLD=1): candidates whose arrays, x and y would
     * fit the 256 MB memory-side cache are timed one run at a time with 512 MB streamed through the
     * cache before each, i.e. as a run that finds nothing in it.  Zero: candidates are timed back to back
     * on the same buffers, as an iterative solver would run them. */
    int search_cold;
} spmv_options_t;

/*
 * Build a plan for A (Sections IV-VI).  The CSR arrays are HOST memory, borrowed for the
 * duration of the call only; the plan keeps its own device copy in its own layout.
 *   row_ptr : nrows+1 entries, row_ptr[0] == 0, non-decreasing, row_ptr[nrows] == nnz
 *   col_idx : nnz entries, 0 <= c < ncols
 *   values  : nnz entries of `dtype`
 * On success *out is a plan to be released with spmv_plan_destroy; on failure *out is NULL.
 * Synchronises the device (uploads, timed candidate runs on a private stream).
 */
spmv_status_t spmv_plan_create(spmv_plan_t **out, int64_t nrows, int64_t ncols, int64_t nnz,
                               const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                               spmv_dtype_t dtype, const spmv_options_t *opts);

/*
 * y = A*x with the plan's kernels (Section V-C), enqueued on `stream`; returns without
 * synchronising.
 *   x_dev  : DEVICE, ncols elements of the plan's dtype, finite; must not alias y_dev
 *   y_dev  : DEVICE, nrows elements, every element OVERWRITTEN
 *   stream : a hipStream_t (NULL = the default stream)
 * No allocation, no host synchronisation.  A plan's format arrays are immutable.  Plans whose
 * description reports "scratch_bytes" > 0 keep partial sums in a buffer of their own between two
 * of their launches: runs of such a plan must not overlap (same stream, or ordered by events);
 * other plans may run concurrently on different streams as long as their y buffers differ.
 */
spmv_status_t spmv_run(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream);

/*
 * spmv_run for callers that cannot allocate device memory and cannot let the library do so either:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * launches as spmv_run, except that the partial sums and products that pass from one launch of
 * the plan to the next (its "scratch_bytes") live in a static device array of the library,
 * SPMV_STATIC_SCRATCH_BYTES per device, instead of the buffers the plan allocated when it was
 * created.  The array's device address is looked up when a plan is created on the device (at the
 * latest on the first call here); the call itself allocates and frees nothing, on host or device,
 * and does not synchronise.  x_dev, y_dev, stream as for spmv_run.
 * Errors: a plan whose scratch buffers (each rounded up to 256 bytes) do not fit the array ->
 * SPMV_ERR_UNSUPPORTED, nothing is launched; otherwise as spmv_run.
 * Every call on a device shares that device's array, and the array keeps the last call's contents:
 * each plan's launches overwrite, or clear with a kernel, every element they later read, so a
 * call never depends on what an earlier one left there.  Calls that overlap on one device (two
 * streams, two threads) race on the array: order them, or use spmv_run.
 */
#define SPMV_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
spmv_status_t spmv_run_noalloc(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream);

/*
 * Y[:, v] = A * X[:, v] for k right-hand sides with one plan (multi-vector SpMM; the paper's tool
 * produces a kernel that "can be directly called" for any vector, Section III -- this is the same
 * call for several vectors at once).  Vector v of X starts at x_dev + v*ldx elements, vector v of
 * Y at y_dev + v*ldy elements (ldx >= ncols, ldy >= nrows); every element of the k result vectors is
 * overwritten.  Launches of the diagonal, SELL and CSR-segment designs read the matrix once for
 * 8, 4 or 2 vectors at a time; launches that hand partial sums to each other through the plan's
 * scratch run vector by vector on `stream`.  No allocation, no host synchronisation.
 * k = 0 is a no-op; k outside [0, 4096] or a leading dimension that is too small ->
 * SPMV_ERR_INVALID_ARG.
 */
spmv_status_t spmv_run_multi(const spmv_plan_t *plan, const void *x_dev, int64_t ldx, void *y_dev,
                             int64_t ldy, int k, void *stream);

/*
 * Plan files.  The paper's tool leaves its result behind as generated code plus the format arrays
 * it reads, to be used without searching again (Section III "Overview"; artifact description).
 * spmv_plan_save writes the plan -- spec, census, launch list, every format array (copied from the
 * device), search log -- to `path`; spmv_plan_load rebuilds an equivalent plan from such a file
 * without the CSR matrix, the search or the host format construction.  Of `opts` only dev_alloc /
 * dev_free / user and host_only are used (NULL = defaults); a host_only load needs no device.
 * The file is little endian, carries a hash of its payload, and is meant to be read by the library
 * version that wrote it: a file that is truncated, damaged or not a plan file gives
 * SPMV_ERR_INVALID_ARG and *out = NULL.  A plan file is trusted input (its offsets are not
 * re-derived from a matrix): load only files this library wrote.
 */
spmv_status_t spmv_plan_save(const spmv_plan_t *plan, const char *path);
spmv_status_t spmv_plan_load(spmv_plan_t **out, const char *path, const spmv_options_t *opts);

/*
 * Same as spmv_run, but records a HIP event on `stream` before the first and after every launch,
 * waits for the last one (this call SYNCHRONISES the stream) and writes the duration of launch i
 * in milliseconds to launch_ms[i] (spmv_plan_launch_count entries).  For benchmarks and profiles.
 */
spmv_status_t spmv_run_timed(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream,
                             float *launch_ms);

/*
 * Benchmark helper, the same routine the search uses to time a candidate (Section VI-A, level two):
 * two warm-up runs, then `repeats` samples, each a batch of back-to-back spmv_run launches on
 * `stream` bracketed by HIP events; *median_us receives the median time of one run in microseconds.
 * Synchronises the stream.  x_dev / y_dev as for spmv_run.
 */
spmv_status_t spmv_plan_time(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream,
                             int repeats, double *median_us);

/*
 * Duration of each launch of the plan on its own, for roofline records: launch i is issued
 * `repeats` + 1 times back to back on `stream` (the first is a warm-up) between two HIP events, after
 * the launches before it ran, and launch_us[i] (spmv_plan_launch_count entries) receives the mean
 * duration of one of the repeats in microseconds -- without the gaps that an event around every
 * single launch would add.  Synchronises the stream.  Launches that accumulate into y run several
 * times here: y_dev holds no meaningful result afterwards.  1 <= repeats <= 10000.
 */
spmv_status_t spmv_plan_time_launches(const spmv_plan_t *plan, const void *x_dev, void *y_dev, void *stream,
                                      int repeats, float *launch_us);

/* Free the plan's device arrays (through the allocator pair it was created with). NULL is OK. */
spmv_status_t spmv_plan_destroy(spmv_plan_t *plan);

/* ---- introspection (used by the parity tests and the benchmark) ------------------------- */

/*
 * JSON description: the plan-spec string, the same design spelled as a chain of the paper's
 * operators (Table II names), census statistics, per-part sizes and the search log.
 * An entry of "search": "spec", "build_ms", "run_us" (median time; -1: not timed), "pred_us" (the cost
 * model's prediction; -1: no model), "playoff_us" (median in the play-off of the near-ties at the end of
 * the search; -1: did not take part) and "note" ("kept", "forced", or why it was skipped or rejected).
 * Writes at most cap bytes including the terminating NUL; *needed (may be NULL) receives the
 * full size including the NUL.
 */
spmv_status_t spmv_plan_describe(const spmv_plan_t *plan, char *buf, size_t cap, size_t *needed);

/* The plan's device format arrays (Section V-B, "Format Construction"): count, metadata, copy. */
spmv_status_t spmv_plan_array_count(const spmv_plan_t *plan, int *n);
/* *name points into the plan and stays valid until spmv_plan_destroy. */
spmv_status_t spmv_plan_array_info(const spmv_plan_t *plan, int i, const char **name,
                                   int *elem_bytes, int64_t *count);
/* Synchronous device-to-host copy of array i into host_dst (elem_bytes * count bytes). */
spmv_status_t spmv_plan_array_copy(const spmv_plan_t *plan, int i, void *host_dst);

/*
 * Algorithmic bytes of one spmv_run:
 *   *b_plan = sum over the plan's launches of: the format arrays the launch reads, the elements
 *             of x it can touch (at most one per stored entry, at most all of x), the partial
 *             sums it writes to or reads from scratch, and the y elements it writes (twice if it
 *             updates them);
 *   *b_csr  = nnz*(v+4) + 4*(nrows+1) + v*ncols + v*nrows, the same for plain CSR (v = 4 or 8).
 */
spmv_status_t spmv_plan_bytes(const spmv_plan_t *plan, int64_t *b_plan, int64_t *b_csr);

/*
 * The search's cost model, for inspection (Section VI-A, level three): fit the regression tree to the
 * corpus file `corpus_path` (lines appended by searches run with cost_log_path) and predict the run
 * time, in microseconds, of the plan `spec` on the matrix whose census `plan` carries (a host-only plan
 * will do).  *pred_us = -1 when the corpus holds too few usable lines (fewer than 8) to fit anything;
 * *samples (may be NULL) receives the number of lines used.  A spec that does not parse ->
 * SPMV_ERR_INVALID_ARG.  HOST pointers throughout; no device is touched.
 */
spmv_status_t spmv_cost_predict(const spmv_plan_t *plan, const char *corpus_path, const char *spec,
                                double *pred_us, int64_t *samples);

/*
 * Model-driven format compression, for inspection (Section V-D): fit the linear, step and
 * periodic-linear models (each with a few "if" patches) to `count` 4- or 8-byte integers at `data`
 * (HOST) and write the accepted model as text, e.g. "linear(base=0,step=640)", or "" when none
 * reproduces every element, to buf (at most cap bytes including the NUL).  The same routine is applied
 * to every metadata array of a plan ("arrays"[i]."model" in the description); a plan built with jit=1
 * compiles the fitted expressions into its kernels in place of the array loads.
 */
spmv_status_t spmv_fit_array(const void *data, int elem_bytes, int64_t count, char *buf, size_t cap);

/*
 * Run-time kernel generation, compile-only check (Section V-C, "Kernel Builder"): for every launch of
 * the plan that has a specialised kernel, generate its source (the library's device code preceded by
 * the launch's constants and fitted index expressions) and compile it with hipRTC for the current
 * device, or for gfx950 when there is none.  Nothing is loaded or launched, so a host-only plan on a
 * machine without a GPU will do.  *compiled receives the number of launches compiled; failures are
 * listed in log (may be NULL; at most cap bytes including the NUL).  A plan built from a spec with
 * jit=1 on a device compiles, loads and uses these kernels by itself; its description then reports
 * "jit": true per launch, and "jit_note" says why a launch kept its ahead-of-time kernel.
 */
spmv_status_t spmv_plan_jit_check(const spmv_plan_t *plan, int *compiled, char *log, size_t cap);

/* Number of kernel launches spmv_run makes for this plan, and the name of launch i. */
spmv_status_t spmv_plan_launch_count(const spmv_plan_t *plan, int *n);
spmv_status_t spmv_plan_launch_name(const spmv_plan_t *plan, int i, const char **name);

/*
 * Measurement helper: the streaming ceiling of the current device, against which achieved
 * bandwidths are read (SpMV is memory-bound: Section I, Section VII-B).  Allocates `bytes` bytes of
 * DEVICE memory (hipMalloc), reads them with 16-byte non-temporal loads, then copies one half to the
 * other; *read_gbps and *copy_gbps (bytes read + written per second for the copy) receive the best
 * of `repeats` timed launches on `stream`, in GB/s.  Synchronises the stream, frees the buffer.
 * bytes >= 1 MiB (use >= 2 GiB to get past the caches), 1 <= repeats <= 1000.
 */
spmv_status_t spmv_stream_ceiling(size_t bytes, int repeats, void *stream, double *read_gbps,
                                  double *copy_gbps);

/* ---- Matrix Market input ------------------------------------------------------------------ */

/*
 * Read a Matrix Market coordinate file, the input of the paper's tool (Section III "Overview";
 * artifact description), into CSR arrays ready for spmv_plan_create.
 *   path   : HOST, NUL-terminated file name
 *   dtype  : type of the values array to produce; "integer" files are converted, "pattern" files
 *            give the value 1 for every entry
 *   *nrows, *ncols, *nnz : sizes; nnz counts the entries after a symmetric or skew-symmetric file
 *            has been expanded to both triangles
 *   *row_ptr (nrows+1), *col_idx (nnz), *values (nnz of dtype) : HOST arrays allocated by the
 *            library and OWNED BY THE CALLER, to be released with spmv_mm_free.  Rows ascend,
 *            columns ascend inside a row, repeated positions are kept (in file order; they add).
 * Errors: unreadable file, malformed banner / size line / entry -> SPMV_ERR_INVALID_ARG; an entry
 * outside the matrix -> SPMV_ERR_BAD_CSR; dense ("array") files, complex or hermitian matrices,
 * sizes >= 2^31 -> SPMV_ERR_UNSUPPORTED.  On failure the three pointers are NULL.
 */
spmv_status_t spmv_mm_read(const char *path, spmv_dtype_t dtype, int64_t *nrows, int64_t *ncols,
                           int64_t *nnz, int32_t **row_ptr, int32_t **col_idx, void **values);
/* Release the arrays of spmv_mm_read (NULLs are fine). */
spmv_status_t spmv_mm_free(int32_t *row_ptr, int32_t *col_idx, void *values);

/* Message of the last failure on the calling thread ("" if none). */
const char *spmv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPMV_MI355_H */
