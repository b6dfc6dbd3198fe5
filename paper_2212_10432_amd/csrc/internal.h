// Internal types shared by the host format builder, the kernel launchers, the search and the
// C ABI.  Nothing here is visible to users of include/spmv.h.
#pragma once

#include <atomic>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <memory>
#include <sstream>
#include <string>
#include <thread>
#include <vector>

#include "../../include/spmv.h"
#include "constants.h"

namespace spmv {

// Size of the library's static device scratch array (spmv_run_noalloc).
constexpr size_t kStaticScratchBytes = SPMV_STATIC_SCRATCH_BYTES;

struct Error {
    spmv_status_t code;
    std::string msg;
};
[[noreturn]] inline void fail(spmv_status_t code, const std::string &msg) { throw Error{code, msg}; }

// ---- host-side threading -------------------------------------------------------------------
// parallel_for splits [0, n) into chunks handed out dynamically to `threads` std::threads.
void parallel_for(int64_t n, int64_t chunk, int threads,
                  const std::function<void(int64_t, int64_t, int)> &body);
int default_threads();

// ---- the input matrix ----------------------------------------------------------------------
struct HostCsr {
    int64_t nrows = 0, ncols = 0, nnz = 0;
    const int32_t *row_ptr = nullptr;
    const int32_t *col = nullptr;
    const void *val = nullptr;
    spmv_dtype_t dtype = SPMV_F64;
    size_t vsize() const { return dtype == SPMV_F64 ? 8 : 4; }
    int64_t len(int64_t r) const { return (int64_t)row_ptr[r + 1] - row_ptr[r]; }
};

// Owned CSR storage (used when the builder has to derive a matrix: sorted columns, the
// remainder after diagonal extraction).
struct OwnedCsr {
    std::vector<int32_t> row_ptr, col;
    std::vector<char> val;
    HostCsr view;
};

// ---- census (Section VI-B: the sparsity pattern prunes the candidate designs) --------------
struct Census {
    int64_t nrows = 0, ncols = 0, nnz = 0;
    int64_t min_len = 0, max_len = 0, empty_rows = 0;
    double mean_len = 0, var_len = 0;       // "irregular" when var_len > 100 (Section I)
    // nnz held by rows longer than 2^k, k = 0..20 (tail mass, for the heavy-row threshold)
    int64_t rows_over[21] = {0};
    int64_t nnz_over[21] = {0};
    // diagonals: offsets that are at least half populated, and the nnz they hold
    std::vector<int32_t> diag_offsets;
    int64_t diag_nnz = 0;
    // aligned square blocks b x b, b = 2,3,4: number of non-empty blocks and fill = nnz/(b*b*blocks)
    int64_t blocks[5] = {0};
    double block_fill[5] = {0};
    bool cols_sorted = true;
};
Census take_census(const HostCsr &A, int threads);

// ---- plan specification --------------------------------------------------------------------
enum LightKind { L_CSRV = 0, L_SELL = 1, L_BSELL = 2, L_BIN = 3, L_XS = 4, L_NNZB = 5, L_XNB = 6, L_COO = 7, L_XL = 8, L_WBM = 9 };

// A plan is a tree (the paper's Operator Graph, Section IV-B: a chain of operators that branches at
// every ROW_DIV / COL_DIV, each branch designed on its own).  Inner nodes divide the rows or columns of
// their sub-matrix among their children; a leaf carries one flat design (everything below `node`).
enum NodeKind {
    N_LEAF = 0,
    N_ROWS,   // ROW_DIV by row length: cuts c1 < c2 < ...; child i takes the rows with c_i < length <= c_(i+1)
    N_BIN2,   // BIN: one part per power-of-two length class below 2^cuts[0] (child 0), the rest to child 1
    N_CUT,    // ROW_DIV after SORT: cut where length[i] >= cuts[0] * length[i+1], parts of >= cuts[1] rows
    N_COLS    // COL_DIV into cuts[0] equal column stripes; stripes after the first accumulate into y
};

struct PlanSpec {
    int node = N_LEAF;
    std::vector<int64_t> cuts;
    std::vector<PlanSpec> kids;   // one per class / stripe, or a single design applied to all of them
    int dia = 0;             // extract well-populated diagonals into a DIA part first
    double dia_fill = 0.5;   //   minimum population of a diagonal to be extracted
    int drows = 1;           //   rows per lane of the DIA kernel (1, 2 or 4)
    int64_t heavy = 0;       // ROW_DIV: rows longer than this go to the heavy part (0 = no split)
    int tile = 8192;         //   COL_DIV width of the heavy part (columns per LDS tile of x)
    int hd = 0;              //   1 = the heavy part stores 8-bit column deltas instead of 16-bit columns
    int piece = 0;           //   > 0: a heavy row's entries inside a stripe are cut into pieces of at most this many,
                             //   each piece a lane of its own (0: one lane per row and stripe)
    int light = L_CSRV;      // design of the remaining rows
    int lpr = 0;             // csrv: lanes per row (power of two <= 64; 0 = from the mean length)
    int64_t chunk = 0;       // csrv: rows longer than this are cut into segments (0 = never)
                             // xl: most entries per item of the multiply launch (0 = 32768)
    int sigma = 0;           // sell/bsell: sort window in rows (0 = no sort, -1 = whole part)
    int block = 3;           // bsell: block edge (2, 3 or 4)
    int smax = 16;           // bin: rows up to this length go to the SELL bin
    int wg = 0;              // bin: 1 = the long rows take one workgroup each (SHMEM_TOTAL_RED) instead of one wavefront
    int remap = 0;           // 1 = give each XCD a contiguous range of workgroups
    int r = 8;               // nnzb: consecutive non-zeros per lane (4, 8 or 16)
    int k = 8;               // xs: column stripes (8 or 16: one or two per XCD)
    int xwin = 0;            // bsell: stage the x window of 32 slices in LDS when it fits
    int w = 0;               // xl: columns per LDS x window (0 = 64 KiB worth)
    int rb = 16384;          // xl: rows per block of the reduce launch (their sums live in LDS)
    int jit = 0;             // 1 = compile this plan's kernels at run time with its constants and fitted index models
};
PlanSpec parse_spec(const std::string &s);
std::string print_spec(const PlanSpec &p);
std::string operator_chain(const PlanSpec &p);   // the design in the paper's operator names

// ---- model-driven compression of index arrays (fit.cc; Section V-D) -----------------------------
// value(i) = base + step * (i / period) + inner * (i % period), except at the patched indices.
struct ArrayModel {
    int kind = 0;   // 0 none, 1 linear (period 1), 2 step (inner 0), 3 periodic-linear
    int64_t base = 0, step = 0, period = 1, inner = 0;
    std::vector<std::pair<int64_t, int64_t>> patches;   // (index, value): the "if" branches for outliers
    int64_t at(int64_t i) const;
    std::string text() const;                          // for the plan description
    std::string expr(const std::string &var) const;    // C expression for the run-time kernel compile
};
ArrayModel fit_array(const void *host_data, int elem_bytes, int64_t n);   // exact over every index, or kind 0
bool is_metadata_array(const std::string &name);

// ---- device layout -------------------------------------------------------------------------
struct DevArray {
    std::string name;
    void *ptr = nullptr;
    int elem_bytes = 0;
    int64_t count = 0;
    bool read_per_run = true;    // counts towards the algorithmic bytes of one run
    ArrayModel model;            // closed form of a metadata array, when one fits exactly
};

enum PartKind { K_ZERO = 0, K_DIA, K_SELL, K_CSRV, K_BSELL, K_STRIPE, K_REDUCE_WIDE, K_XS, K_REDUCE_ROWS, K_NNZB, K_XNB, K_ZERO_SCRATCH, K_REDUCE_LDS, K_COO, K_XL_MUL, K_XL_REDUCE, K_WBM, K_LAST = K_WBM };

// One kernel launch of spmv_run.  Pointers refer to entries of Plan::arrays.
struct Part {
    PartKind kind = K_ZERO;
    std::string name;            // e.g. "sell", "csrv16", used as array-name prefix and in describe
    int64_t nrows = 0;           // rows (or block rows) this part owns
    int64_t nnz = 0;             // real non-zeros
    int64_t stored = 0;          // stored entries including padding
    int64_t units = 0;           // slices / segments / stripes: the launch's work items
    bool accumulate = false;     // y += instead of y =
    bool has_rows = false;       // an origin-row array is present (else row = arithmetic)
    int lanes = 1;               // lanes per row / segment
    int block = 1;               // bsell block edge
    int ndiag = 0;
    int32_t dia_offsets[8] = {0};   // host copy of the first offsets (kernel arguments when ndiag <= 8)
    int tile = 0;
    int remap = 0;
    int64_t ld = 0;              // dia leading dimension
    int64_t nslices = 0;         // heavy part: slices of 64 heavy rows per stripe
    int64_t ngroups = 0;         // heavy part: workgroups (= partial-sum rows in scratch)
    int64_t per_group = 0;       // heavy part: stripes per workgroup
    void *scratch = nullptr;     // partial sums written by one launch and read by the next
    void *scratch2 = nullptr;    // two-pass reduce that also sums a heavy part: that part's partial sums
    int uniform_w = -1;          // sell / csrv: width shared by every slice / row (-1: read the offsets)
                                 // bsell with an x window: 1 = a group's block rows lie in its own range
    int delta = 0;               // heavy part: columns stored as 8-bit deltas
    int64_t lds_bytes = 0;       // bsell: size of the LDS x window (0 = gather from memory)
    const void *p0 = nullptr, *p1 = nullptr, *p2 = nullptr, *p3 = nullptr, *p4 = nullptr, *p5 = nullptr;
    int64_t bytes = 0;           // algorithmic bytes of one launch: arrays read + x + scratch + y
    void *jit_fn = nullptr;      // kernel compiled at run time for this launch (a hipFunction_t), else the ahead-of-time one
    std::string jit_kernel, jit_defines;   // what was compiled: instantiation and specialisation constants
};

struct Allocator {
    void *(*alloc)(size_t, void *) = nullptr;
    void (*free)(void *, void *) = nullptr;
    void *user = nullptr;
    bool host_only = false;   // arrays live in host memory; the plan can be inspected, not run
};

struct CandidateLog {
    std::string spec;
    double build_ms = 0, run_us = -1;
    double pred_us = -1;      // the cost model's prediction (-1: no model)
    double playoff_us = -1;   // median of its three times in the play-off of the near-ties (-1: did not take part)
    std::string note;
};

struct Plan {
    spmv_dtype_t dtype = SPMV_F64;
    int64_t nrows = 0, ncols = 0, nnz = 0;
    PlanSpec spec;
    std::vector<DevArray> arrays;    // format arrays (inspectable)
    std::vector<DevArray> scratch;   // partial-sum buffers: written and read back in every run
    std::vector<Part> parts;
    Allocator mem;
    Census census;
    std::vector<CandidateLog> log;
    std::string describe_cache;
    std::string prefix;              // while building: path of the tree node whose arrays are being made
    std::vector<void *> jit_modules; // hipModule_t of the kernels compiled at run time (unloaded with the plan)
    std::string jit_note;            // why nothing was compiled, when a plan asked for it
    ~Plan();
    size_t vsize() const { return dtype == SPMV_F64 ? 8 : 4; }
    int64_t bytes_plan() const;
    int64_t bytes_csr() const;
};

// Host format builder: CSR + spec -> device layout (Sections IV, V-A, V-B).
// Throws Error (SPMV_ERR_UNSUPPORTED when the spec cannot be applied to this matrix).
std::unique_ptr<Plan> build_plan(const HostCsr &A, const Census &cen, const PlanSpec &spec,
                                 const Allocator &mem, int threads);

// Kernel launchers (kernels.hip).  Returns a hipError_t as int.
// scratch_override / scratch2_override, when not NULL, replace the part's own scratch buffers.
int launch_part(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x,
                void *y, void *stream, void *scratch_override = nullptr, void *scratch2_override = nullptr);
// The same launch for k = 2, 4 or 8 right-hand sides stored ldx / ldy elements apart; returns -1 when
// the part has no fused multi-vector kernel (the caller runs the vectors one by one).
int launch_part_multi(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x,
                      int64_t ldx, void *y, int64_t ldy, int k, void *stream);
// Run-time kernel generation (jit.cc, kernels.hip).  jit_describe: instantiation name and #define lines
// of the specialised kernel for one launch (false: this launch keeps its ahead-of-time kernel);
// jit_compile_plan compiles and loads them; launch_jit launches one.
bool jit_describe(const Plan &plan, const Part &p, std::string &kernel, std::string &defines);
void jit_compile_plan(Plan &plan);
bool plan_wants_jit(const PlanSpec &spec);
int launch_jit(const Part &p, spmv_dtype_t dtype, int64_t nrows, int64_t ncols, const void *x, void *y, void *stream, void *scratch,
               void *scratch2);
void jit_release_plan(Plan &plan);
int jit_check_plan(const Plan &plan, std::string &log);
// Once per device, when a plan is created there: raises the dynamic-LDS limit of the kernels that
// need more than 64 KiB and looks up the device address of the library's static scratch array.
int prepare_device();
// Device address of the static scratch array on the current device (kStaticScratchBytes bytes).
int static_scratch(void **ptr);
const char *hip_error_text(int err);
// Streaming ceiling of the current device (read, copy) in GB/s; returns a hipError_t as int.
int stream_ceiling(size_t bytes, int repeats, void *stream, double *read_gbps, double *copy_gbps);

// Search (Section VI): enumerate pruned candidates, time them, keep the fastest.
std::vector<PlanSpec> enumerate_candidates(const Census &cen, spmv_dtype_t dtype);
std::unique_ptr<Plan> search_plan(const HostCsr &A, const Census &cen, const spmv_options_t &opts,
                                  const Allocator &mem, int threads);
// flush, when not NULL: flush_bytes of zero-filled device memory streamed through the caches before every
// timed run (each run is then timed alone).
double time_plan(const Plan &plan, const void *x, void *y, int repeats, void *stream, void *flush = nullptr,
                 size_t flush_bytes = 0);
// Reads `bytes` bytes of the zero-filled buffer `buf` (kernels.hip).  Returns a hipError_t as int.
int flush_read(void *buf, size_t bytes, void *stream);

// ---- learned cost model of the search (cost.cc) -----------------------------------------------
struct CostCensus {   // what a corpus line keeps of a census
    spmv_dtype_t dtype = SPMV_F64;
    int64_t nrows = 0, ncols = 0, nnz = 0, max_len = 0, nnz_over_64 = 0, nnz_over_1024 = 0, rows_over_1024 = 0, diag_nnz = 0;
    double mean_len = 0, var_len = 0, block_fill_3 = 0;
};
CostCensus cost_census(const Census &c, spmv_dtype_t dtype);
std::vector<double> cost_features(const CostCensus &c, const PlanSpec &spec);
std::string cost_line(const CostCensus &c, const std::string &spec, double us);
void cost_append(const std::string &path, const std::vector<std::string> &lines);
class CostModel {
public:
    struct Node {
        int feature = -1, left = -1, right = -1;
        double threshold = 0, value = 0;
    };
    int load(const std::string &path);                              // corpus file -> samples; returns lines used
    void add(const CostCensus &c, const PlanSpec &spec, double us);
    void train();
    bool ready() const { return !trees_.empty(); }
    size_t samples() const { return y_.size(); }
    double predict_us(const CostCensus &c, const PlanSpec &spec) const;   // -1 without a trained model
private:
    int grow(std::vector<Node> &tree, const std::vector<double> &target, std::vector<int> &mark, int node, int count,
             int depth);
    std::vector<std::vector<double>> x_;
    std::vector<double> y_;
    std::vector<std::vector<int>> order_;   // while training: the samples sorted by every feature
    std::vector<std::vector<Node>> trees_;
    double base_ = 0;
    int next_mark_ = 1;
};

std::string describe_json(const Plan &plan);

// Plan files (serialize.cc).  Both throw Error.
void save_plan(const Plan &plan, const char *path);
std::unique_ptr<Plan> load_plan(const char *path, const Allocator &mem);

// Matrix Market coordinate file -> CSR in malloc'ed arrays (mmio.cc).  Throws Error.
struct MmCsr {
    int64_t nrows = 0, ncols = 0, nnz = 0;
    int32_t *row_ptr = nullptr, *col = nullptr;
    void *val = nullptr;
};
void read_matrix_market(const char *path, spmv_dtype_t dtype, MmCsr &out);

}  // namespace spmv
