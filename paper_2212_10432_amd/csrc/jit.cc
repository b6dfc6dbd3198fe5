// Run-time kernel generation (Section V-C, "Kernel Builder"; Section V-D, format compression).
// The paper splices kernel fragments into source text and compiles one program per candidate.
// Here the kernel source is the library's own device code (device_kernels.h, embedded as text);
// what is generated per launch is the list of #define lines in front of it: the launch's sizes,
// widths, tile shapes and diagonal offsets as literals, and a closed-form expression for every
// offset array a model was fitted to.  hipRTC compiles that text for the device at hand, the
// instantiation the launch needs is looked up by name, and spmv_run launches it in place of the
// ahead-of-time kernel.  Without hipRTC (or when a compile fails) the plan keeps its ahead-of-time
// kernels and says why in its description.
#include <hip/hip_runtime_api.h>
#include <hip/hiprtc.h>

#include <map>
#include <mutex>
#include <sstream>

#include "internal.h"
#include "jit_source.inc"

namespace spmv {

bool plan_wants_jit(const PlanSpec &q) {
    if (q.node == N_LEAF) return q.jit != 0;
    for (const PlanSpec &k : q.kids)
        if (plan_wants_jit(k)) return true;
    return false;
}

// For one launch: the instantiation the ahead-of-time dispatch above would pick, spelled as a name
// expression, and the #define lines that turn its run-time arguments into literals (and fitted offset
// arrays into arithmetic).  Launch kinds without an entry here keep their ahead-of-time kernel.  The
// instantiations named here are the ones the ahead-of-time dispatch in kernels.hip picks.
bool jit_describe(const Plan &plan, const Part &p, std::string &kernel, std::string &defines) {
    const char *T = plan.dtype == SPMV_F64 ? "double" : "float";
    auto B = [](bool b) { return b ? "true" : "false"; };
    std::ostringstream k, d;
    auto def = [&](const char *name, int64_t v) { d << "#define SPMV_JIT_" << name << " " << v << "LL\n"; };
    auto defi = [&](const char *name, int64_t v) { d << "#define SPMV_JIT_" << name << " " << v << "\n"; };
    auto model = [&](const char *name, const void *ptr) {   // closed form of an offset array, if one was fitted
        for (const DevArray &a : plan.arrays)
            if (a.ptr == ptr && a.model.kind) d << "#define SPMV_JIT_" << name << "(i) " << a.model.expr("i") << "\n";
    };
    switch (p.kind) {
    case K_DIA:
        if (p.ndiag < 1 || p.ndiag > 8) return false;
        if (p.lanes == 2 || p.lanes == 4) k << "spmv::dev::k_dia_rows<" << T << ", " << p.ndiag << ", " << p.lanes << ", " << B(p.accumulate) << ">";
        else k << "spmv::dev::k_dia_fixed<" << T << ", " << p.ndiag << ", " << B(p.accumulate) << ">";
        d << "#define SPMV_JIT_DIA_OFFS ";
        for (int i = 0; i < 8; ++i) d << (i ? "," : "") << (i < p.ndiag ? p.dia_offsets[i] : 0);
        d << "\n";
        def("DIA_LD", p.ld);
        def("DIA_NROWS", plan.nrows);
        def("DIA_NCOLS", plan.ncols);
        break;
    case K_CSRV:
        if (p.lanes > kWave) return false;
        k << "spmv::dev::k_csrv<" << T << ", " << p.lanes << ", " << B(p.has_rows) << ", " << B(p.accumulate) << ">";
        def("CSRV_NSEG", p.units);
        defi("CSRV_ULEN", p.uniform_w);
        defi("CSRV_REMAP", p.remap);
        if (p.uniform_w < 0) model("SEG_PTR", p.p0);
        break;
    case K_SELL:
        k << "spmv::dev::k_sell<" << T << ", " << B(p.has_rows) << ", " << B(p.accumulate) << ">";
        def("SELL_NSLICES", p.units);
        def("SELL_NROWS", p.nrows);
        defi("SELL_REMAP", p.remap);
        defi("SELL_UW", p.uniform_w);
        if (p.uniform_w < 0) model("SLICE_PTR", p.p0);
        break;
    case K_BSELL:
        if (p.lds_bytes > 0) k << "spmv::dev::k_bsell_xwin<" << T << ", " << p.block << ", " << B(p.has_rows) << ", " << B(p.uniform_w == 1) << ">";
        else k << "spmv::dev::k_bsell<" << T << ", " << p.block << ", " << B(p.has_rows) << ">";
        def("BSELL_NSLICES", p.units);
        def("BSELL_NBROWS", p.nrows);
        defi("BSELL_REMAP", p.remap);
        model("SLICE_PTR", p.p0);
        break;
    case K_STRIPE:
        k << (p.delta ? "spmv::dev::k_hsell_delta<" : "spmv::dev::k_hsell<") << T << ", " << B(p.p5 != nullptr) << ", " << (p.lanes == 1024 ? 1024 : 512) << ">";
        defi("HS_NSL", p.nslices);
        defi("HS_NH", p.nrows);
        defi("HS_TILE", p.tile);
        def("HS_NCOLS", plan.ncols);
        defi("HS_NS", p.units);
        defi("HS_SPW", p.per_group);
        break;
    case K_REDUCE_WIDE:
        k << "spmv::dev::k_reduce_wide<" << T << ", " << B(p.accumulate) << ">";
        defi("RW_NP", p.ngroups);
        def("RW_N", p.nrows);
        break;
    case K_XL_MUL:
        k << "spmv::dev::k_xl_mul<" << T << ">";
        defi("XL_W", p.tile);
        def("XL_NCOLS", plan.ncols);
        break;
    case K_XL_REDUCE:
        k << "spmv::dev::k_xl_reduce<" << T << ", " << B(p.has_rows) << ", " << B(p.accumulate) << ", " << B(p.p4 != nullptr) << ">";
        defi("XLR_RB", p.tile);
        def("XLR_N", p.nrows);
        model("GPTR", p.p0);
        break;
    default: return false;
    }
    kernel = k.str();
    defines = d.str();
    return true;
}

namespace {

std::string device_arch() {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return "gfx950";
    }
    std::string a = prop.gcnArchName;   // e.g. "gfx950:sramecc+:xnack-"
    return a.empty() ? "gfx950" : a;
}

// Compiles defines + device code, returns the code object and the lowered name of `kernel`.
std::string compile(const std::string &defines, const std::string &kernel, std::vector<char> &code, std::string &lowered) {
    const std::string src = defines + "#include \"device_kernels.h\"\n";
    const char *headers[] = {kJitDeviceKernels, kJitConstants};
    const char *names[] = {"device_kernels.h", "constants.h"};
    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, src.c_str(), "spmv_jit.hip", 2, headers, names) != HIPRTC_SUCCESS) return "hiprtcCreateProgram failed";
    std::string err;
    const std::string arch = "--offload-arch=" + device_arch();
    const char *opts[] = {arch.c_str(), "-O3", "-std=c++17", "-munsafe-fp-atomics", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    if (hiprtcAddNameExpression(prog, kernel.c_str()) != HIPRTC_SUCCESS) err = "hiprtcAddNameExpression failed";
    if (err.empty() && hiprtcCompileProgram(prog, (int)(sizeof opts / sizeof opts[0]), opts) != HIPRTC_SUCCESS) {
        size_t n = 0;
        (void)hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n) (void)hiprtcGetProgramLog(prog, &log[0]);
        err = "hipRTC compile failed: " + log.substr(0, 600);
    }
    if (err.empty()) {
        const char *low = nullptr;
        if (hiprtcGetLoweredName(prog, kernel.c_str(), &low) != HIPRTC_SUCCESS || !low) err = "no lowered name for " + kernel;
        else lowered = low;
    }
    if (err.empty()) {
        size_t n = 0;
        if (hiprtcGetCodeSize(prog, &n) != HIPRTC_SUCCESS || n == 0) err = "empty code object";
        else {
            code.resize(n);
            if (hiprtcGetCode(prog, code.data()) != HIPRTC_SUCCESS) err = "hiprtcGetCode failed";
        }
    }
    (void)hiprtcDestroyProgram(&prog);
    return err;
}

// Does this device take module-loaded kernels with more than 64 KiB of dynamic LDS?  (There is no
// per-function attribute to raise for them.)  Asked once per process with a kernel that touches
// nothing but its own LDS.
std::mutex g_probe_mutex;
int g_big_lds = -1;
bool big_lds_ok() {
    std::lock_guard<std::mutex> lock(g_probe_mutex);
    if (g_big_lds >= 0) return g_big_lds == 1;
    g_big_lds = 0;
    const std::string src = "extern \"C\" __global__ void spmv_lds_probe(int n) { extern __shared__ int s[]; s[threadIdx.x] = n; }\n";
    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, src.c_str(), "probe.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS) return false;
    const std::string arch = "--offload-arch=" + device_arch();
    const char *opts[] = {arch.c_str()};
    std::vector<char> code;
    bool ok = hiprtcCompileProgram(prog, 1, opts) == HIPRTC_SUCCESS;
    size_t n = 0;
    ok = ok && hiprtcGetCodeSize(prog, &n) == HIPRTC_SUCCESS && n > 0;
    if (ok) {
        code.resize(n);
        ok = hiprtcGetCode(prog, code.data()) == HIPRTC_SUCCESS;
    }
    (void)hiprtcDestroyProgram(&prog);
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
    ok = ok && hipModuleLoadData(&mod, code.data()) == hipSuccess;
    ok = ok && hipModuleGetFunction(&fn, mod, "spmv_lds_probe") == hipSuccess;
    if (ok) {
        int arg = 0;
        void *args[] = {&arg};
        ok = hipModuleLaunchKernel(fn, 1, 1, 1, 64, 1, 1, 128 * 1024, nullptr, args, nullptr) == hipSuccess;
        ok = (hipDeviceSynchronize() == hipSuccess) && ok;
    }
    (void)hipGetLastError();
    if (mod) (void)hipModuleUnload(mod);
    g_big_lds = ok ? 1 : 0;
    return ok;
}

}  // namespace

void jit_compile_plan(Plan &plan) {
    if (plan.mem.host_only) {
        plan.jit_note = "host-only plan: nothing to compile";
        // the description still shows what would be compiled
        for (Part &p : plan.parts) (void)jit_describe(plan, p, p.jit_kernel, p.jit_defines);
        return;
    }
    std::map<std::string, void *> cache;   // identical (defines, kernel) pairs share a function
    int done = 0;
    for (Part &p : plan.parts) {
        std::string kernel, defines;
        if (!jit_describe(plan, p, kernel, defines)) continue;
        p.jit_kernel = kernel;
        p.jit_defines = defines;
        const bool needs_big = (p.kind == K_STRIPE && ((size_t)p.tile + (size_t)p.nrows) * plan.vsize() > 65536) ||
                               (p.kind == K_XL_MUL && (size_t)p.tile * plan.vsize() > 65536) ||
                               (p.kind == K_XL_REDUCE && (size_t)p.tile * 8 > 65536) || (p.kind == K_BSELL && p.lds_bytes > 65536);
        if (needs_big && !big_lds_ok()) {
            plan.jit_note += p.name + ": more than 64 KiB of LDS, kept ahead-of-time; ";
            continue;
        }
        const std::string key = defines + "\n" + kernel;
        auto it = cache.find(key);
        if (it != cache.end()) {
            p.jit_fn = it->second;
            ++done;
            continue;
        }
        std::vector<char> code;
        std::string lowered;
        const std::string err = compile(defines, kernel, code, lowered);
        if (!err.empty()) {
            plan.jit_note += p.name + ": " + err + "; ";
            continue;
        }
        hipModule_t mod = nullptr;
        hipFunction_t fn = nullptr;
        if (hipModuleLoadData(&mod, code.data()) != hipSuccess || hipModuleGetFunction(&fn, mod, lowered.c_str()) != hipSuccess) {
            (void)hipGetLastError();
            if (mod) (void)hipModuleUnload(mod);
            plan.jit_note += p.name + ": loading the compiled kernel failed; ";
            continue;
        }
        plan.jit_modules.push_back((void *)mod);
        p.jit_fn = (void *)fn;
        cache[key] = p.jit_fn;
        ++done;
    }
    if (done == 0 && plan.jit_note.empty()) plan.jit_note = "no launch of this plan has a run-time specialisation";
}

// Compile-only pass over every launch that has a specialisation (nothing is loaded or launched, so it
// also works where no device is present).  Returns the number compiled; failures are listed in `log`.
int jit_check_plan(const Plan &plan, std::string &log) {
    int ok = 0;
    for (const Part &p : plan.parts) {
        std::string kernel, defines, lowered;
        if (!jit_describe(plan, p, kernel, defines)) continue;
        std::vector<char> code;
        const std::string err = compile(defines, kernel, code, lowered);
        if (err.empty()) ++ok;
        else log += p.name + ": " + err + "\n";
    }
    return ok;
}

void jit_release_plan(Plan &plan) {
    for (void *m : plan.jit_modules) (void)hipModuleUnload((hipModule_t)m);
    plan.jit_modules.clear();
    for (Part &p : plan.parts) p.jit_fn = nullptr;
}

}  // namespace spmv
