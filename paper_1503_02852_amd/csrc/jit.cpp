// Run-time specialisation of the persistent recurrent-step kernel.
//
// The planner's element-wise programs are straight-line slot programs; here one component's
// programs (one direction) are printed as HIP source -- one descriptor struct per phase whose
// ops() is the program as plain C++ statements -- and compiled with hiprtc together with the
// shared kernel text of step_device.h.  Buffer ids, widths, offsets and weight offsets are not
// part of the source (the kernel reads them from the plan words at set-up), so components of
// equal structure, e.g. all LSTM layers of a stack, share one compiled kernel.  If hiprtc is
// not available or a compile fails, callers keep using the interpreted kernel of step.hip.
#include "jit.h"

#include <dlfcn.h>
#include <hip/hiprtc.h>

#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <sstream>
#include <vector>

#include "embedded_sources.h"

namespace rnng {
namespace {

struct Rtc {
    bool tried = false, ok = false;
    decltype(&hiprtcCreateProgram) create = nullptr;
    decltype(&hiprtcCompileProgram) compile = nullptr;
    decltype(&hiprtcGetProgramLogSize) log_size = nullptr;
    decltype(&hiprtcGetProgramLog) log = nullptr;
    decltype(&hiprtcGetCodeSize) code_size = nullptr;
    decltype(&hiprtcGetCode) code = nullptr;
    decltype(&hiprtcDestroyProgram) destroy = nullptr;
    void load() {
        if (tried) return;
        tried = true;
        void* h = dlopen("libhiprtc.so", RTLD_NOW | RTLD_LOCAL);
        if (!h) h = dlopen("/opt/rocm/lib/libhiprtc.so", RTLD_NOW | RTLD_LOCAL);
        if (!h) return;
#define RNNG_SYM(field, name) field = reinterpret_cast<decltype(field)>(dlsym(h, name)); if (!field) return
        RNNG_SYM(create, "hiprtcCreateProgram"); RNNG_SYM(compile, "hiprtcCompileProgram");
        RNNG_SYM(log_size, "hiprtcGetProgramLogSize"); RNNG_SYM(log, "hiprtcGetProgramLog");
        RNNG_SYM(code_size, "hiprtcGetCodeSize"); RNNG_SYM(code, "hiprtcGetCode"); RNNG_SYM(destroy, "hiprtcDestroyProgram");
#undef RNNG_SYM
        ok = true;
    }
};

struct CacheEntry { std::vector<char> code; hipModule_t module = nullptr; hipFunction_t fn = nullptr; bool failed = false; };

std::mutex g_mutex;
Rtc g_rtc;
std::map<std::string, CacheEntry> g_cache;   // key: generated source

void emit_ops(std::ostringstream& o, const int32_t* pw) {
    const int ng = pw[PG_NGATHER], ni = pw[PG_NINV], nops = pw[PG_NOPS];
    const int32_t* mo = pw + PG_HEADER_WORDS + ng * GA_WORDS + ni * IV_WORDS;
    for (int p = 0; p < nops; ++p) {
        const int packed = mo[p * MO_WORDS + MO_PACKED], c = mo[p * MO_WORDS + MO_C];
        const int opc = packed & 0xFF, d = (packed >> 8) & 0xFF, a = (packed >> 16) & 0xFF, b = (packed >> 24) & 0xFF;
        o << "        s[" << d << "] = ";
        switch (opc) {
            case MOP_MOV: o << "s[" << a << "]"; break;
            case MOP_ADD: o << "s[" << a << "] + s[" << b << "]"; break;
            case MOP_MUL: o << "s[" << a << "] * s[" << b << "]"; break;
            case MOP_FMA: o << "fmaf(s[" << a << "], s[" << b << "], s[" << c << "])"; break;
            case MOP_SIG: o << "step_sigmoid(s[" << a << "])"; break;
            case MOP_TANH: o << "step_tanh(s[" << a << "])"; break;
            case MOP_DSIG: o << "s[" << a << "] * s[" << b << "] * (1.0f - s[" << b << "])"; break;
            case MOP_DTANH: o << "s[" << a << "] * (1.0f - s[" << b << "] * s[" << b << "])"; break;
            default: o << "0.0f"; break;
        }
        o << ";\n";
    }
}

}  // namespace

std::string jit_step_source(const Plan& P, const CompPlan& cp, bool backward, int NB) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    int acc_phase = 0;
    for (size_t p = 0; p < phases.size(); ++p) {
        const PhasePlan& ph = phases[p];
        const int32_t* pw = &P.words[ph.prog_off];
        const int ng = pw[PG_NGATHER], ni = pw[PG_NINV], nops = pw[PG_NOPS], nst = pw[PG_NSTORES];
        if (ph.mv_off >= 0) acc_phase = (int)p;
        o << "struct PH" << p << " {\n";
        o << "    static constexpr int P = " << p << ", NG = " << ng << ", NI = " << ni << ", NST = " << nst
          << ", HAS_TASKS = " << (ph.mv_off >= 0 ? 1 : 0) << ", ACC_PHASE = " << acc_phase << ";\n";
        o << "    static __device__ __forceinline__ constexpr int gkind(int g) {\n        switch (g) {\n";
        for (int g = 0; g < ng; ++g)
            if (pw[PG_HEADER_WORDS + g * GA_WORDS + GA_KIND] == GA_KIND_ACC) o << "            case " << g << ": return 1;\n";
        o << "            default: return 0;\n        }\n    }\n";
        const int32_t* st = pw + PG_HEADER_WORDS + ng * GA_WORDS + ni * IV_WORDS + nops * MO_WORDS;
        o << "    static __device__ __forceinline__ constexpr int stslot(int q) {\n        switch (q) {\n";
        for (int q = 0; q < nst; ++q) o << "            case " << q << ": return " << st[q * ST_WORDS + ST_SLOT] << ";\n";
        o << "            default: return 0;\n        }\n    }\n";
        o << "    static __device__ __forceinline__ void ops(float* s) {\n";
        emit_ops(o, pw);
        o << "    }\n};\n";
    }
    o << "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n"
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ StepShared sh;\n"
         "    const int w = step_prologue<" << NB << ">(a, sh, lds);\n"
         "    if (w < 0) return;\n"
         "    const int tid = threadIdx.x;\n";
    for (size_t p = 0; p < phases.size(); ++p)
        o << "    PhaseRegs<PH" << p << "> r" << p << "; phase_setup<PH" << p << ", " << NB << ">(r" << p << ", a, sh, w, tid);\n";
    o << "    bool dead = false;\n"
         "    for (int step = 0; step < a.T; ++step) {\n"
         "        const int t = a.backward ? a.T - 1 - step : step;\n";
    for (size_t p = 0; p < phases.size(); ++p)
        o << "        phase_step<PH" << p << ", " << NB << ", " << phases.size() << ">(r" << p << ", a, sh, lds, t, tid, dead);\n";
    o << "    }\n}\n";
    return o.str();
}

bool jit_compile(const std::string& source, std::string* log_out) {
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_cache.find(source);
    if (it != g_cache.end()) return !it->second.failed;
    CacheEntry& ce = g_cache[source];
    ce.failed = true;
    g_rtc.load();
    if (!g_rtc.ok) { if (log_out) *log_out = "libhiprtc.so could not be loaded"; return false; }
    const char* header_src[3] = {RNNG_SRC_program_h, RNNG_SRC_step_layout_h, RNNG_SRC_step_device_h};
    const char* header_names[3] = {"program.h", "step_layout.h", "step_device.h"};
    hiprtcProgram prog = nullptr;
    if (g_rtc.create(&prog, source.c_str(), "rnng_step_jit.hip", 3, header_src, header_names) != HIPRTC_SUCCESS) {
        if (log_out) *log_out = "hiprtcCreateProgram failed";
        return false;
    }
    const char* opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-munsafe-fp-atomics",
                          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    const hiprtcResult r = g_rtc.compile(prog, (int)(sizeof(opts) / sizeof(opts[0])), opts);
    size_t ls = 0;
    g_rtc.log_size(prog, &ls);
    if (ls > 1 && log_out) { log_out->assign(ls, '\0'); g_rtc.log(prog, &(*log_out)[0]); }
    if (r != HIPRTC_SUCCESS) { g_rtc.destroy(&prog); return false; }
    size_t cs = 0;
    g_rtc.code_size(prog, &cs);
    ce.code.resize(cs);
    g_rtc.code(prog, ce.code.data());
    g_rtc.destroy(&prog);
    ce.failed = cs == 0;
    return !ce.failed;
}

hipFunction_t jit_step_function(const std::string& source) {
    if (!jit_compile(source, nullptr)) return nullptr;
    std::lock_guard<std::mutex> lock(g_mutex);
    CacheEntry& ce = g_cache[source];
    if (ce.fn) return ce.fn;
    if (ce.failed) return nullptr;
    if (hipModuleLoadData(&ce.module, ce.code.data()) != hipSuccess) { ce.failed = true; return nullptr; }
    if (hipModuleGetFunction(&ce.fn, ce.module, "rnng_step_jit") != hipSuccess) { ce.failed = true; ce.fn = nullptr; return nullptr; }
    // more than 64 KiB of dynamic LDS needs an opt-in; an error here surfaces at launch
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(ce.fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)STEP_LDS_LIMIT);
    return ce.fn;
}

void jit_mark_failed(const std::string& source) {
    std::lock_guard<std::mutex> lock(g_mutex);
    g_cache[source].failed = true;
    g_cache[source].fn = nullptr;
}

hipError_t jit_launch(hipFunction_t fn, StepArgs& a, const StepLaunchPlan& lp, hipStream_t stream) {
    void* params[1] = {&a};
    return hipModuleLaunchKernel(fn, (unsigned)(lp.G * lp.xcd_stride), 1, 1, STEP_THREADS, 1, 1, (unsigned)lp.lds_bytes, stream,
                                 params, nullptr);
}

}  // namespace rnng
