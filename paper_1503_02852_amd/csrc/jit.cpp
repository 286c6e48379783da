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
#include <algorithm>
#include <cstdlib>
#include <map>
#include <mutex>
#include <sstream>
#include <vector>

#include "embedded_sources.h"
#include "step_device.h"

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

struct CacheEntry { std::vector<char> code; hipModule_t module = nullptr; hipFunction_t fn = nullptr; bool failed = false; std::string log; };

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
            case MOP_RELU: o << "fmaxf(s[" << a << "], 0.0f)"; break;
            case MOP_DRELU: o << "(s[" << b << "] > 0.0f ? s[" << a << "] : 0.0f)"; break;
            case MOP_MAX: o << "fmaxf(s[" << a << "], s[" << b << "])"; break;
            case MOP_GE: o << "(s[" << a << "] >= s[" << b << "] ? 1.0f : 0.0f)"; break;
            case MOP_GT: o << "(s[" << a << "] > s[" << b << "] ? 1.0f : 0.0f)"; break;
            default: o << "0.0f"; break;
        }
        o << ";\n";
    }
}

}  // namespace

namespace {

void emit_phase_descriptor(std::ostringstream& o, const Plan& P, const PhasePlan& ph, int p, int acc_phase) {
    const int32_t* pw = &P.words[ph.prog_off];
    const int ng = pw[PG_NGATHER], ni = pw[PG_NINV], nops = pw[PG_NOPS], nst = pw[PG_NSTORES];
    o << "struct PH" << p << " {\n";
    o << "    static constexpr int P = " << p << ", NG = " << ng << ", NI = " << ni << ", NST = " << nst
      << ", HAS_TASKS = " << (ph.mv_off >= 0 ? 1 : 0) << ", ACC_PHASE = " << acc_phase << ";\n";
    auto gw = [&](int g, int field) { return pw[PG_HEADER_WORDS + g * GA_WORDS + field]; };
    auto emit_switch = [&](const char* name, const char* arg, const std::vector<std::pair<int, int>>& cases) {
        o << "    static __device__ __forceinline__ constexpr int " << name << "(int " << arg << ") {\n        switch (" << arg << ") {\n";
        for (auto& c : cases) o << "            case " << c.first << ": return " << c.second << ";\n";
        o << "            default: return 0;\n        }\n    }\n";
    };
    std::vector<std::pair<int, int>> kinds, auxs, sidx, cidx, sgather;
    int ns = 0, nc = 0;
    for (int g = 0; g < ng; ++g) {
        const int kind = gw(g, GA_KIND);
        kinds.push_back({g, kind});
        if (kind == GA_KIND_CARRY) { auxs.push_back({g, gw(g, GA_AUX)}); cidx.push_back({g, nc++}); }
        if (kind == GA_KIND_ACC) auxs.push_back({g, gw(g, GA_FRAME_OFF)});   // index of the task in its phase
        if (kind == GA_KIND_STATIC) { sidx.push_back({g, ns}); sgather.push_back({ns, g}); ++ns; }
    }
    o << "    static constexpr int NS = " << ns << ", NC = " << nc << ";\n";
    emit_switch("gkind", "g", kinds); emit_switch("gaux", "g", auxs); emit_switch("sidx", "g", sidx);
    emit_switch("cidx", "g", cidx); emit_switch("sgather", "si", sgather);
    const int32_t* st = pw + PG_HEADER_WORDS + ng * GA_WORDS + ni * IV_WORDS + nops * MO_WORDS;
    std::vector<std::pair<int, int>> slots, shareds, twins;
    for (int q = 0; q < nst; ++q) {
        slots.push_back({q, st[q * ST_WORDS + ST_SLOT]});
        if (st[q * ST_WORDS + ST_FLAGS] & 1) shareds.push_back({q, 1});
        const int b = st[q * ST_WORDS + ST_BUF];
        if (P.twin_base >= 0 && b < P.twin_base && P.buf_alloc[P.twin_base + b] == 3) twins.push_back({q, 1});
    }
    // (sttwin: the stored tensor has a tile-blocked twin, which many-stream kernels poll instead of it)
    emit_switch("stslot", "q", slots); emit_switch("stshared", "q", shareds); emit_switch("sttwin", "q", twins);
    o << "    static __device__ __forceinline__ void ops(float* s) {\n";
    emit_ops(o, pw);
    o << "    }\n};\n";
}

}  // namespace

std::string jit_step_source(const Plan& P, const CompPlan& cp, bool backward, int NB) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    int acc_phase = 0;
    for (size_t p = 0; p < phases.size(); ++p) {
        if (phases[p].mv_off >= 0) acc_phase = (int)p;
        emit_phase_descriptor(o, P, phases[p], (int)p, acc_phase);
    }
    o << "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n"
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ StepShared sh;\n"
         "    const int w = step_prologue<" << NB << ">(a, sh, lds);\n"
         "    if (w < 0) return;\n"
         "    const int tid = threadIdx.x;\n";
    for (size_t p = 0; p < phases.size(); ++p)
        o << "    PhaseRegs<PH" << p << "> r" << p << "; phase_setup<PH" << p << ", " << NB << ">(r" << p << ", a, sh, lds, w, tid);\n";
    o << "    __syncthreads();\n"
         "    bool dead = false;\n"
         "    const int nsteps = step_count(a);\n"
         "    for (int step = 0; step < nsteps; ++step) {\n"
         "        const int t = step_frame(a, step);\n";
    for (size_t p = 0; p < phases.size(); ++p)
        o << "        phase_step<PH" << p << ", " << NB << ", " << phases.size() << ">(r" << p << ", a, sh, lds, step, t, tid, dead);\n";
    o << "    }\n}\n";
    return o.str();
}

// Wave-autonomous variant: single-phase components whose weight rows fit the register file.
// Emits namespace <ns> { PH0, MV, body(a, w) } for one component; false if the component (with
// G workgroups and N streams) is not eligible.
namespace {
// Tensors that the wave-autonomous kernel of this component polls (an exchange bundle's
// interleaved tensor stands for its members).
std::vector<int> polled_buffers(const Plan& P, const CompPlan& cp, bool backward, int N, int G) {
    std::vector<int> out;
    const int NB = step_nb_for(N);
    StepLayout lay;
    compute_step_layout(P.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, G, NB > 0 ? NB : 1, N, lay);
    if (!lay.ok) return out;
    for (int s = 0; s < lay.n_sources; ++s) {
        const int bi = P.bundle_of[lay.src[s].buf];
        out.push_back(bi >= 0 ? P.bundles[bi].ebuf : lay.src[s].buf);
    }
    // and the sums of a helper member that the element-wise program polls
    for (const PhasePlan& ph : backward ? cp.bwd_phases : cp.fwd_phases) {
        const int32_t* pw = &P.words[ph.prog_off];
        for (int g = 0; g < pw[PG_NGATHER]; ++g)
            if (pw[PG_HEADER_WORDS + g * GA_WORDS + GA_KIND] == GA_KIND_POLLED) out.push_back(pw[PG_HEADER_WORDS + g * GA_WORDS + GA_BUF]);
    }
    return out;
}

// group: index of this component in a chain launch (0 for a launch of its own); foreign: tensors
// that the other groups of the chain poll.
// *lds_bytes (optional): the static LDS of the group's body.
bool emit_wave_group(std::ostringstream& o, const Plan& P, const CompPlan& cp, bool backward, int N, int G, const std::string& ns,
                     int group, const std::vector<int>& foreign, size_t* lds_bytes = nullptr) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    const int NB = step_nb_for(N);
    if (phases.size() != 1 || NB == 0) return false;
    StepLayout lay;
    compute_step_layout(P.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, G, NB, N, lay);
    if (!lay.ok) return false;
    const StepPhase& ph = lay.ph[0];
    const int UW = (ph.item_chunk + 3) / 4;
    if (UW * NB > 8) return false;
    std::vector<int> F(lay.n_sources), xoff(lay.n_sources);
    int XF = 0;
    for (int s = 0; s < lay.n_sources; ++s) { F[s] = (lay.src[s].k_len + 63) / 64; xoff[s] = XF; XF += F[s]; }
    if (XF * NB > 128) return false;
    for (int s = 0; s < lay.n_sources; ++s) if (F[s] > 32) return false;
    int per_unit = 0;
    for (int t = 0; t < ph.n_tasks; ++t) for (int e = 0; e < ph.task[t].n_edges; ++e) per_unit += F[ph.task[t].e[e].src];
    const int RW = UW * per_unit;
    if (RW > 384) return false;
    if (lds_bytes) {
        const int32_t* pw = P.words.data() + phases[0].prog_off;
        int n_static = 0, xs = 0;
        for (int g = 0; g < pw[PG_NGATHER]; ++g) n_static += pw[PG_HEADER_WORDS + g * GA_WORDS + GA_KIND] == GA_KIND_STATIC;
        for (int s = 0; s < lay.n_sources; ++s) xs += NB * 64 * ((F[s] + 3) / 4 * 4);
        const size_t ring = (size_t)4 * 16 * std::max(1, n_static * UW * NB), tables = (size_t)STEP_MAX_PHASES * STEP_THREADS * 6;
        *lds_bytes = 4 * (ring + 2 * (size_t)std::max(1, xs)) + sizeof(StepLayout) + tables;
    }
    // Rows of more than 1,024 elements (or very wide source sets): the weights, the source values,
    // the partial sums and the polling registers of a lane together must fit the 512 registers of a
    // wavefront that has a SIMD to itself with room to spare, else the kernel spills (a 2,048-wide
    // LSTM layer forward: fine at 1 and 2 streams, 257 registers spilled at 4).
    bool long_rows = XF * NB > 96;
    for (int s = 0; s < lay.n_sources; ++s) long_rows = long_rows || F[s] > 16;
    if (long_rows) {
        int polled_words = 0;
        for (int s = 0; s < lay.n_sources; ++s) polled_words += NB * lay.src[s].k_len;
        if (RW + XF * NB + 2 * UW * ph.n_tasks * NB + (polled_words + 255) / 256 > 440) return false;
    }
    o << "namespace " << ns << " {\n";
    emit_phase_descriptor(o, P, phases[0], 0, 0);
    auto emit_switch = [&](const char* name, const char* arg, const std::vector<std::pair<int, int>>& cases) {
        o << "    static __device__ __forceinline__ constexpr int " << name << "(int " << arg << ") {\n        switch (" << arg << ") {\n";
        for (auto& c : cases) o << "            case " << c.first << ": return " << c.second << ";\n";
        o << "            default: return 0;\n        }\n    }\n";
    };
    // polled regions: sources that belong to an exchange bundle share the bundle's interleaved tensor
    struct Region { int buf, foff, rk, fr, off; };
    std::vector<Region> regs;
    std::vector<int> sreg(lay.n_sources), sb(lay.n_sources), sj(lay.n_sources);
    int XFR = 0;
    for (int s = 0; s < lay.n_sources; ++s) {
        const int bi = P.bundle_of[lay.src[s].buf];
        int rbuf = lay.src[s].buf, B = 1, j = 0;
        if (bi >= 0) {
            const BundlePlan& bp = P.bundles[bi];
            rbuf = bp.ebuf; B = bp.B;
            for (int m = 0; m < 4; ++m) if (bp.members[m] == lay.src[s].buf) j = m;
        }
        int r = 0;
        for (; r < (int)regs.size(); ++r) if (regs[r].buf == rbuf && regs[r].foff == lay.src[s].frame_off) break;
        if (r == (int)regs.size()) {
            const int fr = F[s] * B;
            regs.push_back(Region{rbuf, lay.src[s].frame_off, lay.src[s].k_len * B, fr, XFR});
            XFR += fr;
        }
        sreg[s] = r; sb[s] = B; sj[s] = j;
    }
    for (const Region& rg : regs) if (NB * rg.rk > ((rg.rk & 1) ? 4096 : 8192)) return false;
    // bundle stores: stores of this program into bundle members
    const int32_t* pw0 = P.words.data() + phases[0].prog_off;
    const int32_t* st0 = pw0 + PG_HEADER_WORDS + pw0[PG_NGATHER] * GA_WORDS + pw0[PG_NINV] * IV_WORDS + pw0[PG_NOPS] * MO_WORDS;
    struct BStore { int bundle; int q[4]; };
    std::vector<BStore> bstores;
    std::vector<std::pair<int, int>> bundled;
    for (int q = 0; q < pw0[PG_NSTORES]; ++q) {
        if (!(st0[q * ST_WORDS + ST_FLAGS] & 1)) continue;
        const int bi = P.bundle_of[st0[q * ST_WORDS + ST_BUF]];
        if (bi < 0) continue;
        size_t k = 0;
        for (; k < bstores.size(); ++k) if (bstores[k].bundle == bi) break;
        if (k == bstores.size()) bstores.push_back(BStore{bi, {-1, -1, -1, -1}});
        for (int m = 0; m < 4; ++m) if (P.bundles[bi].members[m] == st0[q * ST_WORDS + ST_BUF]) bstores[k].q[m] = q;
        bundled.push_back({q, 1});
    }
    for (const BStore& b : bstores) {
        // every member must be stored by this program, member 0 included
        for (int m = 0; m < 4; ++m) if ((P.bundles[b.bundle].members[m] >= 0) != (b.q[m] >= 0)) return false;
    }
    // who polls an exchanged tensor: 0 this group only, 1 other groups only, 2 both
    auto reader_mode = [&](int buf) {
        bool own = false, other = false;
        for (const Region& rg : regs) own = own || rg.buf == buf;
        for (int f : foreign) other = other || f == buf;
        return other ? (own ? 2 : 1) : 0;
    };
    std::vector<std::pair<int, int>> xmode, bs_xmode;
    for (int q = 0; q < pw0[PG_NSTORES]; ++q) {
        if (!(st0[q * ST_WORDS + ST_FLAGS] & 1) || P.bundle_of[st0[q * ST_WORDS + ST_BUF]] >= 0) continue;
        xmode.push_back({q, reader_mode(st0[q * ST_WORDS + ST_BUF])});
    }
    for (size_t b = 0; b < bstores.size(); ++b) bs_xmode.push_back({(int)b, reader_mode(P.bundles[bstores[b].bundle].ebuf)});
    // Two placements, both measured.  (1) The stores of values nobody polls go out right behind
    // the exchanged ones (their acknowledgements overlap the exchange) or one step late, behind
    // the next step's poll: forward loops are faster with the first; backward loops with the
    // second when a wavefront has a long matrix-vector part for the late stores to hide under
    // (charlm_n1: 4 units per wavefront, 1.35 against 1.48 ms), with the first when it is short
    // (speech_n1: 2 units, 1.22 against 1.27 ms).  (2) When every wavefront owns units (one loop,
    // no helper path), a step's first polling attempt can go out at the end of the step before:
    // faster wherever the stores are early (speech_n1 0.98 -> 0.96 / 1.22 -> 1.20 ms, charlm_n1
    // forward 0.85 -> 0.83), slower behind deferred stores (1.35 -> 1.44) and with helper
    // wavefronts (tiny).  RNNG_WAVE_EARLY_STORES / RNNG_WAVE_POLL_EARLY = 0 / 1 override.
    const bool all_own = 3 * UW < ph.item_chunk;
    bool early_stores = !backward || (all_own && UW <= 2);
    if (const char* env = std::getenv("RNNG_WAVE_EARLY_STORES")) early_stores = std::atoi(env) != 0;
    bool poll_early = all_own && early_stores;
    if (const char* env = std::getenv("RNNG_WAVE_POLL_EARLY")) poll_early = std::atoi(env) != 0;
    o << "struct MV {\n    static constexpr int NT = " << ph.n_tasks << ", UW = " << UW << ", NSRC = " << lay.n_sources
      << ", RW = " << RW << ", XF = " << XF << ", EARLY = " << (early_stores ? 1 : 0) << ", NREG = " << regs.size()
      << ", XFR = " << XFR << ", NBS = " << bstores.size() << ", PE = " << (poll_early ? 1 : 0) << ", SW = RNNG_STORE_WINDOW, N = " << N << ";\n";
    std::vector<std::pair<int, int>> ne, es, fs, xo, wo, ks;
    for (int s = 0; s < lay.n_sources; ++s) ks.push_back({s, lay.src[s].k_len});
    for (int t = 0; t < ph.n_tasks; ++t) {
        ne.push_back({t, ph.task[t].n_edges});
        for (int e = 0; e < ph.task[t].n_edges; ++e) es.push_back({t * STEP_MAX_EDGES + e, ph.task[t].e[e].src});
    }
    for (int s = 0; s < lay.n_sources; ++s) { fs.push_back({s, F[s]}); xo.push_back({s, xoff[s]}); }
    int woff = 0;
    for (int ul = 0; ul < UW; ++ul)
        for (int t = 0; t < ph.n_tasks; ++t)
            for (int e = 0; e < ph.task[t].n_edges; ++e) {
                wo.push_back({(ul * (ph.n_tasks > 0 ? ph.n_tasks : 1) + t) * STEP_MAX_EDGES + e, woff});
                woff += F[ph.task[t].e[e].src];
            }
    emit_switch("nedges", "task", ne); emit_switch("esrc_", "key", es); emit_switch("F", "s", fs);
    emit_switch("xoff", "s", xo); emit_switch("woff_", "key", wo); emit_switch("K", "s", ks);
    {
        std::vector<std::pair<int, int>> rb, rf, rk, fr, ro, sr, sbb, sjj, be, bB, bd, bm, bq;
        for (int r = 0; r < (int)regs.size(); ++r) {
            rb.push_back({r, regs[r].buf}); rf.push_back({r, regs[r].foff}); rk.push_back({r, regs[r].rk});
            fr.push_back({r, regs[r].fr}); ro.push_back({r, regs[r].off});
        }
        for (int s2 = 0; s2 < lay.n_sources; ++s2) { sr.push_back({s2, sreg[s2]}); sbb.push_back({s2, sb[s2]}); sjj.push_back({s2, sj[s2]}); }
        for (int k = 0; k < (int)bstores.size(); ++k) {
            const BundlePlan& bp = P.bundles[bstores[k].bundle];
            be.push_back({k, bp.ebuf}); bB.push_back({k, bp.B}); bd.push_back({k, bp.dim}); bm.push_back({k, bp.members[0]});
            for (int m = 0; m < 4; ++m) bq.push_back({k * 4 + m, bstores[k].q[m]});
        }
        std::vector<std::pair<int, int>> rbf, rsr;
        for (int r = 0; r < (int)regs.size(); ++r) {
            int B = 1;
            for (int s2 = 0; s2 < lay.n_sources; ++s2) if (sreg[s2] == r) B = sb[s2];
            rbf.push_back({r, B});
            for (int m = 0; m < 4; ++m) {
                int src = -1;
                for (int s2 = 0; s2 < lay.n_sources; ++s2) if (sreg[s2] == r && sj[s2] == m) src = s2;
                rsr.push_back({r * 4 + m, src});
            }
        }
        emit_switch("rbuf", "r", rb); emit_switch("rfoff", "r", rf); emit_switch("RK", "r", rk); emit_switch("RB", "r", rbf);
        emit_switch("rsrc_", "key", rsr);
        o << "    static __device__ __forceinline__ constexpr int rsrc(int r, int j) { return rsrc_(r * 4 + j); }\n";
        emit_switch("bs_ebuf", "b", be); emit_switch("bs_B", "b", bB); emit_switch("bs_dim", "b", bd); emit_switch("bs_member0", "b", bm);
        emit_switch("bs_q_", "key", bq); emit_switch("bundled", "q", bundled);
        emit_switch("xmode", "q", xmode); emit_switch("bs_xmode", "b", bs_xmode);
        o << "    static __device__ __forceinline__ constexpr int bs_q(int b, int j) { return bs_q_(b * 4 + j); }\n";
    }
    o << "    static __device__ __forceinline__ constexpr int esrc(int task, int e) { return esrc_(task * " << STEP_MAX_EDGES << " + e); }\n";
    o << "    static __device__ __forceinline__ constexpr int woff(int ul, int task, int e) { return woff_((ul * "
      << (ph.n_tasks > 0 ? ph.n_tasks : 1) << " + task) * " << STEP_MAX_EDGES << " + e); }\n};\n";
    // (the group's LDS as one struct: a chain launch overlays those of its groups, of which a
    // workgroup runs exactly one)
    o << "struct Lds {\n"
         "    StepShared sh;\n"
         "    float ring_all[4][WaveRing<PH0, MV, " << NB << ">::FLOATS];\n"
         "    __attribute__((aligned(16))) float xs_all[2 * GroupX<MV, " << NB << ">::FLOATS];\n"
         "};\n"
         "__device__ __forceinline__ void body(const StepArgs& a, int w, Lds& l) {\n"
         "    StepShared& sh = l.sh;\n"
         "    auto& ring_all = l.ring_all;\n"
         "    float* xs_all = l.xs_all;\n"
         "    wave_prologue<MV, " << NB << ">(a, sh);\n"
         "    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;\n"
         "    // same in all lanes; false: the wavefront only helps polling\n"
         "    const bool has_units = suni((int)(wave * MV::UW < sh.lay.ph[0].item_chunk)) != 0;\n"
         "    for (int i = tid; i < 2 * GroupX<MV, " << NB << ">::FLOATS; i += 256) xs_all[i] = 0.0f;\n"
         "    float* ring = ring_all[wave];\n"
         "    PhaseRegs<PH0> r0; phase_setup<PH0, " << NB << ", 1>(r0, a, sh, nullptr, w, tid);\n"
         "    wave_store_setup<PH0, MV>(r0, a);\n"
         "    WaveRegs<MV> wv; wave_setup<MV>(wv, a, sh, w, tid);\n"
         "    wave_bundle_setup<PH0, MV>(wv, r0, a);\n"
         "    wave_xcd_setup<MV>(wv, a, " << group << ");\n"
         "    WaveRing<PH0, MV, " << NB << "> rg; wave_ring_setup<PH0, MV, " << NB << ">(rg, a, sh, w, tid);\n"
         "    if (PH0::NS > 0) wave_ring_fill<PH0, MV, " << NB << ">(rg, a, ring, lane);\n"
         "    float pf[2][WaveRing<PH0, MV, " << NB << ">::QNA] = {{0.0f}};\n"
         "    __syncthreads();\n"
         "    float dfv[PH0::NST > 0 ? PH0::NST : 1] = {0.0f};\n"
         "    bool dead = false;\n"
         "    const int nsteps = step_count(a);\n"
         "    if (nsteps > 0) wave_carry_init<PH0>(r0, a);\n"
         "    PollRegs<MV> pr;\n"
         "    if (MV::NSRC > 0 && nsteps > 0 && MV::PE) group_poll_issue<MV, " << NB << ">(pr, wv, a, step_frame(a, 0), tid);\n"
         "    auto loop = [&](auto hu) {\n"
         "        constexpr int HU = decltype(hu)::value;\n"
         "        int step = 0;\n"
         "        for (; step + 1 < nsteps; step += 2) {\n"
         "            wave_step<PH0, MV, " << NB << ", 0, HU>(r0, wv, rg, pf, dfv, pr, a, ring, xs_all, has_units, step, step_frame(a, step), tid, dead);\n"
         "            wave_step<PH0, MV, " << NB << ", 1, HU>(r0, wv, rg, pf, dfv, pr, a, ring, xs_all, has_units, step + 1, step_frame(a, step + 1), tid, dead);\n"
         "        }\n"
         "        if (step < nsteps) wave_step<PH0, MV, " << NB << ", 0, HU>(r0, wv, rg, pf, dfv, pr, a, ring, xs_all, has_units, step, step_frame(a, step), tid, dead);\n"
         "        const bool owns = HU == 2 ? has_units : HU != 0;\n"
         "        if (!MV::EARLY && owns && nsteps > 0) wave_flush_stores<PH0, MV>(r0, dfv, a);\n"
         "        if (wave_has_late_stores<MV>() && owns && nsteps > 0) wave_store_through_late<PH0, MV>(r0, wv, dfv, a, step_frame(a, nsteps - 1), MV::EARLY != 0);\n"
         "    };\n"
         "    // every wavefront owns units: one loop without the helper's path\n"
         "    if (MV::NSRC > 0 && !(3 * MV::UW < " << ph.item_chunk << ")) loop(StepIntC<2>{});\n"
         "    else if (has_units) loop(StepIntC<1>{});\n"
         "    else if (MV::NSRC > 0) loop(StepIntC<0>{});\n"
         "}\n}  // namespace " << ns << "\n";
    return true;
}
}  // namespace

std::string jit_wave_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G) {
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    if (!emit_wave_group(o, P, cp, backward, N, G, "grp0", 0, std::vector<int>())) return "";
    o << "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n"
         "void rnng_step_jit(StepArgs a) {\n"
         "    __shared__ grp0::Lds l;\n"
         "    const int w = step_part_index(a);\n"
         "    if (w < 0) return;\n"
         "    grp0::body(a, w, l);\n"
         "}\n";
    return o.str();
}

// Chain of recurrent components side by side in one launch: group g (component members[g], with
// G[g] workgroups on XCD g) runs its own wave-autonomous body; a member's full connections from
// earlier members are ordinary polled sources, so the groups trail each other by about one step.
std::string jit_chain_source(const Plan& P, const std::vector<CompPlan>& members, bool backward, int N, const std::vector<int>& G) {
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    const int n = (int)members.size();
    if (n < 2 || n > STEP_MAX_GROUPS || (int)G.size() != n) return "";
    size_t lds_total = 0;
    for (int g = 0; g < n; ++g) {
        std::vector<int> foreign;
        for (int h = 0; h < n; ++h)
            if (h != g)
                for (int b : polled_buffers(P, members[h], backward, N, G[h])) foreign.push_back(b);
        size_t lds = 0;
        if (G[g] > 32 || !emit_wave_group(o, P, members[g], backward, N, G[g], "grp" + std::to_string(g), g, foreign, &lds)) return "";
        lds_total = std::max(lds_total, lds);
    }
    if (lds_total > 158 * 1024) return "";      // of 160 KiB (the groups' areas lie on top of each other)
    o << "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n"
         "void rnng_step_jit(StepArgs a) {\n"
         "    __shared__ union Lds {\n";
    for (int g = 0; g < n; ++g) o << "        grp" << g << "::Lds l" << g << ";\n";
    o << "    } lds;\n"
         "    const int grp = blockIdx.x & 7, w = blockIdx.x >> 3;\n"
         "    if (grp >= a.n_groups || w >= a.grp_G[grp]) return;\n"
         "    StepArgs b = a;\n"
         "    b.desc_off = a.grp_desc_off[grp]; b.G = a.grp_G[grp];\n"
         "    switch (grp) {\n";
    for (int g = 0; g < n; ++g) o << "        case " << g << ": grp" << g << "::body(b, w, lds.l" << g << "); break;\n";
    o << "        default: break;\n    }\n}\n";
    return o.str();
}

// Matrix-core variant for N >= 9 streams (single-phase components).  Empty if not eligible;
// otherwise *lds_bytes receives the dynamic LDS size.
namespace {
// One component of a matrix-core kernel: descriptors PH0 and MM inside namespace ns.
// blocked: exchange through the tile-blocked twins (only if every exchanged tensor has one and the
// streams come in whole 16-stream tiles).
bool emit_mstep_group(std::ostringstream& o, const Plan& P, const CompPlan& cp, bool backward, int N_all, int G, int J, int NW, bool blocked,
                      const std::string& ns, size_t* lds_bytes, int* rows) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    if (phases.size() != 1 || N_all < 1 || J < 1 || G * J > 256) return false;
    if (J > 1 && N_all % (16 * J) != 0) return false;      // stream groups of whole 16-stream tiles
    const int N = (N_all + J - 1) / J;                   // streams per workgroup
    StepLayout lay;
    compute_step_layout(P.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, G, 1, N, lay);
    if (!lay.ok) return false;
    const int CW = 16 * NW;      // columns of a chunk
    MLayout ml;
    compute_mstep_layout(lay, N, NW, 0u, (int)(MSTEP_LDS_LIMIT / 4), ml);
    // Weight rows that do not fit LDS go to vector registers, whole sources at a time and the
    // largest first (eight wavefronts only: 256 registers per lane, of which the weights may
    // take 144; the chunk sequence must be short enough to be unrolled, so that every register
    // index is static).  A lane keeps 4 words per (chunk, row tile the source feeds).
    unsigned reg_mask = 0;
    int reg_words = 0;
    if (!ml.ok && lay.ok && lay.n_phases == 1 && NW == 8 && !(std::getenv("RNNG_MSTEP_REGS") && std::atoi(std::getenv("RNNG_MSTEP_REGS")) == 0)) {
        const StepPhase& ph0 = lay.ph[0];
        const int ntu0 = (ph0.n_tasks * ph0.cmax + 15) / 16;
        int nch0 = 0;
        for (int s = 0; s < lay.n_sources; ++s) nch0 += (lay.src[s].k_len + CW - 1) / CW;
        auto words_of = [&](int s) {      // registers per lane if source s lives there
            int tiles = 0;
            for (int nt = 0; nt < ntu0; ++nt) {
                bool any = false;
                for (int col = nt * 16; col < nt * 16 + 16 && !any; ++col) {
                    const int t = col / ph0.cmax;
                    if (t >= ph0.n_tasks) continue;
                    for (int e = 0; e < ph0.task[t].n_edges; ++e) if (ph0.task[t].e[e].src == s) any = true;
                }
                tiles += any;
            }
            return (lay.src[s].k_len + CW - 1) / CW * tiles * 4;
        };
        int flat_max0 = 64;
        if (const char* env = std::getenv("RNNG_MSTEP_FLAT_MAX")) flat_max0 = std::max(0, std::min(64, std::atoi(env)));
        while (nch0 <= flat_max0) {
            int pick = -1;
            for (int s = 0; s < lay.n_sources; ++s)
                if (!((reg_mask >> s) & 1) && (pick < 0 || words_of(s) > words_of(pick))) pick = s;
            if (pick < 0 || reg_words + words_of(pick) > 144) break;
            reg_mask |= 1u << pick; reg_words += words_of(pick);
            compute_mstep_layout(lay, N, NW, reg_mask, (int)(MSTEP_LDS_LIMIT / 4), ml);
            if (ml.ok) break;
        }
    }
    if (!ml.ok || (size_t)ml.total_floats * 4 > MSTEP_LDS_LIMIT) return false;
    if (blocked) {
        if (N_all < 16 || N_all % 16 != 0 || N % 16 != 0 || P.twin_base < 0) return false;
        auto has_twin = [&](int b) { return b >= 0 && b < P.twin_base && P.buf_alloc[P.twin_base + b] == 3; };
        // (a helper member's sums are read element by element from the row-major tensor)
        if (!cp.helper) for (int b : backward ? cp.bwd_shared_bufs : cp.fwd_shared_bufs) if (!has_twin(b)) return false;
        for (int s = 0; s < ml.n_src; ++s) if (!has_twin(lay.src[s].buf) || lay.src[s].k_len != P.buf_dim[lay.src[s].buf]) return false;
    }
    const StepPhase& ph = lay.ph[0];
    const int MT = (N + 15) / 16, NTU = (ph.n_tasks * ph.cmax + 15) / 16;
    if (MT * NTU > 16) return false;     // accumulator registers
    // D register sets, D - 1 chunks in flight (see the kernel): about a dozen 128-bit loads per lane
    // (measured: more in flight is slower), and among the depths up to that the one that pads the
    // sources' chunk sequences least
    int kmax = 0;
    for (int s = 0; s < ml.n_src; ++s) kmax = std::max(kmax, lay.src[s].k_len);
    // short chunk sequences are unrolled whole: the chunks in flight may then span several sources
    int nch = 0;
    for (int s = 0; s < ml.n_src; ++s) nch += (lay.src[s].k_len + CW - 1) / CW;
    int flat_max = 64;
    if (const char* env = std::getenv("RNNG_MSTEP_FLAT_MAX")) flat_max = std::max(0, std::min(64, std::atoi(env)));      // (tests: the grouped sequence on small shapes)
    const bool flat = nch <= flat_max;
    // loads in flight per lane: about four with eight wavefronts (measured on two workloads: 4 / 8 / 12
    // in flight give 1.81 / 1.88 / 1.91 ms and 3.56 / 3.59 / 3.70 ms), a dozen with four
    const int inflight = NW == 8 ? 4 : 12;
    const int dmax = flat ? std::max(2, std::min(inflight / MT + 1, nch + 1)) : std::max(2, std::min(inflight / MT + 1, (kmax + CW - 1) / CW + 1));
    int D = dmax, best_slots = 1 << 30;
    for (int d = dmax; !flat && d >= std::max(2, dmax / 2); --d) {
        int slots = 0;
        for (int s = 0; s < ml.n_src; ++s) slots += ((lay.src[s].k_len + CW - 1) / CW + d - 1) / d * d;
        if (slots < best_slots) { best_slots = slots; D = d; }
    }
    if (const char* env = std::getenv("RNNG_MSTEP_DEPTH")) D = std::max(2, std::min(flat ? std::min(16 / MT + 1, nch + 1) : dmax, std::atoi(env)));      // (measurement)
    o << "namespace " << ns << " {\n";
    emit_phase_descriptor(o, P, phases[0], 0, 0);
    auto emit_switch = [&](const char* name, const char* arg, const std::vector<std::pair<int, int>>& cases, int dflt) {
        o << "    static __device__ __forceinline__ constexpr int " << name << "(int " << arg << ") {\n        switch (" << arg << ") {\n";
        for (auto& c : cases) o << "            case " << c.first << ": return " << c.second << ";\n";
        o << "            default: return " << dflt << ";\n        }\n    }\n";
    };
    o << "struct MM {\n    static constexpr int NJ = " << N << ", MT = " << MT << ", NSRC = " << ml.n_src << ", NTU = " << NTU
      << ", D = " << D << ", CMAX = " << ml.cmax << ", ACCS = " << ml.accstride << ", NW = " << NW << ", NCH = " << nch << ";\n"
      << "    static constexpr bool FLAT = " << (flat ? "true" : "false") << ", XB = " << (blocked ? "true" : "false")
      << ", HELPER = " << (cp.helper ? "true" : "false") << ";\n"
      ;
    std::vector<std::pair<int, int>> ks, blk, used, ngr, csrc, ck0;
    // The unrolled chunk sequence takes the sources in the order in which their values arrive: what
    // another component of the launch produces (it runs ahead) and the component's own values of
    // older frames first, the values that the other workgroups have produced in the step before
    // (frame offset +- 1) last, so that the first multiplications run while those are on their way.
    // CLATE: the first chunk of the latter.
    int clate = 0;
    if (flat) {
        const std::vector<int>& own = backward ? cp.bwd_shared_bufs : cp.fwd_shared_bufs;
        auto late = [&](int s) { return std::find(own.begin(), own.end(), lay.src[s].buf) != own.end() && std::abs(lay.src[s].frame_off) <= 1; };
        std::vector<int> ord;
        for (int s = 0; s < ml.n_src; ++s) if (!late(s)) ord.push_back(s);
        for (int s = 0; s < ml.n_src; ++s) if (late(s)) ord.push_back(s);
        int c = 0;
        bool seen_late = false;
        for (int s : ord) {
            if (late(s) && !seen_late) { clate = c; seen_late = true; }
            for (int k = 0; k < lay.src[s].k_len; k += CW, ++c) { csrc.push_back({c, s}); ck0.push_back({c, k}); }
        }
        if (!seen_late) clate = c;
    }
    for (int s = 0; s < ml.n_src; ++s) {
        ks.push_back({s, lay.src[s].k_len});
        for (int t = 0; t < ph.n_tasks; ++t) if (ml.blk[s][t] >= 0) blk.push_back({s * STEP_MAX_TASKS + t, ml.blk[s][t]});
        for (int nt = 0; nt < NTU; ++nt) {
            bool any = false;
            for (int col = nt * 16; col < nt * 16 + 16; ++col) {
                const int t = col / ml.cmax;
                if (t < ph.n_tasks && ml.blk[s][t] >= 0) any = true;
            }
            if (any) used.push_back({s * 16 + nt, 1});
        }
        ngr.push_back({s, ((lay.src[s].k_len + CW - 1) / CW + D - 1) / D});
    }
    emit_switch("K", "s", ks, 0); emit_switch("blk_", "key", blk, -1); emit_switch("used_", "key", used, 0);
    emit_switch("ngr", "s", ngr, 0); emit_switch("csrc", "c", csrc, 0); emit_switch("ck0", "c", ck0, 0);
    // register-resident weights: index of (chunk, row tile) in the lane's register array
    std::vector<std::pair<int, int>> widx;
    if (reg_mask && !flat) return false;
    for (auto& cs : csrc)
        if ((reg_mask >> cs.second) & 1)
            for (int nt = 0; nt < NTU; ++nt)
                if (std::find(used.begin(), used.end(), std::make_pair(cs.second * 16 + nt, 1)) != used.end()) { const int i = (int)widx.size(); widx.push_back({cs.first * 16 + nt, i}); }
    emit_switch("widx", "key", widx, 0);
    o << "    static constexpr unsigned REGMASK = " << reg_mask << "u;\n    static constexpr int NRW = " << widx.size() << ", CLATE = " << clate << ";\n";
    o << "    static __device__ __forceinline__ constexpr int blk(int s, int task) { return blk_(s * " << STEP_MAX_TASKS << " + task); }\n";
    o << "    static __device__ __forceinline__ constexpr bool used(int s, int nt) { return used_(s * 16 + nt) != 0; }\n};\n";
    o << "}  // namespace " << ns << "\n";
    if (lds_bytes) *lds_bytes = (size_t)ml.total_floats * 4;
    if (rows) *rows = ph.n_tasks * ph.cmax;
    return true;
}
}  // namespace

// Wavefronts per workgroup of the matrix-core variant: eight where that fits (twice the loads in
// flight per compute unit), else four.  RNNG_MSTEP_WAVES = 4 / 8 allows only that count.
static std::vector<int> mstep_wave_counts() {
    if (const char* env = std::getenv("RNNG_MSTEP_WAVES")) { const int v = std::atoi(env); if (v == 4 || v == 8) return {v}; }
    return {8, 4};
}
static const char* mstep_kernel_attributes(int NW) {
    return NW == 8 ? "extern \"C\" __global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))\n"
                   : "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n";
}

// RNNG_MSTEP_BLOCKED = 0: no exchange through tile-blocked twins (the row-major path, as for ragged stream counts).
static std::vector<int> mstep_blocked_choices() {
    if (const char* env = std::getenv("RNNG_MSTEP_BLOCKED")) if (std::atoi(env) == 0) return {0};
    return {1, 0};
}

std::string jit_mstep_source(const Plan& P, const CompPlan& cp, bool backward, int N_all, int G, int J, size_t* lds_bytes, int* rows, int* threads,
                             bool* blocked) {
    std::ostringstream o;
    int NW = 0; bool xb = false;
    for (int nw : mstep_wave_counts()) {
        for (int b : mstep_blocked_choices()) {
            o.str("");
            o << "#include \"step_device.h\"\nusing namespace rnng;\n";
            if (emit_mstep_group(o, P, cp, backward, N_all, G, J, nw, b != 0, "grp0", lds_bytes, rows)) { NW = nw; xb = b != 0; break; }
        }
        if (NW) break;
    }
    if (!NW) return "";
    if (threads) *threads = 64 * NW;
    if (blocked) *blocked = xb;
    o << mstep_kernel_attributes(NW) <<
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ MShared ms;\n"
         "    int w = blockIdx.x;\n"
         "    if (a.xcd_stride > 1) {\n"
         "        if (w % a.xcd_stride) return;\n"
         "        w /= a.xcd_stride;\n"
         "    }\n"
         "    mstep_kernel_body<grp0::PH0, grp0::MM>(a, ms, lds, w);\n"
         "}\n";
    return o.str();
}

// Matrix-core variant with the two-dimensional split (G workgroups in row groups of GJ).  Empty
// if not eligible; otherwise *lds_bytes receives the dynamic LDS size and *partial_floats the
// floats per frame of the partial-sum tensor.
std::string jit_mstep2_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, int GJ, size_t* lds_bytes,
                              int64_t* partial_floats) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    if (phases.size() != 1 || N < 1 || N > 64 || G > 256 || (GJ != 16 && GJ != 4) || G % GJ != 0) return "";
    StepLayout lay;
    compute_step_layout(P.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, G, 1, N, lay);
    if (!lay.ok) return "";
    M2Layout ml;
    compute_mstep2_layout(lay, N, GJ, (int)(STEP_LDS_LIMIT / 4), ml);
    if (!ml.ok || (size_t)ml.total_floats * 4 > STEP_LDS_LIMIT) return "";
    const StepPhase& ph = lay.ph[0];
    const int MT = (N + 15) / 16, RT = ph.n_tasks * ph.cmax;
    {   // the row tiles must divide among the wavefronts (see the kernel)
        const int RP = RT <= 4 ? 4 : RT <= 8 ? 8 : 16, TT = GJ / (16 / RP);
        const int WPS = (MT == 1 || MT == 2 || MT == 4) ? 4 / MT : 4;
        if (TT < 1 || TT % WPS != 0) return "";
    }
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    emit_phase_descriptor(o, P, phases[0], 0, 0);
    auto emit_switch = [&](const char* name, const char* arg, const std::vector<std::pair<int, int>>& cases, int dflt) {
        o << "    static __device__ __forceinline__ constexpr int " << name << "(int " << arg << ") {\n        switch (" << arg << ") {\n";
        for (auto& c : cases) o << "            case " << c.first << ": return " << c.second << ";\n";
        o << "            default: return " << dflt << ";\n        }\n    }\n";
    };
    std::vector<std::pair<int, int>> ks, kss, nch, pos0, blk;
    int pos = 0, nchmax = 0;
    for (int s = 0; s < ml.n_src; ++s) {
        const int K = lay.src[s].k_len, KS = K / GJ;
        ks.push_back({s, K}); kss.push_back({s, KS}); nch.push_back({s, KS / 64}); pos0.push_back({s, pos});
        pos += KS / 64; nchmax = std::max(nchmax, KS / 64);
        for (int t = 0; t < ph.n_tasks; ++t) if (ml.blk[s][t] >= 0) blk.push_back({s * STEP_MAX_TASKS + t, ml.blk[s][t]});
    }
    if (pos > 24) return "";      // the chunk sequence is unrolled
    // register sets: one position in flight while one is multiplied (measured: loads issued
    // earlier come back with sentinels more often, and the reloads cost more than the overlap gains)
    const int DS = std::max(1, std::min(pos, 2));
    std::vector<std::pair<int, int>> psrc, pchunk;
    for (int s2 = 0, q = 0; s2 < ml.n_src; ++s2)
        for (int c = 0; c < lay.src[s2].k_len / GJ / 64; ++c, ++q) { psrc.push_back({q, s2}); pchunk.push_back({q, c}); }
    (void)nchmax;
    o << "struct M2 {\n    static constexpr int NJ = " << N << ", MT = " << MT << ", NSRC = " << ml.n_src << ", GJ = " << GJ << ", RT = " << RT
      << ", CMAX = " << ml.cmax << ", ACCS = " << ml.accstride << ", PT = " << pos << ", DS = " << DS << ";\n";
    emit_switch("K", "s", ks, 0); emit_switch("KS", "s", kss, 0); emit_switch("psrc", "p", psrc, 0); emit_switch("pchunk", "p", pchunk, 0);
    emit_switch("blk_", "key", blk, -1);
    o << "    static __device__ __forceinline__ constexpr int blk(int s, int task) { return blk_(s * " << STEP_MAX_TASKS << " + task); }\n};\n";
    o << "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n"
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ M2Shared ms;\n"
         "    mstep2_kernel_body<PH0, M2>(a, ms, lds, (int)blockIdx.x);\n"
         "}\n";
    if (lds_bytes) *lds_bytes = (size_t)ml.total_floats * 4;
    if (partial_floats) *partial_floats = (int64_t)G * GJ * RT * (MT * 16);
    return o.str();
}

// Several components side by side (a chain): group g takes the blocks [grp_first[g], ...).
std::string jit_mstep_chain_source(const Plan& P, const std::vector<CompPlan>& members, bool backward, int N, const std::vector<int>& G,
                                   const std::vector<int>& J, size_t* lds_bytes, int* threads, bool* blocked) {
    std::ostringstream o;
    const int n = (int)members.size();
    if (n < 2 || n > STEP_MAX_GROUPS || (int)G.size() != n || (int)J.size() != n) return "";
    size_t lds_max = 0;
    int total = 0, NW = 0; bool xb = false;
    for (int nw : mstep_wave_counts()) {      // one launch: the same number of wavefronts and the same exchange for all members
        for (int b : mstep_blocked_choices()) {
            o.str("");
            o << "#include \"step_device.h\"\nusing namespace rnng;\n";
            lds_max = 0; total = 0;
            bool all = true;
            for (int g = 0; g < n && all; ++g) {
                size_t lds = 0;
                all = emit_mstep_group(o, P, members[g], backward, N, G[g], J[g], nw, b != 0, "grp" + std::to_string(g), &lds, nullptr);
                lds_max = std::max(lds_max, lds);
                total += G[g] * J[g];
            }
            if (all) { NW = nw; xb = b != 0; break; }
        }
        if (NW) break;
    }
    if (!NW) return "";
    if (blocked) *blocked = xb;
    if (total > 256) return "";      // every workgroup must be resident: they wait for each other
    if (threads) *threads = 64 * NW;
    o << mstep_kernel_attributes(NW) <<
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ MShared ms;\n"
         "    const int b = blockIdx.x;\n"
         "    StepArgs c = a;\n";
    for (int g = 0; g < n; ++g)
        o << "    if (b >= a.grp_first[" << g << "] && b < a.grp_first[" << g << "] + a.grp_G[" << g << "] * a.grp_J[" << g << "]) {\n"
             "        c.desc_off = a.grp_desc_off[" << g << "]; c.G = a.grp_G[" << g << "]; c.J = a.grp_J[" << g << "];\n"
             "        mstep_kernel_body<grp" << g << "::PH0, grp" << g << "::MM>(c, ms, lds, b - a.grp_first[" << g << "]);\n"
             "        return;\n"
             "    }\n";
    o << "}\n";
    if (lds_bytes) *lds_bytes = lds_max;
    return o.str();
}

// Streaming variant for N <= 8 streams and layers whose weights do not fit on chip: G unit chunks,
// weights read from memory every step.  Empty if not eligible; otherwise *lds_bytes receives the
// dynamic LDS size and *transposed whether the kernel reads transposed copies of some matrices.
std::string jit_sstep_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, size_t* lds_bytes, bool* transposed) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    if (phases.size() != 1 || N < 1 || N > 8 || G < 1 || G > 256) return "";
    if (P.n_params * 4 >= (int64_t(1) << 31)) return "";      // 32-bit byte offsets into the weight buffers
    StepLayout lay;
    compute_step_layout(P.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, G, 1, N, lay);
    if (!lay.ok || lay.n_sources < 1) return "";
    const StepPhase& ph = lay.ph[0];
    if (ph.n_tasks < 1 || ph.item_chunk * N > STEP_THREADS) return "";
    const int NT = ph.n_tasks, CMAX = ph.cmax, UW = (CMAX + 3) / 4;
    struct Seg { int ul, task, edge, src, tr; };
    std::vector<Seg> segs;
    bool any_t = false;
    for (int ul = 0; ul < UW; ++ul)
        for (int t = 0; t < NT; ++t)
            for (int e = 0; e < ph.task[t].n_edges; ++e) {
                segs.push_back(Seg{ul, t, e, ph.task[t].e[e].src, ph.task[t].e[e].transposed});
                any_t = any_t || ph.task[t].e[e].transposed;
                if (ph.task[t].e[e].k_len != lay.src[ph.task[t].e[e].src].k_len) return "";
            }
    const int NSEG = (int)segs.size(), NACC = UW * NT;
    if (NSEG < 1 || NSEG > 32 || NACC * N > 128) return "";
    int JMAX = 0, XF = 0, PQ = 0;
    std::vector<int> xoff(lay.n_sources), pq0(lay.n_sources), pqn(lay.n_sources);
    for (int sidx = 0; sidx < lay.n_sources; ++sidx) {
        const int K = lay.src[sidx].k_len;
        if (K % 4 != 0) return "";
        const int KP = (K + 255) / 256 * 256;
        JMAX = std::max(JMAX, KP / 256);
        xoff[sidx] = XF; XF += N * KP;
        pq0[sidx] = PQ; pqn[sidx] = (N * K / 4 + STEP_THREADS - 1) / STEP_THREADS; PQ += pqn[sidx];
    }
    if (PQ > 48) return "";
    const int ACCS = NT * CMAX + 1;
    const size_t lds = (size_t)(XF + N * ACCS) * 4;
    if (lds > STEP_LDS_LIMIT) return "";
    // prefetch depth: about 32 128-bit loads per lane in flight, a power of two that divides the
    // chunk count where it can (then the loop needs no bounds tests)
    int PD = 1;
    while (PD * 2 * NSEG <= 32 && PD * 2 <= 8 && PD * 2 <= JMAX) PD *= 2;
    while (PD > 1 && JMAX % PD != 0) PD /= 2;
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    emit_phase_descriptor(o, P, phases[0], 0, 0);
    auto emit_switch = [&](const char* name, const char* arg, const std::vector<std::pair<int, int>>& cases, int dflt) {
        o << "    static __device__ __forceinline__ constexpr int " << name << "(int " << arg << ") {\n        switch (" << arg << ") {\n";
        for (auto& c : cases) o << "            case " << c.first << ": return " << c.second << ";\n";
        o << "            default: return " << dflt << ";\n        }\n    }\n";
    };
    o << "struct SS {\n    static constexpr int NB = " << N << ", CMAX = " << CMAX << ", UW = " << UW << ", NT = " << NT << ", NSRC = " << lay.n_sources
      << ", NSEG = " << NSEG << ", PD = " << PD << ", JMAX = " << JMAX << ", NACC = " << NACC << ", XF = " << XF << ", ACCS = " << ACCS
      << ", PQ = " << PQ << ";\n";
    std::vector<std::pair<int, int>> sul, stask, sedge, ssrc, str_, ks, kps, xo, p0, pn;
    for (int i = 0; i < NSEG; ++i) {
        sul.push_back({i, segs[i].ul}); stask.push_back({i, segs[i].task}); sedge.push_back({i, segs[i].edge});
        ssrc.push_back({i, segs[i].src}); str_.push_back({i, segs[i].tr});
    }
    for (int sidx = 0; sidx < lay.n_sources; ++sidx) {
        ks.push_back({sidx, lay.src[sidx].k_len}); kps.push_back({sidx, (lay.src[sidx].k_len + 255) / 256 * 256});
        xo.push_back({sidx, xoff[sidx]}); p0.push_back({sidx, pq0[sidx]}); pn.push_back({sidx, pqn[sidx]});
    }
    emit_switch("seg_ul", "i", sul, 0); emit_switch("seg_task", "i", stask, 0); emit_switch("seg_edge", "i", sedge, 0);
    emit_switch("seg_src", "i", ssrc, 0); emit_switch("seg_tr", "i", str_, 0);
    emit_switch("K", "s", ks, 0); emit_switch("KP", "s", kps, 0); emit_switch("xoff", "s", xo, 0);
    emit_switch("pq0", "s", p0, 0); emit_switch("pqn", "s", pn, 0);
    o << "};\n";
    o << "extern \"C\" __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))\n"
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ SShared ms;\n"
         "    sstep_kernel_body<PH0, SS>(a, ms, lds, (int)blockIdx.x);\n"
         "}\n";
    if (lds_bytes) *lds_bytes = lds;
    if (transposed) *transposed = any_t;
    return o.str();
}

// Streaming matrix-core variant for N >= 9 streams and layers whose weights do not fit on chip.
std::string jit_smstep_source(const Plan& P, const CompPlan& cp, bool backward, int N, int G, size_t* lds_bytes, bool* transposed, bool* blocked,
                              int* threads) {
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    if (phases.size() != 1 || N < 9 || G < 1 || G > 256) return "";
    if (P.n_params * 4 >= (int64_t(1) << 31)) return "";      // 32-bit byte offsets into the weight buffers
    const int32_t* pg = P.words.data() + phases[0].prog_off;
    const int ic = (pg[PG_MAXDIM] + G - 1) / G;
    if (ic < 1 || ic > STEP_THREADS) return "";
    const int SPP = std::min(N, STEP_THREADS / ic), IPT = (N + SPP - 1) / SPP;
    if (IPT > 8) return "";
    StepLayout lay;
    compute_step_layout(P.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, G, 1, SPP, lay);
    if (!lay.ok || lay.n_sources < 1) return "";
    const StepPhase& ph = lay.ph[0];
    if (ph.n_tasks < 1) return "";
    const int NT = ph.n_tasks, CMAX = ph.cmax;
    const int MT = (N + 15) / 16, NTU = (NT * CMAX + 15) / 16;
    if (MT * NTU > 16) return "";
    int tr = -1;
    std::vector<std::pair<int, int>> edge_of;      // (s * STEP_MAX_TASKS + task) -> edge
    for (int t = 0; t < NT; ++t)
        for (int e = 0; e < ph.task[t].n_edges; ++e) {
            const StepEdge& ed = ph.task[t].e[e];
            if (tr >= 0 && tr != ed.transposed) return "";
            tr = ed.transposed;
            if (ed.k_len != lay.src[ed.src].k_len || ed.k_len % 4 != 0) return "";
            for (auto& pr : edge_of) if (pr.first == ed.src * STEP_MAX_TASKS + t) return "";      // two connections of one task from one source
            edge_of.push_back({ed.src * STEP_MAX_TASKS + t, e});
        }
    if (tr < 0) return "";
    int kmax = 0;
    for (int sidx = 0; sidx < lay.n_sources; ++sidx) kmax = std::max(kmax, lay.src[sidx].k_len);
    // Eight wavefronts (256 registers per lane) where the operand sets and accumulators fit, else
    // four; RNNG_SMSTEP_WAVES = 4 / 8 allows only that count.  D register sets, D - 1 chunks of
    // (MT + NTU) 128-bit loads per lane in flight: about 40 with four wavefronts, 20 with eight.
    int NW = 8;
    if (const char* env = std::getenv("RNNG_SMSTEP_WAVES")) NW = std::atoi(env) == 4 ? 4 : 8;
    if (NW == 8 && 4 * (MT * NTU + 2 * (MT + NTU)) > 160) NW = 4;
    const int CW = 16 * NW, inflight = NW == 8 ? 20 : 40;
    const int dmax = std::max(2, std::min({8, inflight / (MT + NTU) + 1, (kmax + CW - 1) / CW + 1}));
    int D = dmax, best_slots = 1 << 30;
    for (int d = dmax; d >= std::max(2, dmax - 2); --d) {
        int slots = 0;
        for (int sidx = 0; sidx < lay.n_sources; ++sidx) slots += ((lay.src[sidx].k_len + CW - 1) / CW + d - 1) / d * d;
        if (slots < best_slots) { best_slots = slots; D = d; }
    }
    const int ACCS = NTU * 16 + 4;
    const size_t lds = (size_t)NW * MT * 16 * ACCS * 4;
    if (lds > STEP_LDS_LIMIT) return "";
    // exchange through the tile-blocked twins: whole 16-stream tiles in the window and in every
    // pass of the element-wise part, every exchanged tensor with a twin
    bool xb = N % 16 == 0 && (IPT == 1 || SPP % 16 == 0) && P.twin_base >= 0 && !mstep_blocked_choices().empty() && mstep_blocked_choices()[0] != 0;
    auto has_twin = [&](int b) { return b >= 0 && b < P.twin_base && P.buf_alloc[P.twin_base + b] == 3; };
    for (int b : backward ? cp.bwd_shared_bufs : cp.fwd_shared_bufs) xb = xb && has_twin(b);
    for (int sidx = 0; sidx < lay.n_sources; ++sidx) xb = xb && has_twin(lay.src[sidx].buf) && lay.src[sidx].k_len == P.buf_dim[lay.src[sidx].buf];
    std::ostringstream o;
    o << "#include \"step_device.h\"\nusing namespace rnng;\n";
    emit_phase_descriptor(o, P, phases[0], 0, 0);
    auto emit_switch = [&](const char* name, const char* arg, const std::vector<std::pair<int, int>>& cases, int dflt) {
        o << "    static __device__ __forceinline__ constexpr int " << name << "(int " << arg << ") {\n        switch (" << arg << ") {\n";
        for (auto& c : cases) o << "            case " << c.first << ": return " << c.second << ";\n";
        o << "            default: return " << dflt << ";\n        }\n    }\n";
    };
    o << "struct SM {\n    static constexpr int NJ = " << N << ", MT = " << MT << ", NSRC = " << lay.n_sources << ", NTU = " << NTU << ", D = " << D
      << ", CMAX = " << CMAX << ", ACCS = " << ACCS << ", TR = " << tr << ", IPT = " << IPT << ", SPP = " << SPP << ", NW = " << NW << ";\n"
      << "    static constexpr bool XB = " << (xb ? "true" : "false") << ";\n";
    std::vector<std::pair<int, int>> ks, used, ngr;
    for (int sidx = 0; sidx < lay.n_sources; ++sidx) {
        ks.push_back({sidx, lay.src[sidx].k_len});
        for (int nt = 0; nt < NTU; ++nt) {
            bool any = false;
            for (int col = nt * 16; col < nt * 16 + 16; ++col) {
                const int t = col / CMAX;
                for (auto& pr : edge_of) if (t < NT && pr.first == sidx * STEP_MAX_TASKS + t) any = true;
            }
            if (any) used.push_back({sidx * 16 + nt, 1});
        }
        ngr.push_back({sidx, ((lay.src[sidx].k_len + CW - 1) / CW + D - 1) / D});
    }
    emit_switch("K", "s", ks, 0); emit_switch("edge_", "key", edge_of, -1); emit_switch("used_", "key", used, 0); emit_switch("ngr", "s", ngr, 0);
    o << "    static __device__ __forceinline__ constexpr int edge(int s, int task) { return edge_(s * " << STEP_MAX_TASKS << " + task); }\n";
    o << "    static __device__ __forceinline__ constexpr bool used(int s, int nt) { return used_(s * 16 + nt) != 0; }\n};\n";
    o << mstep_kernel_attributes(NW) <<
         "void rnng_step_jit(StepArgs a) {\n"
         "    extern __shared__ __attribute__((aligned(16))) float lds[];\n"
         "    __shared__ SShared ms;\n"
         "    smstep_kernel_body<PH0, SM>(a, ms, lds, (int)blockIdx.x);\n"
         "}\n";
    if (lds_bytes) *lds_bytes = lds;
    if (transposed) *transposed = tr != 0;
    if (blocked) *blocked = xb;
    if (threads) *threads = 64 * NW;
    return o.str();
}

bool jit_compile(const std::string& source, std::string* log_out) {
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_cache.find(source);
    if (it != g_cache.end()) { if (it->second.failed && log_out) *log_out = it->second.log; return !it->second.failed; }
    CacheEntry& ce = g_cache[source];
    ce.failed = true;
    if (const char* dump = std::getenv("RNNG_JIT_DUMP")) {   // debugging aid: keep the generated sources
        static int counter = 0;
        const std::string path = std::string(dump) + "/rnng_step_jit_" + std::to_string(counter++) + ".hip";
        if (FILE* f = std::fopen(path.c_str(), "w")) { std::fwrite(source.data(), 1, source.size(), f); std::fclose(f); }
    }
    g_rtc.load();
    if (!g_rtc.ok) { ce.log = "libhiprtc.so could not be loaded"; if (log_out) *log_out = ce.log; return false; }
    const char* header_src[3] = {RNNG_SRC_program_h, RNNG_SRC_step_layout_h, RNNG_SRC_step_device_h};
    const char* header_names[3] = {"program.h", "step_layout.h", "step_device.h"};
    hiprtcProgram prog = nullptr;
    if (g_rtc.create(&prog, source.c_str(), "rnng_step_jit.hip", 3, header_src, header_names) != HIPRTC_SUCCESS) {
        ce.log = "hiprtcCreateProgram failed";
        if (log_out) *log_out = ce.log;
        return false;
    }
    std::vector<const char*> opts = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-munsafe-fp-atomics",
                                     "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    std::string minc_opt;
    if (const char* env = std::getenv("RNNG_MSTEP_POLL_INC")) { minc_opt = "-DMSTEP_POLL_INC=" + std::to_string(std::atoi(env)); opts.push_back(minc_opt.c_str()); }
    std::string wsleep_opt;
    // tuning aid: further -D options for the run-time build, separated by blanks
    std::vector<std::string> extra_defs;
    if (const char* env = std::getenv("RNNG_JIT_DEFINES")) {
        std::istringstream in(env);
        for (std::string d; in >> d;)
            if (d.rfind("-D", 0) == 0) extra_defs.push_back(d);
    }
    for (const std::string& d : extra_defs) opts.push_back(d.c_str());
    if (const char* env = std::getenv("RNNG_WAVE_SLEEP")) { wsleep_opt = "-DWAVE_RETRY_SLEEP=" + std::to_string(std::atoi(env)); opts.push_back(wsleep_opt.c_str()); }
    std::string sleep_opt;
    if (const char* env = std::getenv("RNNG_MSTEP_SLEEP")) { sleep_opt = "-DMSTEP_RETRY_SLEEP=" + std::to_string(std::atoi(env)); opts.push_back(sleep_opt.c_str()); }
    std::string trace_at_opt;
    if (const char* env = std::getenv("RNNG_STEP_TRACE_AT")) { trace_at_opt = "-DRNNG_STEP_TRACE_AT=" + std::to_string(std::atoi(env)); opts.push_back(trace_at_opt.c_str()); }
    std::string trace_opt;
    if (const char* env = std::getenv("RNNG_STEP_TRACE"))
        if (std::atoi(env) > 0) { trace_opt = "-DRNNG_STEP_TRACE=" + std::to_string(std::atoi(env)); opts.push_back(trace_opt.c_str()); }
    const hiprtcResult r = g_rtc.compile(prog, (int)opts.size(), opts.data());
    size_t ls = 0;
    g_rtc.log_size(prog, &ls);
    if (ls > 1) { ce.log.assign(ls, '\0'); g_rtc.log(prog, &ce.log[0]); if (log_out) *log_out = ce.log; }
    if (r != HIPRTC_SUCCESS) { g_rtc.destroy(&prog); return false; }
    size_t cs = 0;
    g_rtc.code_size(prog, &cs);
    ce.code.resize(cs);
    g_rtc.code(prog, ce.code.data());
    g_rtc.destroy(&prog);
    ce.failed = cs == 0;
    return !ce.failed;
}

bool jit_available() {
    std::lock_guard<std::mutex> lock(g_mutex);
    g_rtc.load();
    return g_rtc.ok;
}

hipFunction_t jit_step_function(const std::string& source, std::string* err, bool allow_load, unsigned max_dynamic_lds) {
    if (!allow_load) {
        std::lock_guard<std::mutex> lock(g_mutex);
        auto it = g_cache.find(source);
        if (it != g_cache.end() && it->second.fn) return it->second.fn;
        if (err) *err = "the kernel has not been loaded yet";
        return nullptr;
    }
    std::string log;
    if (!jit_compile(source, &log)) { if (err) *err = "compilation failed: " + log; return nullptr; }
    std::lock_guard<std::mutex> lock(g_mutex);
    CacheEntry& ce = g_cache[source];
    if (ce.fn) return ce.fn;
    hipError_t e = hipModuleLoadData(&ce.module, ce.code.data());
    if (e != hipSuccess) { (void)hipGetLastError(); if (err) *err = std::string("hipModuleLoadData: ") + hipGetErrorString(e); return nullptr; }
    e = hipModuleGetFunction(&ce.fn, ce.module, "rnng_step_jit");
    if (e != hipSuccess) { (void)hipGetLastError(); ce.fn = nullptr; if (err) *err = std::string("hipModuleGetFunction: ") + hipGetErrorString(e); return nullptr; }
    // more than 64 KiB of dynamic LDS needs an opt-in; an error here surfaces at launch
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(ce.fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
    (void)hipGetLastError();   // a refusal must not linger as the thread's last error
    return ce.fn;
}

hipError_t jit_launch(hipFunction_t fn, StepArgs& a, const StepLaunchPlan& lp, hipStream_t stream) {
    void* params[1] = {&a};
    return hipModuleLaunchKernel(fn, (unsigned)(lp.G * lp.xcd_stride), 1, 1, (unsigned)lp.threads, 1, 1, (unsigned)lp.lds_bytes, stream,
                                 params, nullptr);
}

}  // namespace rnng
