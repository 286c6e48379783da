// C-ABI boundary (declared in include/rnngraph.h) and the executor that walks the plan.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <array>
#include <tuple>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/rnngraph.h"
#include "../../include/rnngraph_aux.h"
#include "jit.h"
#include "kernels.h"
#include "plan.h"

using namespace rnng;

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string& msg) { g_last_error = msg; return code; }
int fail_hip(hipError_t e, const char* what) {
    return fail(RNN_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct Layout {
    int64_t table_off = 0, dims_off = 0, words_off = 0, blob_bytes = 0;
    int64_t sync_off = 0;                 // 1 KiB of zero-initialised control words; the loss (double) sits at its start
    std::vector<int64_t> buf_off;         // per buffer id, bytes; -1 = not in the workspace
    int64_t partial_off = -1;             // partial sums of the two-dimensional matrix-core kernels (one launch at a time)
    std::vector<int64_t> idx_off;         // per exec node id: int32 [(hist + T)][N] copy of a one-hot input's class indices, or -1
    int64_t wt_off = -1;                  // transposed copies of the matrices the streaming kernels read transposed (parameter layout)
    int64_t flags_off = 0;                // per buffer id: 1 = frame tensor of the workspace (has history frames)
    int64_t total = 0;
};
constexpr int64_t SYNC_BYTES = 1024;

int64_t g_layout_skew = 4352;      // bytes, a multiple of 256 (RNNG_LAYOUT_SKEW overrides: tuning aid)

// partial_floats: floats per frame of the largest partial-sum tensor any launch of the window needs
// transposed_copy: a streaming kernel of the window reads matrices transposed
Layout make_layout(const Plan& P, int T, int N, int64_t partial_floats, bool transposed_copy) {
    Layout L;
    int n_alloc = 0;
    const int K = (int)P.xnodes.size();
    int64_t cur = 0;
    L.table_off = cur; cur += (int64_t)P.n_bufs * 8;
    L.dims_off = cur; cur += (int64_t)P.n_bufs * 4;
    L.flags_off = cur; cur += (int64_t)P.n_bufs * 4;
    cur = align_up(cur, 16);
    L.words_off = cur; cur += (int64_t)P.words.size() * 4;
    L.blob_bytes = cur;
    cur = align_up(cur, 256);
    L.sync_off = cur; cur += SYNC_BYTES;
    L.buf_off.assign(P.n_bufs, -1);
    const int64_t F = (int64_t)(T + P.hist) * N;      // every frame tensor has P.hist history frames in front
    (void)K;
    auto place = [&](int b) {
        const int64_t rows = P.buf_alloc[b] == 2 ? N : F;
        L.buf_off[b] = cur; cur = align_up(cur + rows * P.buf_dim[b] * 4, 256);
        // Tensors of the same shape would lie a power of two apart, so the lines that a step polls
        // in several tensors at the same frame would all fall on the same memory channel: skew them.
        cur += g_layout_skew * (1 + n_alloc % 13);
        ++n_alloc;
    };
    for (int b = 0; b < P.n_bufs; ++b)
        if (P.buf_alloc[b] == 1 || P.buf_alloc[b] == 2) place(b);
    if (partial_floats > 0) { L.partial_off = cur; cur = align_up(cur + (int64_t)(T + P.hist) * partial_floats * 4, 256); }
    if (transposed_copy) { L.wt_off = cur; cur = align_up(cur + P.n_params * 4, 256); }
    // an input whose connections are delayed may be given as class indices: room for its indices with history frames
    L.idx_off.assign(P.xnodes.size(), -1);
    for (size_t k = 0; k < P.xnodes.size(); ++k)
        if (P.xnodes[k].kind == NODE_INPUT && P.input_delayed[k]) { L.idx_off[k] = cur; cur = align_up(cur + F * 4, 256); }
    // tile-blocked twins (whole 16-stream tiles only), behind everything else
    if (N >= 16 && N % 16 == 0)
        for (int b = 0; b < P.n_bufs; ++b)
            if (P.buf_alloc[b] == 3) place(b);
    L.total = cur;
    return L;
}

}  // namespace

// Optional kernel-class timing with HIP events on the caller's stream.
struct Profiler {
    struct Rec { int cls; hipEvent_t a, b; int64_t launches; };
    int mask = 0;
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    bool on(int cls) const { return (mask >> cls) & 1; }
    // returns the index of the open record or -1
    int begin(int cls, hipStream_t s) {
        if (!on(cls)) return -1;
        Rec r{cls, get(), get(), 0};
        if (!r.a || !r.b) return -1;
        (void)hipEventRecord(r.a, s);
        recs.push_back(r);
        return (int)recs.size() - 1;
    }
    void end(int idx, int64_t launches, hipStream_t s) {
        if (idx < 0) return;
        recs[idx].launches = launches;
        (void)hipEventRecord(recs[idx].b, s);
    }
    ~Profiler() {
        for (Rec& r : recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (hipEvent_t e : pool) (void)hipEventDestroy(e);
    }
};

// Which XCD the workgroups of a launch land on, observed once per device: xcc[r] is the hardware id
// of the XCD that ran every workgroup b with b % 8 == r of a probe launch (workgroups are dealt to
// the XCDs in turn), ok = false if some residue class was spread over several XCDs.  The step
// kernels that keep a group of workgroups on one residue class then exchange through that XCD's L2
// with plain stores, and each workgroup checks the id it was given against the one it runs on.
struct XcdMap { bool known = false, ok = false; int xcc[8] = {0, 0, 0, 0, 0, 0, 0, 0}; };

struct rnn_graph {
    Plan plan;
    Profiler prof;
    // state of the current window: T frames as the caller counts them; inside the library a frame
    // tensor has Ti() = hist() + T frames, the caller's frame t being internal frame hist() + t
    int T = 0, N = 0;
    int hist() const { return plan.hist; }
    int Ti() const { return T + plan.hist; }
    char* ws = nullptr;
    Layout layout;
    std::vector<char> blob;               // host copy of the plan tables (kept alive for the async upload)
    std::vector<const float*> inputs;     // per exec node id (input nodes only)
    const XcdMap* xcd = nullptr;          // set by the first forward call on this device
    std::vector<const int32_t*> onehot;   // per exec node id: class indices of a one-hot input, or nullptr
    const float* weights = nullptr;
    bool fwd_done = false, bptt_done = false;
    int fwd_upto = 0;                     // frames [0, fwd_upto) of the current window hold forward results
    bool framewise = false;               // benchmark mode: every frame on its own, no batching over frames
    bool deterministic = false;           // rnn_set_deterministic: one writer per gradient element, fixed summation order
    bool no_alloc = false;                // inside rnn_forward_static: load no code, create no events, stage no host copies
    PlanView view() const {
        PlanView pv;
        pv.buf_ptr = reinterpret_cast<float* const*>(ws + layout.table_off);
        pv.buf_dim = reinterpret_cast<const int32_t*>(ws + layout.dims_off);
        pv.words = reinterpret_cast<const int32_t*>(ws + layout.words_off);
        return pv;
    }
    // internal frame 0 of a workspace tensor; for an input read in place: the caller's tensor
    // (its frame 0 is internal frame hist())
    float* buf(int id) const {
        if (layout.buf_off[id] >= 0) return reinterpret_cast<float*>(ws + layout.buf_off[id]);
        if (id < (int)inputs.size() && inputs[id]) return const_cast<float*>(inputs[id]);
        return nullptr;
    }
    bool caller_input(int id) const { return layout.buf_off[id] < 0 && id < (int)inputs.size() && inputs[id] != nullptr; }
    // the caller's frame 0 of a workspace tensor
    float* frame0(int id) const { return buf(id) + (caller_input(id) ? 0 : (int64_t)hist() * N * plan.buf_dim[id]); }
    bool is_onehot(int buf) const { return buf >= 0 && buf < (int)onehot.size() && onehot[buf] != nullptr; }
    // class indices of a one-hot input with history frames in front (internal frame 0), or nullptr if the node keeps none
    int32_t* onehot_history(int buf) const {
        return buf >= 0 && buf < (int)layout.idx_off.size() && layout.idx_off[buf] >= 0 ? reinterpret_cast<int32_t*>(ws + layout.idx_off[buf]) : nullptr;
    }
    double* loss_ptr() const { return reinterpret_cast<double*>(ws + layout.sync_off); }
    unsigned* ctrl_ptr() const { return reinterpret_cast<unsigned*>(ws + layout.sync_off + 16); }
    int force_step_G = 0;
    int spin_limit = 1 << 22;             // bound of every wait inside a step kernel (polling attempts)
    int cu_count = 0;                     // compute units of the device of the current window (0: not asked yet)
    // which build ran the step loop of component c in direction d at its last launch (RNN_BUILD_*, 0: none yet)
    std::vector<std::array<int, 2>> served;
    bool use_jit = true;
    bool use_store_window = true;
    // Run-time specialised step kernels, chosen once per (component, direction, stream count).
    struct JitChoice { bool wave = false, mstep = false, stream = false, needs_t = false, blocked = false; int J = 1; StepLaunchPlan lp; std::string source, source_window; bool two_d = false; int64_t partial_floats = 0; };
    int force_step_J = 0;
    bool prefer_streaming = false;        // RNNG_STEP_BUILD=stream
    // the workgroups of a step launch wait for each other, so all of them must be resident at once:
    // one per compute unit (256 on a whole MI355X, fewer on a partition)
    int max_workgroups() const { return cu_count > 0 ? cu_count : 256; }
    std::map<std::tuple<int, bool, int>, JitChoice> jit_choices;
    const JitChoice& jit_choice(int comp, bool backward, int N) {
        const std::tuple<int, bool, int> key(comp, backward, N);
        auto it = jit_choices.find(key);
        if (it != jit_choices.end()) return it->second;
        JitChoice c;
        const CompPlan& cp = plan.comps[comp];
        auto try_streaming = [&]() {
            if (!c.source.empty()) return;
            for (int G : {256, 128, 64, 32}) {
                if (force_step_G > 0 && G != force_step_G) continue;
                if (G > max_workgroups()) continue;
                size_t lds = 0; bool tr = false, xb = false; int threads = 256;
                std::string src = N <= 8 ? jit_sstep_source(plan, cp, backward, N, G, &lds, &tr) : jit_smstep_source(plan, cp, backward, N, G, &lds, &tr, &xb, &threads);
                if (src.empty()) continue;
                c.source = src; c.stream = true; c.needs_t = tr; c.blocked = xb; c.lp.threads = threads;
                c.lp.ok = true; c.lp.G = G; c.lp.NB = 1; c.lp.lds_bytes = lds; c.lp.xcd_stride = 1;
                break;
            }
        };
        if (prefer_streaming) try_streaming();      // (tests: the streaming variant on shapes the other variants would take)
        // 1. wave-autonomous variant: weights in registers, no barriers (single-phase components)
        const int wave_G[6] = {32, 64, 128, 256, 16, 8};
        for (int i = 0; i < 6 && c.source.empty() && !c.stream; ++i) {
            const int G = force_step_G > 0 ? force_step_G : wave_G[i];
            if (G > max_workgroups()) { if (force_step_G > 0) break; continue; }
            c.source = jit_wave_source(plan, cp, backward, N, G);
            if (!c.source.empty()) {
                c.wave = true; c.lp.ok = true; c.lp.G = G; c.lp.NB = step_nb_for(N); c.lp.lds_bytes = 0;
                c.lp.xcd_stride = G <= 32 ? 8 : 1;
            }
            if (force_step_G > 0) break;
        }
        // 2. matrix-core variants for many streams (weights in LDS or registers, MFMA)
        // 2a. one-dimensional split: stream groups, as many as possible (every group halves the
        //     bytes a workgroup polls per step); unit chunks: as many as the compute units allow
        //     while a workgroup still fills a 16-row tile, else the smallest count whose weight
        //     rows fit on chip
        JitChoice one_d;
        int one_d_rows = -1;
        if (c.source.empty() && N > 8) {
            for (int J : {4, 2, 1}) {
                if (force_step_J > 0 && J != force_step_J) continue;
                JitChoice best; int best_rows = -1;
                for (int G : {256, 128, 64, 32, 16}) {
                    if (force_step_G > 0 && G != force_step_G) continue;
                    if (G * J > max_workgroups()) continue;
                    size_t lds = 0; int rows = 0, threads = 256; bool blocked = false;
                    std::string src = jit_mstep_source(plan, cp, backward, N, G, J, &lds, &rows, &threads, &blocked);
                    if (src.empty()) continue;
                    if (best_rows < 0 || (best_rows < 16 && rows > best_rows)) {      // first hit = most workgroups; move to fewer only to fill a tile
                        best.source = src; best.mstep = true; best.lp.ok = true; best.lp.G = G; best.lp.NB = 1; best.lp.lds_bytes = lds; best.J = J;
                        best.lp.threads = threads; best.blocked = blocked;
                        best.lp.xcd_stride = G * J <= 32 ? 8 : 1;
                        best_rows = rows;
                    }
                    if (best_rows >= 16) break;
                }
                if (!best.source.empty()) { one_d = best; one_d_rows = best_rows; break; }
            }
        }
        // 2b. the two-dimensional split, where a workgroup polls a sixteenth (or a quarter) of every
        //     source and the row groups' members share 16-row tiles, at the price of a second
        //     exchange per step: only where the one-dimensional split cannot fill its tiles
        //     (RNNG_MSTEP_2D = 1: wherever the kernel can run; = 0: never)
        const char* env2d = std::getenv("RNNG_MSTEP_2D");
        const bool forced_2d = env2d && std::atoi(env2d) != 0, no_2d = env2d && std::atoi(env2d) == 0;
        if (c.source.empty() && N > 8 && force_step_G <= 0 && force_step_J <= 0 && max_workgroups() >= 256 && !no_2d &&
            (forced_2d || one_d_rows < 16)) {
            StepLayout lay;
            compute_step_layout(plan.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, 256, 1, N, lay);
            int64_t polled = 0;
            if (lay.ok) for (int sidx = 0; sidx < lay.n_sources; ++sidx) polled += (int64_t)N * lay.src[sidx].k_len * 4;
            if (polled >= 256 * 1024 || forced_2d) {
                // row groups of 16 while a workgroup has at most 8 rows; of 4 with more rows, so that
                // the partial sums a workgroup writes and polls per step stay at N * 64 values
                const int rows = lay.ph[0].n_tasks * lay.ph[0].cmax;
                int gj = rows <= 8 ? 16 : 4;
                if (const char* env = std::getenv("RNNG_MSTEP_2D_GROUP")) gj = std::atoi(env);
                size_t lds = 0; int64_t pf = 0;
                std::string src = jit_mstep2_source(plan, cp, backward, N, 256, gj, &lds, &pf);
                if (src.empty() && gj != 16) src = jit_mstep2_source(plan, cp, backward, N, 256, 16, &lds, &pf);
                if (!src.empty()) {
                    c.source = src; c.lp.ok = true; c.lp.G = 256; c.lp.NB = 1; c.lp.lds_bytes = lds; c.lp.xcd_stride = 1;
                    c.two_d = true; c.mstep = true; c.partial_floats = pf;
                }
            }
        }
        if (c.source.empty() && !one_d.source.empty()) c = one_d;
        // 3. LDS-resident variant
        if (c.source.empty() && plan_step_launch(plan.words.data(), backward ? cp.bwd_desc_off : cp.fwd_desc_off, N, force_step_G, c.lp))
            c.source = jit_step_source(plan, cp, backward, c.lp.NB);
        // 4. streaming variant: the weights do not fit on chip at all (wide layers); every step reads them from memory
        try_streaming();
        return jit_choices.emplace(key, c).first->second;
    }
    // floats per frame of the largest partial-sum tensor that a step launch of a window with N streams needs
    int64_t partial_frame_floats(int N) {
        int64_t m = 0;
        if (!use_jit) return 0;
        for (size_t c = 0; c < plan.comps.size(); ++c) {
            const CompPlan& cp = plan.comps[c];
            if (!cp.recurrent) continue;
            for (int backward = 0; backward < 2; ++backward) {
                if (backward ? !cp.has_bwd_program : !cp.has_fwd_program) continue;
                if (cp.chain >= 0 && !chain_choice(cp.chain, backward != 0, N).source.empty()) continue;
                const JitChoice& jc = jit_choice((int)c, backward != 0, N);
                if (jc.two_d) m = std::max(m, jc.partial_floats);
            }
        }
        return m;
    }
    // true if a step launch of a window with N streams reads transposed copies of weight matrices
    bool transposed_copy(int N) {
        if (!use_jit) return false;
        for (size_t c = 0; c < plan.comps.size(); ++c) {
            const CompPlan& cp = plan.comps[c];
            if (!cp.recurrent) continue;
            for (int backward = 0; backward < 2; ++backward) {
                if (backward ? !cp.has_bwd_program : !cp.has_fwd_program) continue;
                if (cp.chain >= 0 && !chain_choice(cp.chain, backward != 0, N).source.empty()) continue;
                if (jit_choice((int)c, backward != 0, N).needs_t) return true;
            }
        }
        return false;
    }
    // Chains of recurrent components run side by side in one launch: all members in the
    // wave-autonomous build (N <= 8, member g on XCD g), or all in the matrix-core build (the 256
    // workgroups shared among the members).
    struct ChainChoice {
        std::string source, source_window; std::vector<int> G, J; bool mstep = false, blocked = false; size_t lds_bytes = 0; int threads = 256;
        bool split = false, backward = false;      // split: the launch with helper members (ChainPlan::fwd_split / bwd_split)
    };
    static const std::vector<CompPlan>& chain_members(const ChainPlan& ch, const ChainChoice& cc) {
        return !cc.split ? ch.members : cc.backward ? ch.bwd_split : ch.fwd_split;
    }
    std::map<std::tuple<int, bool, int>, ChainChoice> chain_choices;
    bool use_chains = true;
    // Weights-in-registers launches: a step is mostly exchange latency, and the helper group reads
    // its sources across XCDs (more than a microsecond per step), so it pays where the multiply-adds
    // and polled sources it takes over weigh enough.  Measured, step kernels forward / backward with
    // against without helper groups: charlm_n1 (128 multiply-adds per lane and step moved) 0.76 / 0.79
    // against 0.81 / 1.21 ms; speech_n1 (32 per lane, 0.9 us per step) 1.11 / 0.91 against 0.93 / 1.04:
    // backward launches (the helper halves the lower layer's sources) from 24 per lane on, forward
    // launches from 100.
    bool wave_helpers_pay(const std::vector<CompPlan>& members, bool backward, int N) const {
        int min_fma = backward ? 24 : 100;
        if (const char* env = std::getenv("RNNG_CHAIN_HELPER_MIN")) min_fma = std::atoi(env);
        for (const CompPlan& m : members)
            if (m.helper && m.step_weight_floats * step_nb_for(N) / (32 * 256) >= min_fma) return true;
        return false;
    }
    const ChainChoice& chain_choice(int chain, bool backward, int N) {
        const std::tuple<int, bool, int> key(chain, backward, N);
        auto it = chain_choices.find(key);
        if (it != chain_choices.end()) return it->second;
        ChainChoice c;
        c.backward = backward;
        const ChainPlan& ch = plan.chains[chain];
        // Helper members take the products of the connections between the stacked nodes
        // (RNNG_CHAIN_HELPERS = 0: never; 1: in every launch that can have them; default: in the
        // matrix-core backward launch and in weights-in-registers launches from RNNG_CHAIN_HELPER_MIN
        // multiply-adds per lane and step on, else from 24 backward / 100 forward)
        const char* envh = std::getenv("RNNG_CHAIN_HELPERS");
        const bool helpers_off = envh && std::atoi(envh) == 0, helpers_all = envh && std::atoi(envh) == 1;
        if (use_jit && use_chains && force_step_G <= 0 && !prefer_streaming) {
            for (int attempt = 0; attempt < 2 && c.source.empty(); ++attempt) {
                c.split = attempt == 0 && !helpers_off && !(backward ? ch.bwd_split : ch.fwd_split).empty();
                if (attempt == 0 && !c.split) continue;
                const std::vector<CompPlan>& members = chain_members(ch, c);
                c.G.clear();
                for (const CompPlan& m : members) {
                    int pick = 0;
                    for (int G : {32, 16, 8})
                        if (!jit_wave_source(plan, m, backward, N, G).empty()) { pick = G; break; }
                    if (!pick) break;
                    c.G.push_back(pick);
                }
                if (c.G.size() == members.size() && (!c.split || helpers_all || wave_helpers_pay(members, backward, N)))
                    c.source = jit_chain_source(plan, members, backward, N, c.G);
            }
            if (c.source.empty()) c.split = false;
            if (c.source.empty() && N > 8 && force_step_J <= 0) {
                // matrix-core members: each gets an equal share of the 256 workgroups; per member the
                // most stream groups, then the most unit chunks that fit the share (as for a single
                // component: fewer only while a workgroup does not fill a 16-row tile)
                // Backward launches of a stack are bound by the matrix instructions of the members that
                // also contract the later member's error terms, while compute units idle: helper members
                // take those products (RNNG_CHAIN_HELPERS = 0: never).
                c.split = backward && !ch.bwd_split.empty() && !helpers_off;
                for (int attempt = 0; attempt < 2 && c.source.empty(); ++attempt) {
                    if (attempt == 1) { if (!c.split) break; c.split = false; }
                    const std::vector<CompPlan>& members = chain_members(ch, c);
                    const int share = std::min(256, max_workgroups()) / (int)members.size();
                    c.G.clear(); c.J.clear();
                    for (const CompPlan& m : members) {
                        int pg = 0, pj = 0, best_rows = -1;
                        for (int J : {4, 2, 1}) {
                            for (int G : {128, 64, 32, 16}) {
                                if (G * J > share) continue;
                                size_t lds = 0; int rows = 0;
                                if (jit_mstep_source(plan, m, backward, N, G, J, &lds, &rows).empty()) continue;
                                if (best_rows < 0 || (best_rows < 16 && rows > best_rows)) { pg = G; pj = J; best_rows = rows; }
                                if (best_rows >= 16) break;
                            }
                            if (pg) break;
                        }
                        if (!pg) break;
                        c.G.push_back(pg); c.J.push_back(pj);
                    }
                    if (c.G.size() == members.size()) {
                        c.source = jit_mstep_chain_source(plan, members, backward, N, c.G, c.J, &c.lds_bytes, &c.threads, &c.blocked);
                        c.mstep = !c.source.empty();
                        if (c.split && !c.blocked) { c.source.clear(); c.mstep = false; }      // (helpers pay only with the tile-blocked exchange's full tiles)
                    }
                }
                if (c.source.empty()) c.split = false;
            }
        }
        return chain_choices.emplace(key, c).first->second;
    }
};

namespace {

// Launches the GEMM problems of one component and direction, grouped by up to
// GEMM_MAX_PROBLEMS destinations per launch and GEMM_MAX_PAIRS products per destination.
// Rows of frames [t0, t1) only.
hipError_t run_gemms(rnn_graph* g, const std::vector<GemmProblemPlan>& probs, bool backward, hipStream_t s, int t0, int t1) {
    // t0, t1: internal frames
    const int64_t F = (int64_t)g->Ti() * g->N, HN = (int64_t)g->hist() * g->N;
    const int64_t r0 = (int64_t)t0 * g->N, rows = (int64_t)(t1 - t0) * g->N;
    if (probs.empty() || rows <= 0) return hipSuccess;
    const int prof = g->prof.begin(backward ? RNN_PROF_GEMM_BWD : RNN_PROF_GEMM_FWD, s);
    int64_t n_launch = 0;
    size_t max_pairs = 0;
    for (const auto& p : probs) max_pairs = p.pairs.size() > max_pairs ? p.pairs.size() : max_pairs;
    for (size_t round = 0; round * GEMM_MAX_PAIRS < max_pairs; ++round) {
        GemmGroup grp; std::memset(&grp, 0, sizeof(grp));
        grp.split_k = 1; grp.accumulate = round > 0;
        auto flush = [&]() -> hipError_t {
            if (grp.n_problems == 0) return hipSuccess;
            // Few output tiles and a long contraction (huge input layers): split the contraction over
            // more workgroups, which add their parts atomically into the zeroed destination.
            int64_t tiles = 0; int kmax = 0;
            for (int i = 0; i < grp.n_problems; ++i) {
                tiles += (int64_t)((grp.p[i].M + 127) / 128) * ((grp.p[i].N + 127) / 128);
                for (int q = 0; q < grp.p[i].n_pairs; ++q) kmax = std::max(kmax, grp.p[i].pairs[q].K);
            }
            int split = 1;
            if (tiles < 256 && !g->deterministic) split = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(16, kmax / 512), (512 + tiles - 1) / tiles));
            grp.split_k = split;
            if (split > 1 && !grp.accumulate)
                for (int i = 0; i < grp.n_problems; ++i) {
                    hipError_t e = launch_fill(grp.p[i].C, (int64_t)grp.p[i].M * grp.p[i].ldc, 0.0f, s);
                    if (e != hipSuccess) return e;
                    ++n_launch;
                }
            hipError_t e = launch_gemm_group(backward ? GEMM_NN : GEMM_NT, grp, s);
            grp.n_problems = 0; ++n_launch;
            return e;
        };
        for (const auto& pp0 : probs) {
            // products with a one-hot source are column gathers, done after the GEMMs (below)
            GemmProblemPlan pp; pp.c_buf = pp0.c_buf; pp.n = pp0.n;
            for (const GemmPairPlan& pr : pp0.pairs) if (!g->is_onehot(pr.a_buf)) pp.pairs.push_back(pr);
            if (pp.pairs.size() <= round * GEMM_MAX_PAIRS) continue;
            GemmProblem& gp = grp.p[grp.n_problems];
            gp.C = g->buf(pp.c_buf) + r0 * pp.n; gp.ldc = pp.n; gp.M = (int)rows; gp.N = pp.n; gp.n_pairs = 0;
            for (size_t q = round * GEMM_MAX_PAIRS; q < pp.pairs.size() && gp.n_pairs < GEMM_MAX_PAIRS; ++q) {
                const GemmPairPlan& pr = pp.pairs[q];
                GemmPair& o = gp.pairs[gp.n_pairs++];
                o.A = g->buf(pr.a_buf); o.B = g->weights + pr.b_w_off; o.K = pr.k_len; o.lda = pr.k_len;
                o.ldb = backward ? pp.n : pr.k_len;
                o.a_row_off = (int)r0 + (backward ? pr.delay : -pr.delay) * g->N; o.a_rows = (int)F;
                // an input read in place has the window's frames only: its row 0 is internal row HN
                if (g->caller_input(pr.a_buf)) { o.a_row_off -= (int)HN; o.a_rows = (int)(F - HN); }
            }
            if (++grp.n_problems == GEMM_MAX_PROBLEMS) { hipError_t e = flush(); if (e != hipSuccess) return e; }
        }
        hipError_t e = flush();
        if (e != hipSuccess) return e;
    }
    if (!backward)
        for (const auto& pp : probs) {
            bool first = true;
            for (const GemmPairPlan& pr : pp.pairs) if (!g->is_onehot(pr.a_buf)) first = false;      // the GEMMs have written C
            for (const GemmPairPlan& pr : pp.pairs) {
                if (!g->is_onehot(pr.a_buf)) continue;
                // the caller's indices [T][N] (row 0 = internal row HN), or, for an input with delayed
                // connections, the library's copy with history frames in front
                const int32_t* hist_idx = g->onehot_history(pr.a_buf);
                hipError_t e = hist_idx ? launch_onehot_gather(g->buf(pp.c_buf), g->weights + pr.b_w_off, hist_idx, pp.n, pr.k_len, r0, rows,
                                                               (int64_t)pr.delay * g->N, F, !first, s)
                                        : launch_onehot_gather(g->buf(pp.c_buf), g->weights + pr.b_w_off, g->onehot[pr.a_buf], pp.n, pr.k_len, r0, rows,
                                                               HN + (int64_t)pr.delay * g->N, F - HN, !first, s);
                if (e != hipSuccess) return e;
                first = false; ++n_launch;
            }
        }
    g->prof.end(prof, n_launch, s);
    return hipSuccess;
}

XcdMap g_xcd_map[64];
bool g_xcd_local = true;       // RNNG_XCD_LOCAL=0: always write exchanged tensors through

// scratch: SYNC_BYTES of device memory that may be overwritten
hipError_t ensure_xcd_map(unsigned* scratch, hipStream_t s, const XcdMap** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    static XcdMap none;
    if (dev < 0 || dev >= 64) { *out = &none; return hipSuccess; }
    XcdMap& m = g_xcd_map[dev];
    if (!m.known) {
        constexpr int NB = (int)(SYNC_BYTES / 4);
        unsigned host[NB];
        e = launch_xcc_probe(scratch, NB, s);
        if (e == hipSuccess) e = hipMemcpyAsync(host, scratch, sizeof(host), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return e;
        m.ok = true;
        for (int r = 0; r < 8; ++r) {
            m.xcc[r] = (int)host[r];
            for (int b = r; b < NB; b += 8) m.ok = m.ok && host[b] == host[r];
        }
        m.known = true;
    }
    *out = &m;
    return hipSuccess;
}

// The wave-autonomous kernels and the matrix-core kernels with weights in LDS address a stored
// tensor through one buffer descriptor with 32-bit offsets and park idle lanes 1 GiB beyond:
// every tensor of the window must stay below 1 GiB.
bool wave_tensor_sizes_ok(const rnn_graph* g) {
    int64_t maxdim = 1;
    for (int b = 0; b < g->plan.n_bufs; ++b) {
        // the caller's input tensors are never stored by a step kernel
        if (!g->caller_input(b)) maxdim = std::max<int64_t>(maxdim, g->plan.buf_dim[b]);
    }
    return (int64_t)g->Ti() * g->N * maxdim * 4 < (int64_t(1) << 30);
}

// The wave-autonomous kernels can store through ONE buffer descriptor when everything they store
// lies in a window of at most 2 GiB: the workspace, if it is that small and holds every tensor
// but the caller's inputs (which no step kernel stores).  The kernel variant is the same source
// behind one definition.
bool wave_store_window_ok(const rnn_graph* g) {
    if (!g->use_store_window || g->layout.total > (int64_t(1) << 31)) return false;
    for (int b = 0; b < g->plan.n_bufs; ++b) {
        if (g->caller_input(b)) continue;
        const char* p = reinterpret_cast<const char*>(g->buf(b));
        if (p == nullptr) continue;      // no storage: never stored
        const int64_t bytes = (int64_t)g->Ti() * g->N * g->plan.buf_dim[b] * 4;
        if (p < g->ws || p + bytes > g->ws + g->layout.total) return false;
    }
    return true;
}
// The matrix-core build also loads its element-wise inputs through the window: every tensor that
// the phases' programs gather from must lie in the workspace too (not in a tensor of the caller).
bool gathers_in_workspace(const rnn_graph* g, const std::vector<PhasePlan>& phases) {
    for (const PhasePlan& ph : phases) {
        const int32_t* pw = g->plan.words.data() + ph.prog_off;
        for (int i = 0; i < pw[PG_NGATHER]; ++i) {
            const int32_t* ga = pw + PG_HEADER_WORDS + i * GA_WORDS;
            if (ga[GA_KIND] == GA_KIND_ACC) continue;
            const char* p = reinterpret_cast<const char*>(g->buf(ga[GA_BUF]));
            if (g->caller_input(ga[GA_BUF]) || p == nullptr || p < g->ws || p >= g->ws + g->layout.total) return false;
        }
    }
    return true;
}
const std::string& windowed(const std::string& source, std::string& cache) {
    if (cache.empty()) cache = "#define RNNG_STORE_WINDOW 1\n" + source;
    return cache;
}

// Sentinel prefill of the tensors that workgroups poll during frames [t0, t1).  The wave-autonomous
// kernel polls the interleaved bundle tensors instead of bundled members; the members are filled as
// well, so that a fall-back to another kernel build finds them prepared.
// A kernel with tile-blocked exchange polls the twins and nothing else.
hipError_t fill_shared(rnn_graph* g, const std::vector<int>& bufs, bool with_bundles, int t0, int t1, hipStream_t s, bool twins = false) {
    std::vector<int> list(bufs);
    if (twins) for (int& b : list) if (g->plan.buf_alloc[g->plan.twin_base + b] == 3) b += g->plan.twin_base;      // (tensors without a twin are polled as they are)
    if (with_bundles)
        for (int b : bufs) {
            const int bi = g->plan.bundle_of[b];
            if (bi >= 0 && std::find(list.begin(), list.end(), g->plan.bundles[bi].ebuf) == list.end()) list.push_back(g->plan.bundles[bi].ebuf);
        }
    FillRanges fr; fr.count = 0;
    for (int b : list) {
        const int64_t frame = (int64_t)g->N * g->plan.buf_dim[b];
        fr.p[fr.count] = g->buf(b) + t0 * frame; fr.n[fr.count] = (t1 - t0) * frame;
        if (++fr.count == FILL_MAX_RANGES) {
            hipError_t e = launch_fill_sentinel_ranges(fr, s);
            if (e != hipSuccess) return e;
            fr.count = 0;
        }
    }
    return launch_fill_sentinel_ranges(fr, s);
}

// The workgroups of a persistent step launch wait for each other's results, so every one that takes
// part must be resident at the same time: at most one per compute unit (each takes most of a CU's
// LDS or registers).  A launch that cannot be co-resident is refused here, before it could hang.
bool launch_fits_device(const rnn_graph* g, int participants, std::string& why) {
    if (participants <= g->max_workgroups()) return true;
    why = "the step kernel needs " + std::to_string(participants) + " co-resident workgroups, the device has " +
          std::to_string(g->max_workgroups()) + " compute units";
    return false;
}

// Result of a step-kernel launch attempt.  A specialised kernel that exists but cannot be compiled,
// loaded or launched is an error (text in `err`), never a silent switch to another build; only
// "there is no such kernel for this component" (or no run-time compiler on this machine) moves on
// to the next build.
struct StepRun { hipError_t e = hipSuccess; bool error = false; int code = RNN_ERR_DEVICE; std::string err; };
StepRun step_error(hipError_t e, const std::string& what, int code = RNN_ERR_DEVICE) {
    StepRun r; r.e = e == hipSuccess ? hipErrorUnknown : e; r.error = true; r.code = code;
    r.err = what + (e != hipSuccess ? std::string(": ") + hipGetErrorString(e) : std::string());
    return r;
}

// t0, t1: internal frames
StepRun run_phases(rnn_graph* g, int comp, bool backward, hipStream_t s, int t0, int t1) {
    const CompPlan& cp = g->plan.comps[comp];
    const PlanView pv = g->view();
    const std::vector<PhasePlan>& phases = backward ? cp.bwd_phases : cp.fwd_phases;
    const int T = g->Ti(), N = g->N;
    StepRun ok;
    if (!cp.recurrent) {
        const int prof = g->prof.begin(RNN_PROF_OTHER, s);
        for (const PhasePlan& ph : phases) {
            hipError_t e = launch_node_program(pv, ph.prog_off, ph.max_dim, g->weights, T, N, t0, t1, s);
            if (e != hipSuccess) return step_error(e, "node program launch");
        }
        g->prof.end(prof, (int64_t)phases.size(), s);
        return ok;
    }
    const int prof = g->prof.begin(backward ? RNN_PROF_STEP_BWD : RNN_PROF_STEP_FWD, s);
    int64_t n_launch = 0;
    int& served = g->served[comp][backward ? 1 : 0];
    // Persistent kernel: all steps in one launch.  First choice is the build specialised at run
    // time for this component; the interpreting build serves components no specialised build
    // takes, or all of them when the run-time compiler is unavailable; stepping with per-frame
    // launches is the last resort.
    StepLaunchPlan lp;
    const int desc_off = backward ? cp.bwd_desc_off : cp.fwd_desc_off;
    rnn_graph::JitChoice* jc = (g->use_jit && jit_available()) ? const_cast<rnn_graph::JitChoice*>(&g->jit_choice(comp, backward, N)) : nullptr;
    const bool have_jit = jc && !jc->source.empty() && !g->framewise &&
                          (!(jc->wave || (jc->mstep && !jc->two_d)) || wave_tensor_sizes_ok(g));
    const bool have_interp = !g->framewise && plan_step_launch(g->plan.words.data(), desc_off, N, g->force_step_G, lp);
    const int spin_limit = g->spin_limit;
    if (have_jit) {
        hipError_t fe = fill_shared(g, backward ? cp.bwd_shared_bufs : cp.fwd_shared_bufs, jc->wave, t0, t1, s, jc->blocked);
        if (fe != hipSuccess) return step_error(fe, "sentinel fill");
        // (matrix-core build: measured per direction; backward loops, with more stores and loads per
        // step, gain 3 %, forward loops lose 4 to 6 %)
        const bool window = (jc->wave || (jc->mstep && !jc->two_d && backward && gathers_in_workspace(g, cp.bwd_phases))) && wave_store_window_ok(g);
        std::string why;
        hipFunction_t fn = jit_step_function(window ? windowed(jc->source, jc->source_window) : jc->source, &why, !g->no_alloc,
                                             jc->mstep && !jc->two_d ? MSTEP_LDS_LIMIT : STEP_LDS_LIMIT);
        if (!fn) return step_error(hipSuccess, "specialised step kernel unavailable: " + why, g->no_alloc ? RNN_ERR_SEQUENCE : RNN_ERR_DEVICE);
        StepArgs a;
        fill_step_args(a, pv, jc->lp, desc_off, g->weights, g->ctrl_ptr(), T, N, backward, spin_limit, t0, t1);
        if (window) { a.store_base = reinterpret_cast<float*>(g->ws); a.store_bytes = (unsigned)g->layout.total; }
        a.J = jc->J;
        a.twin_base = g->plan.twin_base;
        if (jc->two_d) {
            if (g->layout.partial_off < 0) return step_error(hipErrorInvalidValue, "partial-sum tensor missing from the workspace");
            a.partial = reinterpret_cast<float*>(g->ws + g->layout.partial_off);
            hipError_t e = launch_fill_sentinel(a.partial + (int64_t)t0 * jc->partial_floats, (int64_t)(t1 - t0) * jc->partial_floats, s);
            if (e != hipSuccess) return step_error(e, "sentinel fill");
        }
        if (jc->stream) {
            a.weight_bytes = (unsigned)(g->plan.n_params * 4);
            a.weights_t = g->weights;
            if (jc->needs_t) {
                // the matrices this direction reads transposed: a transposed copy at the same offsets, made per launch
                if (g->layout.wt_off < 0) return step_error(hipErrorInvalidValue, "transposed weight copy missing from the workspace");
                float* wt = reinterpret_cast<float*>(g->ws + g->layout.wt_off);
                a.weights_t = wt;
                StepLayout lay;
                compute_step_layout(g->plan.words.data(), desc_off, jc->lp.G, 1, 1, lay);      // (one stream: only the task list is needed)
                if (!lay.ok) return step_error(hipErrorInvalidValue, "step layout of a streaming kernel");
                for (int t = 0; t < lay.ph[0].n_tasks; ++t)
                    for (int e2 = 0; e2 < lay.ph[0].task[t].n_edges; ++e2) {
                        const StepEdge& ed = lay.ph[0].task[t].e[e2];
                        if (!ed.transposed) continue;
                        // stored [k_len][n_out]; the kernel streams rows of [n_out][k_len]
                        hipError_t te = launch_transpose(wt + ed.w_off, g->weights + ed.w_off, ed.k_len, lay.ph[0].task[t].n_out, s);
                        if (te != hipSuccess) return step_error(te, "weight transposition");
                    }
            }
        }
        if (jc->wave && jc->lp.xcd_stride == 8 && g_xcd_local && g->xcd && g->xcd->ok) a.xcc_expect[0] = g->xcd->xcc[0];
        StepLaunchPlan lp_all = jc->lp;
        lp_all.G = jc->lp.G * jc->J;       // launch size; a.G stays the number of unit chunks
        if (!launch_fits_device(g, lp_all.G, why)) return step_error(hipSuccess, why);
        hipError_t e = jit_launch(fn, a, lp_all, s);
        if (e != hipSuccess) { (void)hipGetLastError(); return step_error(e, "specialised step kernel launch"); }
        served = jc->wave ? RNN_BUILD_WAVE : jc->two_d ? RNN_BUILD_MATRIX_2D : jc->stream ? RNN_BUILD_STREAMING : jc->mstep ? RNN_BUILD_MATRIX : RNN_BUILD_LDS;
        g->prof.end(prof, 1, s);
        return ok;
    }
    if (have_interp) {
        std::string why;
        if (!launch_fits_device(g, lp.G, why)) return step_error(hipSuccess, why);
        hipError_t fe = fill_shared(g, backward ? cp.bwd_shared_bufs : cp.fwd_shared_bufs, false, t0, t1, s);
        if (fe != hipSuccess) return step_error(fe, "sentinel fill");
        hipError_t e = launch_recurrent_steps(pv, lp, desc_off, g->weights, g->ctrl_ptr(), T, N, backward, spin_limit, t0, t1, s);
        if (e != hipSuccess) return step_error(e, "interpreting step kernel launch");
        served = RNN_BUILD_INTERPRETED;
        g->prof.end(prof, 1, s);
        return ok;
    }
    for (int step = 0; step < t1 - t0; ++step) {
        const int t = backward ? t1 - 1 - step : t0 + step;
        for (const PhasePlan& ph : phases) {
            if (ph.mv_off >= 0) {
                hipError_t e = launch_step_matvec(pv, ph.mv_off, ph.n_mv_tasks, ph.mv_max_out, g->weights, T, N, t, s);
                if (e != hipSuccess) return step_error(e, "per-frame matrix-vector launch");
                ++n_launch;
            }
            hipError_t e = launch_node_program(pv, ph.prog_off, ph.max_dim, g->weights, T, N, t, t + 1, s);
            if (e != hipSuccess) return step_error(e, "per-frame node program launch");
            ++n_launch;
        }
    }
    served = RNN_BUILD_PER_FRAME;
    g->prof.end(prof, n_launch, s);
    return ok;
}

// All members of a chain in one persistent launch.  e == hipErrorNotSupported without `error`: no
// such kernel for this chain (the caller then runs the members one after another).
StepRun run_chain(rnn_graph* g, int chain, bool backward, hipStream_t s, int t0, int t1) {
    const ChainPlan& ch = g->plan.chains[chain];
    StepRun none; none.e = hipErrorNotSupported;
    if (!g->use_jit || !jit_available()) return none;
    rnn_graph::ChainChoice& cc = const_cast<rnn_graph::ChainChoice&>(g->chain_choice(chain, backward, g->N));
    if (cc.source.empty() || !wave_tensor_sizes_ok(g)) return none;
    bool window = wave_store_window_ok(g) && (!cc.mstep || backward);      // (matrix-core build: backward launches only, as for single components)
    if (cc.mstep && window) for (const CompPlan& m : rnn_graph::chain_members(ch, cc)) window = window && gathers_in_workspace(g, m.bwd_phases);
    std::string why;
    hipFunction_t fn = jit_step_function(window ? windowed(cc.source, cc.source_window) : cc.source, &why, !g->no_alloc,
                                         cc.mstep ? MSTEP_LDS_LIMIT : STEP_LDS_LIMIT);
    if (!fn) return step_error(hipSuccess, "specialised chain step kernel unavailable: " + why, g->no_alloc ? RNN_ERR_SEQUENCE : RNN_ERR_DEVICE);
    const PlanView pv = g->view();
    const int T = g->Ti(), N = g->N;
    const int prof = g->prof.begin(backward ? RNN_PROF_STEP_BWD : RNN_PROF_STEP_FWD, s);
    const std::vector<CompPlan>& members = rnn_graph::chain_members(ch, cc);
    {
        std::vector<int> exchanged;      // of all members: one fill launch
        for (const CompPlan& m : members)
            for (int b : backward ? m.bwd_shared_bufs : m.fwd_shared_bufs) exchanged.push_back(b);
        hipError_t e = fill_shared(g, exchanged, !cc.mstep, t0, t1, s, cc.blocked);
        if (e != hipSuccess) return step_error(e, "sentinel fill");
    }
    StepLaunchPlan lp; lp.ok = true; lp.G = 32; lp.NB = step_nb_for(N); lp.lds_bytes = 0; lp.xcd_stride = 8;
    if (cc.mstep) {
        lp.G = 0; lp.NB = 1; lp.lds_bytes = cc.lds_bytes; lp.xcd_stride = 1; lp.threads = cc.threads;
        for (size_t i = 0; i < cc.G.size(); ++i) lp.G += cc.G[i] * cc.J[i];      // launch size
    }
    StepArgs a;
    fill_step_args(a, pv, lp, backward ? members[0].bwd_desc_off : members[0].fwd_desc_off, g->weights, g->ctrl_ptr(),
                   T, N, backward, g->spin_limit, t0, t1);
    if (window) { a.store_base = reinterpret_cast<float*>(g->ws); a.store_bytes = (unsigned)g->layout.total; }
    a.n_groups = (int)members.size();
    a.twin_base = g->plan.twin_base;
    for (int i = 0; i < a.n_groups; ++i) {
        a.grp_desc_off[i] = backward ? members[i].bwd_desc_off : members[i].fwd_desc_off;
        a.grp_G[i] = cc.G[i];
        if (cc.mstep) {
            a.grp_J[i] = cc.J[i];
            a.grp_first[i] = i == 0 ? 0 : a.grp_first[i - 1] + cc.G[i - 1] * cc.J[i - 1];
        } else if (g_xcd_local && g->xcd && g->xcd->ok) {
            a.xcc_expect[i] = g->xcd->xcc[i];
        }
    }
    int participants = 0;
    for (size_t i = 0; i < cc.G.size(); ++i) participants += cc.G[i] * (cc.mstep ? cc.J[i] : 1);
    if (!launch_fits_device(g, participants, why)) return step_error(hipSuccess, why);
    hipError_t e = jit_launch(fn, a, lp, s);
    if (e != hipSuccess) { (void)hipGetLastError(); return step_error(e, "specialised chain step kernel launch"); }
    for (int c = ch.first; c <= ch.last; ++c) g->served[c][backward ? 1 : 0] = (cc.mstep ? RNN_BUILD_MATRIX : RNN_BUILD_WAVE) | RNN_BUILD_CHAIN | (cc.split ? RNN_BUILD_HELPERS : 0);
    g->prof.end(prof, 1, s);
    StepRun ok;
    return ok;
}

}  // namespace

extern "C" {

const char* rnn_last_error(void) { return g_last_error.c_str(); }

int rnn_graph_create(const rnn_node_desc* nodes, int32_t n_nodes, const rnn_edge_desc* edges, int32_t n_edges,
                     rnn_graph** out) {
    if (!out) return fail(RNN_ERR_INVALID_ARGUMENT, "out is NULL");
    *out = nullptr;
    if (!nodes || n_nodes <= 0 || n_edges < 0 || (n_edges > 0 && !edges))
        return fail(RNN_ERR_INVALID_ARGUMENT, "node / edge list missing");
    std::vector<GNode> ns(n_nodes); std::vector<GEdge> es(n_edges);
    for (int i = 0; i < n_nodes; ++i) ns[i] = GNode{nodes[i].kind, nodes[i].act, nodes[i].dim, nodes[i].has_bias != 0, nodes[i].is_output};
    for (int i = 0; i < n_edges; ++i) es[i] = GEdge{edges[i].src, edges[i].dst, edges[i].delay, edges[i].wkind};
    rnn_graph* g = new (std::nothrow) rnn_graph();
    if (!g) return fail(RNN_ERR_NO_MEMORY, "out of host memory");
    std::string err;
    if (!build_plan(ns, es, g->plan, err)) { delete g; return fail(RNN_ERR_INVALID_GRAPH, err); }
    g->served.assign(g->plan.comps.size(), std::array<int, 2>{0, 0});
    if (const char* env = std::getenv("RNNG_SPIN_LIMIT")) g->spin_limit = std::max(1, std::atoi(env));
    if (const char* env = std::getenv("RNNG_STEP_WORKGROUPS")) g->force_step_G = std::atoi(env);
    if (const char* env = std::getenv("RNNG_STEP_STREAM_GROUPS")) g->force_step_J = std::atoi(env);
    if (const char* env = std::getenv("RNNG_CHAIN")) g->use_chains = std::atoi(env) != 0;
    if (const char* env = std::getenv("RNNG_STEP_BUILD")) g->prefer_streaming = std::string(env) == "stream";
    if (const char* env = std::getenv("RNNG_SCHEDULE")) g->framewise = std::string(env) == "framewise";
    if (const char* env = std::getenv("RNNG_LAYOUT_SKEW")) g_layout_skew = std::atoll(env) / 256 * 256;
    if (const char* env = std::getenv("RNNG_BUNDLE"))
        if (std::atoi(env) == 0) g->plan.bundle_of.assign(g->plan.bundle_of.size(), -1);      // tuning aid: no exchange bundles
    if (const char* env = std::getenv("RNNG_JIT")) g->use_jit = std::atoi(env) != 0;
    if (const char* env = std::getenv("RNNG_STORE_WINDOW")) g->use_store_window = std::atoi(env) != 0;
    {
        const char* env = std::getenv("RNNG_XCD_LOCAL");
        g_xcd_local = env ? std::atoi(env) != 0 : true;
    }
    *out = g;
    return RNN_OK;
}

void rnn_graph_destroy(rnn_graph* g) { delete g; }

int rnn_graph_schedule(const rnn_graph* g, int32_t* node_comp, int32_t* node_level, int32_t* comp_level,
                       int32_t* comp_recurrent, int32_t* edge_class, int32_t* n_comps) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    const Schedule& S = g->plan.sched;
    const int K = (int)g->plan.nodes.size(), M = (int)g->plan.edges.size();
    for (int v = 0; v < K; ++v) {
        if (node_comp) node_comp[v] = S.node_comp[v];
        if (node_level) node_level[v] = S.node_level[v];
        if (comp_level) comp_level[v] = S.comp_level[S.node_comp[v]];
        if (comp_recurrent) comp_recurrent[v] = S.comp_recurrent[S.node_comp[v]];
    }
    if (edge_class) for (int m = 0; m < M; ++m) edge_class[m] = S.edge_class[m];
    if (n_comps) *n_comps = S.n_comps;
    return RNN_OK;
}

int64_t rnn_param_count(const rnn_graph* g) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    return g->plan.n_params;
}

int rnn_edge_param_offset(const rnn_graph* g, int32_t edge, int64_t* off, int64_t* len) {
    if (!g || !off || !len) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (edge < 0 || edge >= (int)g->plan.edges.size()) return fail(RNN_ERR_INVALID_ARGUMENT, "edge index out of range");
    *off = g->plan.edge_off[edge]; *len = g->plan.edge_len[edge];
    return RNN_OK;
}

int rnn_bias_param_offset(const rnn_graph* g, int32_t node, int64_t* off, int64_t* len) {
    if (!g || !off || !len) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (node < 0 || node >= (int)g->plan.nodes.size()) return fail(RNN_ERR_INVALID_ARGUMENT, "node index out of range");
    *off = g->plan.bias_off[node]; *len = g->plan.bias_len[node];
    return RNN_OK;
}

int64_t rnn_workspace_bytes(const rnn_graph* g, int32_t T, int32_t N) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (T <= 0 || N <= 0) return fail(RNN_ERR_INVALID_ARGUMENT, "T and N must be positive");
    if ((int64_t)(T + g->plan.hist) * N >= (int64_t(1) << 31)) return fail(RNN_ERR_INVALID_ARGUMENT, "T * N exceeds 2^31 - 1");
    return make_layout(g->plan, T, N, const_cast<rnn_graph*>(g)->partial_frame_floats(N), const_cast<rnn_graph*>(g)->transposed_copy(N)).total;
}

namespace {

// Waits for the stream, then reads the control words of the current window: E_total (to *loss if
// given) and the flags the kernels raise.  A raised flag means the window's results are invalid.
int read_control(rnn_graph* g, double* loss, hipStream_t s) {
    unsigned char back[32];
    hipError_t e = hipMemcpyAsync(back, g->loss_ptr(), sizeof(back), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail_hip(e, "control word read-back");
    if (loss) std::memcpy(loss, back, sizeof(double));
    unsigned flag; std::memcpy(&flag, back + 16, 4);
    if (flag == 3) return fail(RNN_ERR_INVALID_ARGUMENT, "a target class index is not below the output layer's width (that frame was left out)");
    if (flag == 2) return fail(RNN_ERR_DEVICE, "a recurrent step kernel's workgroup ran on another XCD than the probe launch had shown (results are invalid; RNNG_XCD_LOCAL=0 avoids the assumption)");
    if (flag) return fail(RNN_ERR_DEVICE, "a recurrent step kernel ran into its wait limit (results are invalid)");
    return RNN_OK;
}

// Forward pass over internal frames [t0, t1) of the current window: components in schedule order.
int forward_frames(rnn_graph* g, int t0, int t1, hipStream_t s) {
    const Plan& P = g->plan;
    const int N = g->N;
    hipError_t e;
    int chain_done_to = -1;   // components up to this index were run as a chain
    for (const CompPlan& cp : P.comps) {
        if (!cp.has_fwd_program) continue;
        const int c = (int)(&cp - P.comps.data());
        if (c <= chain_done_to) continue;
        if (!g->framewise && cp.chain >= 0 && P.chains[cp.chain].first == c && !g->chain_choice(cp.chain, false, N).source.empty()) {
            const ChainPlan& ch = P.chains[cp.chain];
            for (const CompPlan& m : ch.members) {
                e = run_gemms(g, m.fwd_gemms, false, s, t0, t1);
                if (e != hipSuccess) return fail_hip(e, "forward GEMM");
            }
            const StepRun r = run_chain(g, cp.chain, false, s, t0, t1);
            if (r.error) return fail(r.code, "forward: " + r.err);
            if (r.e == hipSuccess) { chain_done_to = ch.last; continue; }
        }
        e = run_gemms(g, cp.fwd_gemms, false, s, t0, t1);
        if (e != hipSuccess) return fail_hip(e, "forward GEMM");
        const StepRun r = run_phases(g, c, false, s, t0, t1);
        if (r.error) return fail(r.code, "forward: " + r.err);
        if (cp.softmax_node >= 0) {
            const int dim = P.xnodes[cp.softmax_node].dim;
            e = launch_softmax_rows(g->buf(P.ybuf(cp.softmax_node)) + (int64_t)t0 * N * dim, (int64_t)(t1 - t0) * N, dim, s);
            if (e != hipSuccess) return fail_hip(e, "softmax");
        }
    }
    return RNN_OK;
}

}  // namespace

int rnn_forward_range(rnn_graph* g, const float* d_weights, const float* const* d_inputs, int32_t T, int32_t N,
                      int32_t t_begin, int32_t t_end, void* d_workspace, int64_t ws_bytes, void* hip_stream) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (!d_weights || !d_inputs) return fail(RNN_ERR_INVALID_ARGUMENT, "weights / inputs pointer is NULL");
    if (T <= 0 || N <= 0) return fail(RNN_ERR_INVALID_ARGUMENT, "T and N must be positive");
    if ((int64_t)(T + g->plan.hist) * N >= (int64_t(1) << 31)) return fail(RNN_ERR_INVALID_ARGUMENT, "T * N exceeds 2^31 - 1");
    if (t_begin < 0 || t_end > T || t_begin >= t_end) return fail(RNN_ERR_INVALID_ARGUMENT, "frame range must satisfy 0 <= t_begin < t_end <= T");
    const Plan& P = g->plan;
    for (size_t i = 0; i < P.input_nodes.size(); ++i)
        if (!d_inputs[i] && !g->is_onehot(P.input_nodes[i])) return fail(RNN_ERR_INVALID_ARGUMENT, "an input tensor pointer is NULL");
    if (!d_workspace) return fail(RNN_ERR_WORKSPACE, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255) return fail(RNN_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (ws_bytes < make_layout(P, T, N, g->partial_frame_floats(N), g->transposed_copy(N)).total)
        return fail(RNN_ERR_WORKSPACE, "workspace too small: need " + std::to_string(make_layout(P, T, N, g->partial_frame_floats(N), g->transposed_copy(N)).total) + " bytes");
    if (g->cu_count == 0) {
        // The step kernels' launch shapes depend on how many workgroups the device keeps resident.
        int dev = 0, cus = 0;
        hipError_t qe = hipGetDevice(&dev);
        if (qe == hipSuccess) qe = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (qe != hipSuccess || cus <= 0) return fail_hip(qe, "device query");
        if (cus != g->max_workgroups()) { g->jit_choices.clear(); g->chain_choices.clear(); }      // chosen for a whole device
        g->cu_count = cus;
    }
    Layout L = make_layout(P, T, N, g->partial_frame_floats(N), g->transposed_copy(N));
    if (ws_bytes < L.total) return fail(RNN_ERR_WORKSPACE, "workspace too small: need " + std::to_string(L.total) + " bytes");
    if (t_begin > 0) {
        // the earlier frames must be there: same window shape and workspace, computed up to t_begin
        if (g->ws != static_cast<char*>(d_workspace) || g->T != T || g->N != N || g->fwd_upto < t_begin)
            return fail(RNN_ERR_SEQUENCE, "frames before t_begin have not been computed in this workspace");
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    g->fwd_done = g->bptt_done = false;

    g->T = T; g->N = N; g->ws = static_cast<char*>(d_workspace); g->layout = L; g->weights = d_weights;
    g->inputs.assign(P.xnodes.size(), nullptr);
    for (size_t i = 0; i < P.input_nodes.size(); ++i) g->inputs[P.input_nodes[i]] = d_inputs[i];

    // plan tables: buffer pointers, widths, program words
    g->blob.assign(L.blob_bytes, 0);
    for (int b = 0; b < P.n_bufs; ++b) {
        float* p = g->buf(b);
        std::memcpy(&g->blob[L.table_off + 8 * (int64_t)b], &p, 8);
    }
    std::memcpy(&g->blob[L.dims_off], P.buf_dim.data(), (size_t)P.n_bufs * 4);
    for (int b = 0; b < P.n_bufs; ++b) {
        const int32_t flag = ((P.buf_alloc[b] == 1 || P.buf_alloc[b] == 3) && L.buf_off[b] >= 0) ? 1 : 0;
        std::memcpy(&g->blob[L.flags_off + 4 * (int64_t)b], &flag, 4);
    }
    if (!P.words.empty()) std::memcpy(&g->blob[L.words_off], P.words.data(), P.words.size() * 4);
    // (without allocations: as kernel arguments, which need no staging buffer of the runtime's)
    hipError_t e = g->no_alloc ? launch_upload_words(reinterpret_cast<uint32_t*>(g->ws), reinterpret_cast<const uint32_t*>(g->blob.data()), L.blob_bytes / 4, s)
                               : hipMemcpyAsync(g->ws, g->blob.data(), (size_t)L.blob_bytes, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return fail_hip(e, "plan table upload");
    if (!g->xcd) {
        e = ensure_xcd_map(reinterpret_cast<unsigned*>(g->ws + L.sync_off), s, &g->xcd);
        if (e != hipSuccess) return fail_hip(e, "XCD probe");
    }
    const int H = P.hist;
    if (t_begin == 0) {
        // A new window: the control words (loss, error flags) start at zero, and so do the history
        // frames in front of every frame tensor (the state before a fresh window is zero).  Pieces
        // of a window computed later keep the flags an earlier piece has raised.
        e = launch_fill(reinterpret_cast<float*>(g->ws + L.sync_off), SYNC_BYTES / 4, 0.0f, s);
        if (e != hipSuccess) return fail_hip(e, "control word reset");
        if (H > 0) {
            e = launch_zero_history(g->view().buf_ptr, g->view().buf_dim, reinterpret_cast<const int32_t*>(g->ws + L.flags_off), P.n_bufs, (int64_t)H * N, s);
            if (e != hipSuccess) return fail_hip(e, "history reset");
        }
    }
    // one-hot inputs with delayed connections: their class indices likewise (-1, the zero vector, in a fresh window's history)
    for (size_t i = 0; i < P.input_nodes.size(); ++i) {
        const int k = P.input_nodes[i];
        int32_t* hist_idx = g->is_onehot(k) ? g->onehot_history(k) : nullptr;
        if (!hist_idx) continue;
        if (t_begin == 0 && H > 0) {
            e = launch_fill_sentinel(reinterpret_cast<float*>(hist_idx), (int64_t)H * N, s);      // all bits set = -1
            if (e != hipSuccess) return fail_hip(e, "index history reset");
        }
        e = hipMemcpyAsync(hist_idx + (int64_t)(H + t_begin) * N, g->onehot[k] + (int64_t)t_begin * N, (size_t)(t_end - t_begin) * N * sizeof(int32_t),
                           hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail_hip(e, "index copy");
    }
    // inputs that are not read in place: the new frames go behind the history frames of their copy
    for (size_t i = 0; i < P.input_nodes.size(); ++i) {
        const int k = P.input_nodes[i];
        if (!P.input_staged[k] || g->is_onehot(k)) continue;
        const int64_t fr = (int64_t)N * P.xnodes[k].dim;
        e = hipMemcpyAsync(g->buf(P.ybuf(k)) + (int64_t)(H + t_begin) * fr, d_inputs[i] + (int64_t)t_begin * fr,
                           (size_t)(t_end - t_begin) * fr * sizeof(float), hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail_hip(e, "input copy");
    }

    if (g->framewise) {
        for (int t = t_begin; t < t_end; ++t) {
            const int rc = forward_frames(g, H + t, H + t + 1, s);
            if (rc != RNN_OK) return rc;
        }
    } else {
        const int rc = forward_frames(g, H + t_begin, H + t_end, s);
        if (rc != RNN_OK) return rc;
    }
    g->fwd_upto = t_end;
    g->fwd_done = t_end == T;
    return RNN_OK;
}

int rnn_forward(rnn_graph* g, const float* d_weights, const float* const* d_inputs, int32_t T, int32_t N,
                void* d_workspace, int64_t ws_bytes, void* hip_stream) {
    return rnn_forward_range(g, d_weights, d_inputs, T, N, 0, T, d_workspace, ws_bytes, hip_stream);
}

// ---- rnn_forward_static: the workspace of callers that cannot allocate -----------------------
namespace {
// Part of the library image: every GPU the library runs on holds its own copy of this array, at
// its own address, until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; all device work goes through the address that call returns.
static __device__ __align__(256) unsigned char scratch[RNN_STATIC_WORKSPACE_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
void* g_scratch_ptr[STATIC_MAX_DEVICES];      // per device: address of that GPU's copy (nullptr: not asked yet)
std::mutex g_scratch_mutex;
}  // namespace

int rnn_forward_static(rnn_graph* g, const float* d_weights, const float* const* d_inputs, float* const* d_outputs,
                       int32_t T, int32_t N, void* hip_stream) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (!d_outputs) return fail(RNN_ERR_INVALID_ARGUMENT, "outputs pointer is NULL");
    const Plan& P = g->plan;
    for (size_t i = 0; i < P.output_nodes.size(); ++i)
        if (!d_outputs[i]) return fail(RNN_ERR_INVALID_ARGUMENT, "an output tensor pointer is NULL");
    if (T <= 0 || N <= 0) return fail(RNN_ERR_INVALID_ARGUMENT, "T and N must be positive");
    if (g->prof.mask != 0) return fail(RNN_ERR_SEQUENCE, "kernel-class timing creates events: switch it off for rnn_forward_static");
    const int64_t need = make_layout(P, T, N, g->partial_frame_floats(N), g->transposed_copy(N)).total;
    if (need > (int64_t)RNN_STATIC_WORKSPACE_BYTES)
        return fail(RNN_ERR_WORKSPACE, "the window needs " + std::to_string(need) + " bytes of workspace, the static workspace holds " +
                                           std::to_string((int64_t)RNN_STATIC_WORKSPACE_BYTES));
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(RNN_ERR_DEVICE, "device index beyond the static workspace table");
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            // once per device, with that device current: where this GPU keeps its copy of the array
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return fail_hip(e, "hipGetSymbolAddress(static workspace)");
            g_scratch_ptr[dev] = p;
        }
        ws = g_scratch_ptr[dev];
    }
    g->no_alloc = true;
    const int rc = rnn_forward_range(g, d_weights, d_inputs, T, N, 0, T, ws, RNN_STATIC_WORKSPACE_BYTES, hip_stream);
    g->no_alloc = false;
    if (rc != RNN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    for (size_t i = 0; i < P.output_nodes.size(); ++i) {
        const int k = P.output_nodes[i];
        e = launch_copy(d_outputs[i], g->frame0(P.ybuf(k)), (int64_t)T * N * P.nodes[k].dim, s);
        if (e != hipSuccess) return fail_hip(e, "output copy");
    }
    return RNN_OK;
}

int rnn_set_onehot_input(rnn_graph* g, int32_t input, const int32_t* d_indices) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    const Plan& P = g->plan;
    if (input < 0 || input >= (int)P.input_nodes.size()) return fail(RNN_ERR_INVALID_ARGUMENT, "input index out of range");
    const int k = P.input_nodes[input];
    if (d_indices)
        for (const GEdge& e : P.xedges)
            if (e.src == k && e.wkind != W_FULL)
                return fail(RNN_ERR_INVALID_ARGUMENT, "a one-hot input may only have full connections");
    g->onehot.resize(P.xnodes.size(), nullptr);
    g->onehot[k] = d_indices;
    g->fwd_done = g->bptt_done = false; g->fwd_upto = 0;
    return RNN_OK;
}

int rnn_shift_window(rnn_graph* g, int32_t frames, void* hip_stream) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (!g->ws || g->fwd_upto != g->T) return fail(RNN_ERR_SEQUENCE, "rnn_shift_window needs a completely computed window");
    if (frames <= 0 || frames >= g->T) return fail(RNN_ERR_INVALID_ARGUMENT, "frames must lie in [1, T - 1]");
    const Plan& P = g->plan;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int Ti = g->Ti();
    // y(t) <- y(t + frames) for every stored frame, the history frames in front of the window
    // included: they then hold the frames right before the new window start.  Block by block in
    // stream order, so that source and destination of one copy never overlap.
    auto shift = [&](int b) -> hipError_t {
        const int64_t fr = (int64_t)g->N * P.buf_dim[b];
        float* y = g->buf(b);
        for (int t = 0; t + frames < Ti; t += frames) {
            const int n = std::min(frames, Ti - frames - t);
            hipError_t e = hipMemcpyAsync(y + t * fr, y + (t + frames) * fr, (size_t)n * fr * sizeof(float), hipMemcpyDeviceToDevice, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    };
    for (size_t k = 0; k < P.xnodes.size(); ++k) {
        const int b = P.ybuf((int)k);
        if (g->layout.buf_off[b] < 0) continue;      // an input read in place: the caller shifts it
        hipError_t e = shift(b);
        if (e != hipSuccess) return fail_hip(e, "window shift");
        if (P.twin_base >= 0 && g->layout.buf_off[P.twin_base + b] >= 0) {      // its tile-blocked twin has the same frame size
            e = shift(P.twin_base + b);
            if (e != hipSuccess) return fail_hip(e, "window shift");
        }
    }
    for (size_t k = 0; k < P.xnodes.size(); ++k) {
        int32_t* hist_idx = g->is_onehot((int)k) ? g->onehot_history((int)k) : nullptr;
        if (!hist_idx) continue;
        const int64_t fr = g->N;
        for (int t = 0; t + frames < Ti; t += frames) {
            const int n = std::min(frames, Ti - frames - t);
            hipError_t e = hipMemcpyAsync(hist_idx + t * fr, hist_idx + (t + frames) * fr, (size_t)n * fr * sizeof(int32_t), hipMemcpyDeviceToDevice, s);
            if (e != hipSuccess) return fail_hip(e, "window shift");
        }
    }
    // interleaved exchange tensors of forward activations move along with their members
    for (const BundlePlan& bp : P.bundles) {
        if (bp.members[0] >= (int)P.xnodes.size() || g->layout.buf_off[bp.ebuf] < 0) continue;
        hipError_t e = shift(bp.ebuf);
        if (e != hipSuccess) return fail_hip(e, "window shift");
    }
    g->fwd_upto = g->T - frames;
    g->fwd_done = g->bptt_done = false;
    return RNN_OK;
}

int rnn_output(const rnn_graph* g, int32_t node, const float** d_y) {
    if (!g || !d_y) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (node < 0 || node >= (int)g->plan.nodes.size()) return fail(RNN_ERR_INVALID_ARGUMENT, "node index out of range");
    if (!g->fwd_done) return fail(RNN_ERR_SEQUENCE, "rnn_output before rnn_forward");
    const int b = g->plan.ybuf(node);
    *d_y = g->plan.nodes[node].kind == NODE_INPUT ? g->inputs[b] : g->frame0(b);
    return RNN_OK;
}

int rnn_bptt(rnn_graph* g, const float* d_weights, const void* const* d_targets, void* hip_stream) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (!g->fwd_done) return fail(RNN_ERR_SEQUENCE, "rnn_bptt before rnn_forward");
    g->bptt_done = false;
    if (!d_weights || !d_targets) return fail(RNN_ERR_INVALID_ARGUMENT, "weights / targets pointer is NULL");
    const Plan& P = g->plan;
    for (size_t i = 0; i < P.output_nodes.size(); ++i)
        if (!d_targets[i]) return fail(RNN_ERR_INVALID_ARGUMENT, "a target tensor pointer is NULL");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    g->weights = d_weights;
    const int T = g->T, N = g->N, H = g->hist();
    hipError_t e = launch_fill(reinterpret_cast<float*>(g->loss_ptr()), 2, 0.0f, s);
    if (e != hipSuccess) return fail_hip(e, "loss reset");
    // the output deltas of all frames first (they depend on the forward pass only)
    for (const CompPlan& cp : P.comps) {
        const int k = cp.softmax_node >= 0 ? cp.softmax_node : cp.sqerr_node;
        if (k < 0) continue;
        size_t oi = 0;
        while (oi < P.output_nodes.size() && P.output_nodes[oi] != k) ++oi;
        if (cp.softmax_node >= 0)
            e = launch_softmax_ce_delta(g->frame0(P.ybuf(k)), static_cast<const int32_t*>(d_targets[oi]), g->frame0(P.dbuf(k)), g->loss_ptr(),
                                        g->ctrl_ptr(), (int64_t)T * N, P.xnodes[k].dim, s);
        else
            e = launch_squared_error_delta(g->frame0(P.ybuf(k)), static_cast<const float*>(d_targets[oi]), g->frame0(P.dbuf(k)), g->loss_ptr(),
                                           (int64_t)T * N * P.xnodes[k].dim, P.xnodes[k].act, s);
        if (e != hipSuccess) return fail_hip(e, "output delta");
    }
    auto backward_frames = [&](int t0, int t1) -> int {
        for (int c = (int)P.comps.size() - 1; c >= 0; --c) {
            const CompPlan& cp = P.comps[c];
            if (cp.softmax_node >= 0 || cp.sqerr_node >= 0 || !cp.has_bwd_program) continue;
            if (!g->framewise && cp.chain >= 0 && P.chains[cp.chain].last == c && !g->chain_choice(cp.chain, true, N).source.empty()) {
                const ChainPlan& ch = P.chains[cp.chain];
                for (const CompPlan& m : ch.members) {
                    e = run_gemms(g, m.bwd_gemms, true, s, t0, t1);
                    if (e != hipSuccess) return fail_hip(e, "backward GEMM");
                }
                const StepRun r = run_chain(g, cp.chain, true, s, t0, t1);
                if (r.error) return fail(RNN_ERR_DEVICE, "backward: " + r.err);
                if (r.e == hipSuccess) { c = ch.first; continue; }
            }
            e = run_gemms(g, cp.bwd_gemms, true, s, t0, t1);
            if (e != hipSuccess) return fail_hip(e, "backward GEMM");
            const StepRun r = run_phases(g, c, true, s, t0, t1);
            if (r.error) return fail(RNN_ERR_DEVICE, "backward: " + r.err);
        }
        return RNN_OK;
    };
    // Errors are back-propagated through the window's own frames only (Section 2.2: while t > t0');
    // the history frames in front are read (y of earlier frames), never written.
    if (g->framewise) {
        for (int t = T - 1; t >= 0; --t) {
            const int rc = backward_frames(H + t, H + t + 1);
            if (rc != RNN_OK) return rc;
        }
    } else {
        const int rc = backward_frames(H, H + T);
        if (rc != RNN_OK) return rc;
    }
    g->bptt_done = true;
    return RNN_OK;
}

int rnn_state_grad(const rnn_graph* g, int32_t node, const float** d_ds) {
    if (!g || !d_ds) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (node < 0 || node >= (int)g->plan.nodes.size()) return fail(RNN_ERR_INVALID_ARGUMENT, "node index out of range");
    if (g->plan.nodes[node].kind == NODE_INPUT) return fail(RNN_ERR_INVALID_ARGUMENT, "input nodes have no state gradient");
    if (!g->bptt_done) return fail(RNN_ERR_SEQUENCE, "rnn_state_grad before rnn_bptt");
    *d_ds = g->frame0(g->plan.dbuf(node));
    return RNN_OK;
}

int rnn_grads(rnn_graph* g, float* d_grads, double* loss, void* hip_stream) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (!g->bptt_done) return fail(RNN_ERR_SEQUENCE, "rnn_grads before rnn_bptt");
    if (!d_grads) return fail(RNN_ERR_INVALID_ARGUMENT, "gradient pointer is NULL");
    const Plan& P = g->plan;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int T = g->T, N = g->N, H = g->hist();
    const int64_t F = (int64_t)T * N;      // the window's own frames: the sums run over t0' < t <= t1
    hipError_t e = launch_fill(d_grads, P.n_params, 0.0f, s);
    if (e != hipSuccess) return fail_hip(e, "gradient reset");

    // Weight-gradient GEMMs: the contraction runs over frames, split over blockIdx.z.
    GemmGroup grp; std::memset(&grp, 0, sizeof(grp));
    int64_t tiles = 0, n_launch = 0;
    const int prof = g->prof.begin(RNN_PROF_GEMM_GRAD, s);
    auto flush = [&]() -> hipError_t {
        if (grp.n_problems == 0) return hipSuccess;
        ++n_launch;
        int split = (int)((1024 + tiles - 1) / tiles);
        const int max_split = (int)((F + 127) / 128);
        if (split > max_split) split = max_split;
        if (split < 1 || g->deterministic) split = 1;
        // split_k > 1 adds atomically into the zeroed buffer; split_k == 1 must add too (accumulate)
        grp.split_k = split; grp.accumulate = 1;
        hipError_t r = launch_gemm_group(GEMM_TN, grp, s);
        grp.n_problems = 0; tiles = 0;
        return r;
    };
    for (const GradGemmPlan& gg : P.grad_gemms) {
        if (g->is_onehot(gg.src_buf)) {      // scatter-add instead of a GEMM over a one-hot matrix
            if (const int32_t* hist_idx = g->onehot_history(gg.src_buf)) {
                // every frame of the window against the class of frame t - d, which may lie in the history
                e = launch_onehot_scatter(d_grads + gg.w_off, g->frame0(gg.dst_buf), hist_idx + (int64_t)(H - gg.delay) * N, gg.n_dst, gg.n_src, 0, F,
                                          g->deterministic, s);
            } else {
                if (F - (int64_t)gg.delay * N <= 0) continue;
                e = launch_onehot_scatter(d_grads + gg.w_off, g->frame0(gg.dst_buf), g->onehot[gg.src_buf], gg.n_dst, gg.n_src, (int64_t)gg.delay * N, F,
                                          g->deterministic, s);
            }
            if (e != hipSuccess) return fail_hip(e, "one-hot weight gradient");
            ++n_launch;
            continue;
        }
        GemmProblem& gp = grp.p[grp.n_problems];
        gp.C = d_grads + gg.w_off; gp.ldc = gg.n_src; gp.M = gg.n_dst; gp.N = gg.n_src; gp.n_pairs = 1;
        GemmPair& o = gp.pairs[0];
        // eps_m(t) of every frame of the window against y_src(t - d); for the window's first d
        // frames that is a history frame (the real activation of a frame before the window)
        o.A = g->frame0(gg.dst_buf); o.lda = gg.n_dst;
        o.B = g->frame0(gg.src_buf) - (int64_t)gg.delay * N * gg.n_src; o.ldb = gg.n_src; o.K = (int)F; o.a_row_off = 0; o.a_rows = (int)F;
        tiles += (int64_t)((gg.n_dst + 127) / 128) * ((gg.n_src + 127) / 128);
        if (++grp.n_problems == GEMM_MAX_PROBLEMS) { e = flush(); if (e != hipSuccess) return fail_hip(e, "gradient GEMM"); }
    }
    e = flush();
    if (e != hipSuccess) return fail_hip(e, "gradient GEMM");
    g->prof.end(prof, n_launch, s);
    e = launch_colsum(g->view(), P.colsum_off, P.n_colsum, P.colsum_max_dim, g->weights, d_grads, H + T, N, H, g->deterministic, s);
    if (e != hipSuccess) return fail_hip(e, "diagonal / bias gradient");
    if (loss) return read_control(g, loss, s);
    return RNN_OK;
}

int rnn_set_deterministic(rnn_graph* g, int32_t on) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    g->deterministic = on != 0;
    return RNN_OK;
}

int rnn_check(rnn_graph* g, void* hip_stream) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (!g->ws) return fail(RNN_ERR_SEQUENCE, "no window yet");
    return read_control(g, nullptr, static_cast<hipStream_t>(hip_stream));
}

int rnn_step_build(const rnn_graph* g, int32_t node, int32_t backward, int32_t* build) {
    if (!g || !build) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (node < 0 || node >= (int)g->plan.nodes.size()) return fail(RNN_ERR_INVALID_ARGUMENT, "node index out of range");
    const int c = g->plan.xsched.node_comp[node];
    *build = g->plan.comps[c].recurrent ? g->served[c][backward ? 1 : 0] : RNN_BUILD_NONE;
    return RNN_OK;
}

int rnn_specialise(rnn_graph* g, int32_t N) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (N <= 0) return fail(RNN_ERR_INVALID_ARGUMENT, "N must be positive");
    if (!g->use_jit || !jit_available()) return 0;
    int n = 0;
    for (size_t c = 0; c < g->plan.comps.size(); ++c) {
        const CompPlan& cp = g->plan.comps[c];
        if (!cp.recurrent) continue;
        for (int backward = 0; backward < 2; ++backward) {
            if (backward ? !cp.has_bwd_program : !cp.has_fwd_program) continue;
            std::string log;
            const rnn_graph::JitChoice& jc = g->jit_choice((int)c, backward != 0, N);
            if (jc.source.empty()) continue;
            if (!jit_compile(jc.source, &log))
                return fail(RNN_ERR_DEVICE, "step kernel specialisation failed: " + log);
            ++n;
        }
    }
    for (size_t ci = 0; ci < g->plan.chains.size(); ++ci)
        for (int backward = 0; backward < 2; ++backward) {
            const rnn_graph::ChainChoice& cc = g->chain_choice((int)ci, backward != 0, N);
            if (cc.source.empty()) continue;
            std::string log;
            if (!jit_compile(cc.source, &log))
                return fail(RNN_ERR_DEVICE, "chain step kernel specialisation failed: " + log);
            ++n;
        }
    return n;
}

int rnn_plan_work(const rnn_graph* g, int32_t T, int32_t N, int64_t* flops, int64_t* step_bytes) {
    if (!g || !flops || !step_bytes) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (T <= 0 || N <= 0) return fail(RNN_ERR_INVALID_ARGUMENT, "T and N must be positive");
    const Plan& P = g->plan;
    const int64_t F = (int64_t)T * N;
    for (int i = 0; i < 5; ++i) flops[i] = 0;
    step_bytes[0] = step_bytes[1] = 0;
    // diagonal weights inside recurrent nodes (peepholes) are touched once per step as well
    std::vector<int64_t> diag(P.comps.size(), 0);
    for (size_t m = 0; m < P.xedges.size(); ++m)
        if (P.xedges[m].wkind == W_DIAG && P.xsched.edge_class[m] != EDGE_BATCHED)
            diag[P.xsched.node_comp[P.xedges[m].dst]] += P.xnodes[P.xedges[m].dst].dim;
    for (size_t c = 0; c < P.comps.size(); ++c) {
        for (int d = 0; d < 2; ++d) {
            // the lowering that ran: as a member of a chain launch, or on its own
            const CompPlan* cp = &P.comps[c];
            if (cp->chain >= 0 && (g->served[c][d] & RNN_BUILD_CHAIN)) cp = &P.chains[cp->chain].members[c - P.chains[cp->chain].first];
            for (const GemmProblemPlan& gp : d ? cp->bwd_gemms : cp->fwd_gemms)
                for (const GemmPairPlan& pr : gp.pairs)
                    if (!g->is_onehot(pr.a_buf)) flops[d] += 2 * (int64_t)gp.n * pr.k_len * F;
            if (cp->recurrent) {
                flops[3 + d] += 2 * cp->step_weight_floats * F;
                step_bytes[d] += 4 * (cp->step_weight_floats + diag[c]);
            }
        }
    }
    for (const GradGemmPlan& gg : P.grad_gemms)
        if (!g->is_onehot(gg.src_buf)) flops[2] += 2 * (int64_t)gg.n_dst * gg.n_src * F;
    return RNN_OK;
}

int rnn_debug_read_control(rnn_graph* g, void* out, int32_t bytes) {
    if (!g || !out) return fail(RNN_ERR_INVALID_ARGUMENT, "NULL argument");
    if (!g->ws) return fail(RNN_ERR_SEQUENCE, "no window yet");
    if (bytes <= 0 || bytes > (int32_t)SYNC_BYTES) return fail(RNN_ERR_INVALID_ARGUMENT, "at most 1024 bytes");
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(out, g->ws + g->layout.sync_off, (size_t)bytes, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(e, "control word read-back");
    return RNN_OK;
}

int rnn_profile_enable(rnn_graph* g, int32_t class_mask) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    g->prof.mask = class_mask & ((1 << RNN_PROF_CLASSES) - 1);
    return RNN_OK;
}

int rnn_profile_read(rnn_graph* g, int32_t cls, double* ms, int64_t* launches) {
    if (!g) return fail(RNN_ERR_INVALID_ARGUMENT, "graph is NULL");
    if (cls < 0 || cls >= RNN_PROF_CLASSES) return fail(RNN_ERR_INVALID_ARGUMENT, "unknown kernel class");
    double total = 0.0; int64_t n = 0;
    std::vector<Profiler::Rec> keep;
    for (Profiler::Rec& r : g->prof.recs) {
        if (r.cls != cls) { keep.push_back(r); continue; }
        hipError_t e = hipEventSynchronize(r.b);
        float t = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
        g->prof.pool.push_back(r.a); g->prof.pool.push_back(r.b);
        if (e != hipSuccess) { g->prof.recs.swap(keep); return fail_hip(e, "event read"); }
        total += t; n += r.launches;
    }
    g->prof.recs.swap(keep);
    if (ms) *ms = total;
    if (launches) *launches = n;
    return RNN_OK;
}

}  // extern "C"
