// LDS layout of the persistent recurrent-step kernel, computed identically on the host (to
// size the launch and to decide whether a component fits) and on the device.
//
// A component's step descriptor is [n_phases, (mv_off, prog_off) x n_phases] in the plan words.
// G workgroups each own a contiguous chunk of every layer's units.  Per phase, the
// matrix-vector work of a workgroup is a set of output slots, slot = task * cmax + local unit,
// each served by L consecutive lanes that split the contraction; a lane's weights are stored
// lane-major ([edge][j][thread][4 floats]) so every ds_read_b128 of a wavefront is contiguous.
#pragma once
#if !defined(__HIPCC_RTC__)
#include <cstdint>
#endif

#include "program.h"

#if defined(__HIPCC__) || defined(__HIPCC_RTC__)
#define RNNG_HD __host__ __device__
#else
#define RNNG_HD
#endif

namespace rnng {

constexpr int STEP_THREADS = 256;
constexpr unsigned STEP_LDS_LIMIT = 148 * 1024;   // dynamic LDS per workgroup (the static tables take 11.3 KiB of the 160 KiB)
constexpr unsigned MSTEP_LDS_LIMIT = 152 * 1024;  // the same for the matrix-core variant with weights in LDS (tables of 6.4 KiB)
constexpr int STEP_MAX_PHASES = 4;
constexpr int STEP_MAX_TASKS = 8;      // per phase
constexpr int STEP_MAX_EDGES = 8;      // per task
constexpr int STEP_MAX_SOURCES = 8;    // distinct (buffer, frame offset) vectors read per step
constexpr int STEP_PF_MAX_STEPS = 16;  // steps per block of early-loaded static gather values
constexpr int STEP_PF_PAIRS_PER_THREAD = 2;
constexpr int STEP_MAX_GATHERS = 24;   // per program (loads are issued from an unrolled loop)

RNNG_HD inline int step_pow2_floor(int v) { int p = 1; while (p * 2 <= v) p *= 2; return p; }

struct StepEdge { int w_off, k_len, transposed, src; };    // src = index into StepLayout::src
struct StepTask { int n_out, chunk, n_edges; StepEdge e[STEP_MAX_EDGES]; };
struct StepPhase {
    int mv_off, prog_off;
    int n_tasks, cmax, n_slots, L;       // L lanes per slot (power of two), n_slots * L <= 256
    int n_e_max;                         // max edges per task
    int J[STEP_MAX_EDGES];               // float4 iterations per lane for edge index e (max over tasks)
    int w_base[STEP_MAX_EDGES];          // float offset of the weight region of edge index e
    int acc_base;                        // float offset of the accumulators [slot][NB]
    int item_chunk;                      // element-wise items: local unit = tid % item_chunk, stream = tid / item_chunk
    int n_static, pf_steps, pf_base;     // ring of early-loaded STATIC gather values: [2][pf_steps][n_static * items]
    StepTask task[STEP_MAX_TASKS];
};
struct StepSource { int buf, frame_off, k_len, k_pad, x_base, first_phase; };
struct StepLayout {
    int ok;                 // 0: does not fit the kernel's limits (reason in `why`)
    int why;
    int n_phases, n_sources, total_floats;
    StepPhase ph[STEP_MAX_PHASES];
    StepSource src[STEP_MAX_SOURCES];
};

constexpr int STEP_MAX_GROUPS = 4;

struct StepArgs {
    float* const* buf_ptr;                   // buffer table (read-only for the kernel's lifetime)
    const int32_t* words;                    // plan words (likewise)
    const float* weights;
    unsigned* ctrl;                          // [0]: set to 1 when a wait ran into the spin limit
    int desc_off, T, N, backward, G, xcd_stride, spin_limit;
    // Chain launches (several recurrent components side by side): group g runs descriptor
    // grp_desc_off[g] on grp_G[g] workgroups; block b belongs to group b % 8, part b / 8, which
    // puts each group on one XCD.  n_groups == 0: a single component (desc_off, G, xcd_stride).
    int n_groups, grp_desc_off[STEP_MAX_GROUPS], grp_G[STEP_MAX_GROUPS];
    // Chains of the matrix-core build: group g takes the blocks [grp_first[g], grp_first[g] +
    // grp_G[g] * grp_J[g]) (all groups use all XCDs).
    int grp_J[STEP_MAX_GROUPS], grp_first[STEP_MAX_GROUPS];
    // Frames [t_begin, t_end) are computed (forward: ascending, backward: descending); frames of
    // the window outside this range hold the results of earlier calls (T is the whole window).
    int t_begin, t_end;
    // Matrix-core build: the streams are split into J groups of N / J; workgroup w owns unit chunk
    // w % G of stream group w / G (G * J workgroups in all).  1 elsewhere.
    int J;
    // Wave-autonomous builds: hardware id of the XCD on which every workgroup of group g runs
    // (single-component launch: entry 0), as the host has observed for this launch shape, or -1.
    // With an id, tensors exchanged inside the group are written with plain stores (the XCD's L2
    // holds them, and the group's polling loads are served there); a workgroup that finds itself
    // on another XCD sets ctrl[0] = 2.  With -1 every exchanged tensor is written through.
    int xcc_expect[STEP_MAX_GROUPS];
    // Matrix-core build with the two-dimensional split: the partial sums that the workgroups hand
    // to each other, [frame][workgroup][column slice][row][stream] (sentinel-filled by the host).
    float* partial;
    // Wave-autonomous build compiled for one store window (MV::SW): the window that holds every
    // tensor the kernel stores (the workspace; at most 2 GiB).
    float* store_base;
    unsigned store_bytes;
    // Streaming build: a copy of the parameter buffer in which the matrices that the kernel reads
    // transposed are stored transposed (same offsets), and the size of both buffers in bytes.
    const float* weights_t;
    unsigned weight_bytes;
    // Matrix-core build with tile-blocked exchange: buffer twin_base + b is the blocked twin of
    // the exchanged tensor b (see the kernel).
    int twin_base;
};

RNNG_HD inline int step_count(const StepArgs& a) { return a.t_end - a.t_begin; }
RNNG_HD inline int step_frame(const StepArgs& a, int st) { return a.backward ? a.t_end - 1 - st : a.t_begin + st; }


// words: plan words; desc_off: step descriptor; G workgroups; NB streams per pass; N streams.
RNNG_HD inline void compute_step_layout(const int32_t* words, int desc_off, int G, int NB, int N, StepLayout& out) {
    out.ok = 0; out.why = 0; out.n_sources = 0; out.total_floats = 0;
    const int32_t* d = words + desc_off;
    out.n_phases = d[0];
    if (out.n_phases > STEP_MAX_PHASES) { out.why = 1; return; }
    int cur = 0;
    for (int p = 0; p < out.n_phases; ++p) {
        StepPhase& ph = out.ph[p];
        ph.mv_off = d[1 + 2 * p]; ph.prog_off = d[2 + 2 * p];
        ph.n_tasks = 0; ph.cmax = 0; ph.n_slots = 0; ph.L = 1; ph.n_e_max = 0; ph.acc_base = 0;
        for (int e = 0; e < STEP_MAX_EDGES; ++e) { ph.J[e] = 0; ph.w_base[e] = 0; }
        const int32_t* pg = words + ph.prog_off;
        if (pg[PG_NGATHER] > STEP_MAX_GATHERS) { out.why = 2; return; }
        ph.item_chunk = (pg[PG_MAXDIM] + G - 1) / G;
        if (ph.item_chunk * N > STEP_THREADS) { out.why = 3; return; }
        ph.n_static = 0; ph.pf_steps = 0; ph.pf_base = 0;
        for (int g = 0; g < pg[PG_NGATHER]; ++g)
            if (pg[PG_HEADER_WORDS + g * GA_WORDS + GA_KIND] == GA_KIND_STATIC) ++ph.n_static;
        {
            const int pairs = ph.n_static * ph.item_chunk * N;
            if (pairs > 0 && pairs <= STEP_PF_PAIRS_PER_THREAD * STEP_THREADS) {
                int st = step_pow2_floor(4096 / pairs);
                ph.pf_steps = st < 2 ? 2 : st > STEP_PF_MAX_STEPS ? STEP_PF_MAX_STEPS : st;
                ph.pf_base = cur; cur += 2 * ph.pf_steps * pairs;
                cur = (cur + 3) / 4 * 4;
            }
        }
        if (ph.mv_off < 0) continue;
        const int32_t* w = words + ph.mv_off;
        ph.n_tasks = w[0];
        if (ph.n_tasks > STEP_MAX_TASKS) { out.why = 4; return; }
        ++w;
        for (int t = 0; t < ph.n_tasks; ++t) {
            StepTask& tk = ph.task[t];
            tk.n_out = w[MV_NOUT]; tk.n_edges = w[MV_NEDGES]; tk.chunk = (tk.n_out + G - 1) / G;
            if (tk.n_edges > STEP_MAX_EDGES) { out.why = 5; return; }
            if (tk.chunk > ph.cmax) ph.cmax = tk.chunk;
            if (tk.n_edges > ph.n_e_max) ph.n_e_max = tk.n_edges;
            for (int e = 0; e < tk.n_edges; ++e) {
                const int32_t* ed = w + MV_HEADER_WORDS + e * MVE_WORDS;
                tk.e[e].w_off = ed[MVE_W_OFF]; tk.e[e].k_len = ed[MVE_KLEN]; tk.e[e].transposed = ed[MVE_TRANSPOSED];
                int s = 0;
                for (; s < out.n_sources; ++s)
                    if (out.src[s].buf == ed[MVE_SRC_BUF] && out.src[s].frame_off == ed[MVE_FRAME_OFF]) break;
                if (s == out.n_sources) {
                    if (s == STEP_MAX_SOURCES) { out.why = 6; return; }
                    out.src[s].buf = ed[MVE_SRC_BUF]; out.src[s].frame_off = ed[MVE_FRAME_OFF];
                    out.src[s].k_len = ed[MVE_KLEN]; out.src[s].k_pad = (ed[MVE_KLEN] + 255) / 256 * 256;
                    out.src[s].first_phase = p; out.src[s].x_base = 0;
                    ++out.n_sources;
                }
                tk.e[e].src = s;
            }
            w += MV_HEADER_WORDS + tk.n_edges * MVE_WORDS;
        }
        ph.n_slots = ph.n_tasks * ph.cmax;
        if (ph.n_slots > STEP_THREADS) { out.why = 7; return; }
        ph.L = step_pow2_floor(STEP_THREADS / ph.n_slots);
        if (ph.L > 64) ph.L = 64;
        for (int t = 0; t < ph.n_tasks; ++t)
            for (int e = 0; e < ph.task[t].n_edges; ++e) {
                const int j = (ph.task[t].e[e].k_len + 4 * ph.L - 1) / (4 * ph.L);
                if (j > ph.J[e]) ph.J[e] = j;
            }
        for (int e = 0; e < ph.n_e_max; ++e) { ph.w_base[e] = cur; cur += ph.J[e] * STEP_THREADS * 4; }
        ph.acc_base = cur; cur += ph.n_slots * NB;
        cur = (cur + 3) / 4 * 4;
    }
    for (int s = 0; s < out.n_sources; ++s) { out.src[s].x_base = cur; cur += NB * out.src[s].k_pad; }
    out.total_floats = cur;
    out.ok = 1;
}

}  // namespace rnng
