// Device code of the persistent recurrent-step kernel, shared by the ahead-of-time build
// (step.hip: element-wise programs interpreted from the plan words) and by the run-time
// specialised build (the same kernel with the element-wise programs of one component emitted
// as straight-line code and compiled with hiprtc).
//
// Scheme (paper Section 3.1, sequential part): one launch runs all T steps of one recurrent
// node in one direction.  G workgroups each own a chunk of every layer's units and keep their
// rows (forward) or columns (backward) of every full weight matrix inside the recurrent node
// resident in LDS.  Only the source vectors of those full connections cross workgroups.  There
// is no grid barrier: shared vectors are pre-filled with a sentinel bit pattern, a producer
// overwrites each element exactly once with a device-scope store, consumers poll the elements
// they need until none holds the sentinel.  Every wait is bounded by a spin limit; on expiry an
// error word is set and the kernel runs to its end without waiting again, so the grid drains.
#pragma once
#if !defined(__HIPCC_RTC__)
#include <hip/hip_runtime.h>
#endif

#include "program.h"
#include "step_layout.h"

namespace rnng {

constexpr unsigned STEP_SENTINEL = 0xFFFFFFFFu;
typedef float sfloatx4 __attribute__((ext_vector_type(4)));
typedef float sfloatx2 __attribute__((ext_vector_type(2)));


__device__ __forceinline__ float step_sigmoid(float x) { return 1.0f / (1.0f + __expf(-x)); }
__device__ __forceinline__ float step_tanh(float x) {
    const float ax = fabsf(x);
    const float t = __expf(-2.0f * ax);
    return copysignf((1.0f - t) / (1.0f + t), x);
}
__device__ __forceinline__ int suni(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ void store_shared(float* p, float v) {
    unsigned b = __float_as_uint(v);
    if (b == STEP_SENTINEL) b = 0x7FC00000u;    // a NaN result must not look like "not yet written"
    __hip_atomic_store(reinterpret_cast<unsigned*>(p), b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float* p) {
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// Copies rows [n][k] of one frame of a shared vector into LDS x[n * k_pad + k], waiting until
// no element holds the sentinel.
__device__ __forceinline__ void poll_source(float* x, const float* g, int N, int K, int k_pad, int tid,
                                            int spin_limit, bool& dead, unsigned* ctrl) {
    const int total = N * K;
    if ((K & 1) == 0) {
        for (int p = tid; 2 * p < total; p += STEP_THREADS) {
            const unsigned long long* src = reinterpret_cast<const unsigned long long*>(g) + p;
            unsigned lo, hi;
            int spins = 0;
            for (;;) {
                const unsigned long long v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                lo = (unsigned)v; hi = (unsigned)(v >> 32);
                if (lo != STEP_SENTINEL && hi != STEP_SENTINEL) break;
                if (dead) break;
                if (++spins > spin_limit) { dead = true; atomicExch(ctrl, 1u); break; }
            }
            int n = 0, k = 2 * p;
            if (N > 1) { n = k / K; k -= n * K; }
            sfloatx2 o = {__uint_as_float(lo), __uint_as_float(hi)};
            *reinterpret_cast<sfloatx2*>(&x[n * k_pad + k]) = o;
        }
    } else {
        for (int p = tid; p < total; p += STEP_THREADS) {
            const unsigned* src = reinterpret_cast<const unsigned*>(g) + p;
            unsigned v;
            int spins = 0;
            for (;;) {
                v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v != STEP_SENTINEL) break;
                if (dead) break;
                if (++spins > spin_limit) { dead = true; atomicExch(ctrl, 1u); break; }
            }
            const int n = p / K, k = p - n * K;
            x[n * k_pad + k] = __uint_as_float(v);
        }
    }
}

// LDS tables besides the dynamic region.
struct StepShared {
    StepLayout lay;
    unsigned short tinfo[STEP_MAX_PHASES][STEP_THREADS];   // task of the thread's matrix-vector slot (0xFFFF none)
    unsigned iteminfo[STEP_MAX_PHASES][STEP_THREADS];      // element-wise item: local unit | stream << 16 (0xFFFF none)
};

// Everything before the time loop: layout, thread tables, zeroed LDS, resident weights.
// Returns the workgroup's part index, or -1 if this workgroup does not take part.
template <int NB>
__device__ __forceinline__ int step_prologue(const StepArgs& a, StepShared& sh, float* lds) {
    int w = blockIdx.x;
    if (a.xcd_stride > 1) {
        if (w % a.xcd_stride) return -1;   // workgroups are dealt round-robin to the XCDs: keep one XCD's share
        w /= a.xcd_stride;
    }
    if (w >= a.G) return -1;
    const int tid = threadIdx.x;
    StepLayout& lay = sh.lay;
    if (tid == 0) compute_step_layout(a.words, a.desc_off, a.G, NB, a.N, lay);
    __syncthreads();
    const int n_phases = lay.n_phases;
    for (int i = tid; i < lay.total_floats; i += STEP_THREADS) lds[i] = 0.0f;
    for (int p = 0; p < n_phases; ++p) {
        const StepPhase& ph = lay.ph[p];
        unsigned short tk = 0xFFFF;
        if (ph.n_tasks > 0) {
            const int slot = tid / ph.L;
            if (slot < ph.n_slots) tk = (unsigned short)(slot / ph.cmax);
        }
        sh.tinfo[p][tid] = tk;
        const int il = tid % ph.item_chunk, n = tid / ph.item_chunk;
        sh.iteminfo[p][tid] = (unsigned)il | ((unsigned)(n < a.N ? n : 0xFFFF) << 16);
    }
    __syncthreads();
    // Resident weights: lane-major float4 blocks, zero beyond a row's length or a layer's width.
    for (int p = 0; p < n_phases; ++p) {
        const StepPhase& ph = lay.ph[p];
        const int tk = sh.tinfo[p][tid];
        if (tk == 0xFFFF) continue;
        const StepTask& task = ph.task[tk];
        const int slot = tid / ph.L, sl = tid % ph.L;
        const int ul = slot - tk * ph.cmax;
        const int u = w * task.chunk + ul;
        const bool uok = ul < task.chunk && u < task.n_out;
        for (int e = 0; e < task.n_edges; ++e) {
            const StepEdge ed = task.e[e];
            const float* W = a.weights + ed.w_off;
            const int Jt = (ed.k_len + 4 * ph.L - 1) / (4 * ph.L);
            const bool vec = !ed.transposed && (ed.k_len & 3) == 0;
            for (int j = 0; j < Jt; ++j) {
                const int k0 = 4 * (sl + ph.L * j);
                sfloatx4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (uok) {
                    if (vec && k0 + 3 < ed.k_len) {
                        v = *reinterpret_cast<const sfloatx4*>(W + (size_t)u * ed.k_len + k0);
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const int k = k0 + c;
                            if (k < ed.k_len) v[c] = ed.transposed ? W[(size_t)k * task.n_out + u] : W[(size_t)u * ed.k_len + k];
                        }
                    }
                }
                *reinterpret_cast<sfloatx4*>(&lds[ph.w_base[e] + (j * STEP_THREADS + tid) * 4]) = v;
            }
        }
    }
    __syncthreads();
    return w;
}

// Per-thread constants of one phase's matrix-vector part, kept in registers over the time loop.
struct MatvecRegs {
    int n_edges;                 // 0: this thread has no slot
    int L, sl, acc_addr;
    int xb[STEP_MAX_EDGES], kp[STEP_MAX_EDGES], J[STEP_MAX_EDGES], wb[STEP_MAX_EDGES];
};
template <int NB>
__device__ __forceinline__ void matvec_setup(MatvecRegs& r, const StepShared& sh, int p, int tid) {
    const StepPhase& ph = sh.lay.ph[p];
    const int tk = sh.tinfo[p][tid];
    r.n_edges = 0; r.L = ph.L; r.sl = tid & (ph.L - 1); r.acc_addr = ph.acc_base + (tid / ph.L) * NB;
#pragma unroll
    for (int e = 0; e < STEP_MAX_EDGES; ++e) { r.xb[e] = 0; r.kp[e] = 0; r.J[e] = 0; r.wb[e] = 0; }
    if (tk == 0xFFFF) return;
    const StepTask& task = ph.task[tk];
    r.n_edges = task.n_edges;
#pragma unroll
    for (int e = 0; e < STEP_MAX_EDGES; ++e) {
        if (e < task.n_edges) {
            const StepSource& sc = sh.lay.src[task.e[e].src];
            r.xb[e] = sc.x_base + 4 * r.sl; r.kp[e] = sc.k_pad;
            r.J[e] = (task.e[e].k_len + 4 * ph.L - 1) / (4 * ph.L);
            r.wb[e] = ph.w_base[e] + tid * 4;
        }
    }
}
template <int NB>
__device__ __forceinline__ void matvec_run(const MatvecRegs& r, float* lds) {
    if (r.n_edges == 0) return;
    float part[NB];
#pragma unroll
    for (int nn = 0; nn < NB; ++nn) part[nn] = 0.0f;
#pragma unroll
    for (int e = 0; e < STEP_MAX_EDGES; ++e) {
        if (e < r.n_edges) {
            const float* wp = lds + r.wb[e];
            const float* xp = lds + r.xb[e];
            const int J = r.J[e], kp = r.kp[e], L4 = 4 * r.L;
            for (int j = 0; j < J; ++j) {
                const sfloatx4 w4 = *reinterpret_cast<const sfloatx4*>(wp + j * STEP_THREADS * 4);
#pragma unroll
                for (int nn = 0; nn < NB; ++nn) {
                    const sfloatx4 x4 = *reinterpret_cast<const sfloatx4*>(xp + nn * kp + L4 * j);
                    part[nn] += w4.x * x4.x + w4.y * x4.y + w4.z * x4.z + w4.w * x4.w;
                }
            }
        }
    }
    for (int off = r.L >> 1; off > 0; off >>= 1) {
#pragma unroll
        for (int nn = 0; nn < NB; ++nn) part[nn] += __shfl_xor(part[nn], off, 64);
    }
    if (r.sl == 0) {
#pragma unroll
        for (int nn = 0; nn < NB; ++nn) lds[r.acc_addr + nn] = part[nn];
    }
}

// The shared source vectors first used in one phase, as uniform registers.
struct PhaseSources {
    bool used[STEP_MAX_SOURCES];
    const float* base[STEP_MAX_SOURCES];
    int k_len[STEP_MAX_SOURCES], k_pad[STEP_MAX_SOURCES], x_base[STEP_MAX_SOURCES], frame_off[STEP_MAX_SOURCES];
};
__device__ __forceinline__ void sources_setup(PhaseSources& ps, const StepArgs& a, const StepShared& sh, int p) {
    const int ns = suni(sh.lay.n_sources);
#pragma unroll
    for (int q = 0; q < STEP_MAX_SOURCES; ++q) {
        ps.used[q] = false; ps.base[q] = nullptr; ps.k_len[q] = ps.k_pad[q] = ps.x_base[q] = ps.frame_off[q] = 0;
        if (q < ns && suni(sh.lay.src[q].first_phase) == p) {
            const StepSource& sc = sh.lay.src[q];
            ps.used[q] = true;
            ps.base[q] = ((cbufs_t)a.buf_ptr)[suni(sc.buf)]; ps.k_len[q] = suni(sc.k_len); ps.k_pad[q] = suni(sc.k_pad);
            ps.x_base[q] = suni(sc.x_base); ps.frame_off[q] = suni(sc.frame_off);
        }
    }
}
__device__ __forceinline__ void poll_sources(const PhaseSources& ps, const StepArgs& a, float* lds, int t, int tid, bool& dead) {
#pragma unroll
    for (int q = 0; q < STEP_MAX_SOURCES; ++q) {
        if (ps.used[q]) {
            const int k_len = ps.k_len[q], k_pad = ps.k_pad[q];
            const int frame = t + ps.frame_off[q];
            float* x = lds + ps.x_base[q];
            if (frame < 0 || frame >= a.T) {
                for (int i = tid; i < a.N * k_len; i += STEP_THREADS) { const int nn = i / k_len; x[nn * k_pad + i - nn * k_len] = 0.0f; }
            } else {
                poll_source(x, ps.base[q] + (size_t)frame * a.N * k_len, a.N, k_len, k_pad, tid, a.spin_limit, dead, a.ctrl);
            }
        }
    }
}

// Shared source vectors first used in phase p: poll them into LDS (zeros outside the window).
__device__ __forceinline__ void poll_phase_sources(const StepArgs& a, const StepShared& sh, float* lds, int p, int t, int tid,
                                                   bool& dead) {
    const int ns = suni(sh.lay.n_sources);
    for (int q = 0; q < ns; ++q) {
        const StepSource& sc = sh.lay.src[q];
        if (suni(sc.first_phase) != p) continue;
        const int k_len = suni(sc.k_len), k_pad = suni(sc.k_pad);
        const int frame = t + suni(sc.frame_off);
        float* x = lds + suni(sc.x_base);
        if (frame < 0 || frame >= a.T) {
            for (int i = tid; i < a.N * k_len; i += STEP_THREADS) { const int nn = i / k_len; x[nn * k_pad + i - nn * k_len] = 0.0f; }
        } else {
            poll_source(x, ((cbufs_t)a.buf_ptr)[suni(sc.buf)] + (size_t)frame * a.N * k_len, a.N, k_len, k_pad, tid, a.spin_limit, dead, a.ctrl);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Run-time specialised phases.  PH is a generated descriptor:
//   static constexpr int P, NG, NI, NST, HAS_TASKS, ACC_PHASE; constexpr gkind(g), stslot(q);
//   static void ops(float* s)   straight-line code over the slot file.
// Buffer ids, widths, frame offsets and weight offsets are NOT baked into the code: they are read
// from the phase's program words at set-up, so components of equal structure share a binary.
// ---------------------------------------------------------------------------------------------
template <class PH>
struct PhaseRegs {
    const float* gptr[PH::NG > 0 ? PH::NG : 1];   // frame-0 address of the thread's element (nullptr: idle lane)
    long long gstride[PH::NG > 0 ? PH::NG : 1];   // floats per frame
    int goff[PH::NG > 0 ? PH::NG : 1];            // frame offset; for accumulator entries: LDS float index
    float* sptr[PH::NST > 0 ? PH::NST : 1];
    long long sstride[PH::NST > 0 ? PH::NST : 1];
    float inv[PH::NI > 0 ? PH::NI : 1];
    MatvecRegs mv;
    PhaseSources src;
    int n;                                        // stream of the thread's item, -1: none
};

template <class PH, int NB>
__device__ __forceinline__ void phase_setup(PhaseRegs<PH>& r, const StepArgs& a, const StepShared& sh, int w, int tid) {
    const StepPhase& ph = sh.lay.ph[PH::P];
    cwords_t pw = (cwords_t)a.words + suni(ph.prog_off);
    const unsigned item = sh.iteminfo[PH::P][tid];
    const int il = (int)(item & 0xFFFF);
    r.n = (item >> 16) == 0xFFFF ? -1 : (int)(item >> 16);
    const int G = a.G, N = a.N;
    const StepPhase& aph = sh.lay.ph[PH::ACC_PHASE];
#pragma unroll
    for (int g = 0; g < PH::NG; ++g) {
        cwords_t e = pw + PG_HEADER_WORDS + g * GA_WORDS;
        const int dim = e[GA_DIM];
        const int chunk = (dim + G - 1) / G, i = w * chunk + il;
        const bool active = r.n >= 0 && il < chunk && i < dim;
        if (PH::gkind(g) == GA_KIND_ACC) {
            r.gptr[g] = active ? a.weights : nullptr;   // any non-null marker
            r.goff[g] = aph.acc_base + (e[GA_FRAME_OFF] * aph.cmax + il) * NB + (r.n >= 0 ? r.n : 0);
            r.gstride[g] = 0;
        } else {
            r.gptr[g] = active ? ((cbufs_t)a.buf_ptr)[e[GA_BUF]] + (size_t)r.n * dim + i : nullptr;
            r.goff[g] = e[GA_FRAME_OFF];
            r.gstride[g] = (long long)N * dim;
        }
    }
    cwords_t iv = pw + PG_HEADER_WORDS + PH::NG * GA_WORDS;
#pragma unroll
    for (int v = 0; v < PH::NI; ++v) {
        const int dim = iv[v * IV_WORDS + IV_DIM];
        const int chunk = (dim + G - 1) / G, i = w * chunk + il;
        r.inv[v] = (r.n >= 0 && il < chunk && i < dim) ? a.weights[iv[v * IV_WORDS + IV_W_OFF] + i] : 0.0f;
    }
    cwords_t st = iv + PH::NI * IV_WORDS + pw[PG_NOPS] * MO_WORDS;
#pragma unroll
    for (int q = 0; q < PH::NST; ++q) {
        const int dim = st[q * ST_WORDS + ST_DIM];
        const int chunk = (dim + G - 1) / G, i = w * chunk + il;
        const bool active = r.n >= 0 && il < chunk && i < dim;
        r.sptr[q] = active ? ((cbufs_t)a.buf_ptr)[st[q * ST_WORDS + ST_BUF]] + (size_t)r.n * dim + i : nullptr;
        r.sstride[q] = (long long)N * dim;
    }
    if (PH::HAS_TASKS) { matvec_setup<NB>(r.mv, sh, PH::P, tid); sources_setup(r.src, a, sh, PH::P); }
}

template <class PH, int NB, int NPHASES>
__device__ __forceinline__ void phase_step(const PhaseRegs<PH>& r, const StepArgs& a, const StepShared& sh, float* lds,
                                           int t, int tid, bool& dead) {
    float s[MAX_SLOTS];
    // 1. element-wise inputs (own units): issued first, consumed after the matrix-vector part
#pragma unroll
    for (int g = 0; g < PH::NG; ++g) {
        if (PH::gkind(g) == GA_KIND_FRAMES) {
            const int frame = t + r.goff[g];
            float v = 0.0f;
            if (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) v = load_coherent(r.gptr[g] + frame * r.gstride[g]);
            s[g] = v;
        }
    }
#pragma unroll
    for (int v = 0; v < PH::NI; ++v) s[PH::NG + v] = r.inv[v];
    if (PH::HAS_TASKS) {
        poll_sources(r.src, a, lds, t, tid, dead);
        __syncthreads();
        matvec_run<NB>(r.mv, lds);
        __syncthreads();
    }
#pragma unroll
    for (int g = 0; g < PH::NG; ++g)
        if (PH::gkind(g) == GA_KIND_ACC) s[g] = r.gptr[g] != nullptr ? lds[r.goff[g]] : 0.0f;
    PH::ops(s);
#pragma unroll
    for (int q = 0; q < PH::NST; ++q)
        if (r.sptr[q] != nullptr) store_shared(r.sptr[q] + t * r.sstride[q], s[PH::stslot(q)]);
    if (NPHASES > 1) __syncthreads();
}

}  // namespace rnng
