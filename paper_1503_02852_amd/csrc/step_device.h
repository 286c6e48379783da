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
typedef unsigned suintx2 __attribute__((ext_vector_type(2)));
typedef float mfloatx4 __attribute__((ext_vector_type(4)));
typedef unsigned muintx4 __attribute__((ext_vector_type(4)));
// Buffer loads that poll shared vectors are device-coherent (sc1).  Unlike atomic loads they are
// not each followed by a wait, so all loads of a polling attempt are in flight together; a
// compiler barrier at the top of each attempt keeps them from being merged across attempts.
constexpr int STEP_COHERENT_AUX = 16;
__device__ __forceinline__ void step_compiler_barrier() { asm volatile("" ::: "memory"); }
// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait for the
// wavefront's global loads and stores, so loads issued ahead stay in flight across it.
__device__ __forceinline__ void step_lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
constexpr int STEP_RSRC_FLAGS = 0x00020000;


// v_rcp_f32 / v_exp_f32 (about 1 ulp each) instead of an IEEE division: far inside the 1e-4 bar.
__device__ __forceinline__ float step_sigmoid(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
// tanh without cancellation near 0: t = e^{-2|x|}; tanh|x| = (1 - t) / (1 + t).
__device__ __forceinline__ float step_tanh(float x) {
    const float t = __expf(-2.0f * fabsf(x));
    return copysignf((1.0f - t) * __builtin_amdgcn_rcpf(1.0f + t), x);
}
__device__ __forceinline__ int suni(int v) { return __builtin_amdgcn_readfirstlane(v); }
// A pointer that is the same in every lane, said so to the compiler (it then stays in scalar
// registers and can form a buffer descriptor without a loop over lanes).
template <class T>
__device__ __forceinline__ T* suni_ptr(T* p) {
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = (unsigned)suni((int)(unsigned)v), hi = (unsigned)suni((int)(unsigned)(v >> 32));
    return reinterpret_cast<T*>(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ unsigned step_shared_bits(float v) {
    const unsigned b = __float_as_uint(v);
    return b == STEP_SENTINEL ? 0x7FC00000u : b;    // a NaN result must not look like "not yet written"
}
// Every tensor lives in device memory.  A pointer read from the buffer table is a generic one to
// the compiler, and a store through it would be a FLAT instruction, which also counts as an LDS
// operation: each later wait for LDS data would then wait for the store as well.
typedef __attribute__((address_space(1))) unsigned step_guint_t;
typedef __attribute__((address_space(1))) float step_gfloat_t;
__device__ __forceinline__ step_guint_t* step_global_bits(float* p) { return (step_guint_t*)reinterpret_cast<unsigned*>(p); }
__device__ __forceinline__ void store_plain(float* p, float v) { *(step_gfloat_t*)p = v; }
__device__ __forceinline__ void store_shared(float* p, float v) {
    __hip_atomic_store(step_global_bits(p), step_shared_bits(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Plain store of an exchanged value: stays in this XCD's L2 (enough for readers on the same XCD).
__device__ __forceinline__ void store_shared_local(float* p, float v) {
    __hip_atomic_store(step_global_bits(p), step_shared_bits(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}
// Hardware id of the XCD this wavefront runs on.
__device__ __forceinline__ int step_xcc_id() {
    unsigned id;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
    return (int)(id & 0xFu);
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
//   static constexpr int P, NG, NI, NST, NS, NC, HAS_TASKS, ACC_PHASE;
//   constexpr gkind(g), gaux(g) (CARRY: result slot), sidx(g) (index among the STATIC gathers),
//   cidx(g) (index among the CARRY gathers), sgather(si) (gather index of static si), stslot(q);
//   static void ops(float* s)   straight-line code over the slot file.
// Buffer ids, widths, frame offsets and weight offsets are NOT baked into the code: they are read
// from the phase's program words at set-up, so components of equal structure share a binary.
// ---------------------------------------------------------------------------------------------
template <class PH>
struct PhaseRegs {
    const float* gptr[PH::NG > 0 ? PH::NG : 1];   // frame-0 address of the thread's element (nullptr: idle lane)
    int gstride[PH::NG > 0 ? PH::NG : 1];         // floats per frame (uniform)
    int goff[PH::NG > 0 ? PH::NG : 1];            // frame offset; ACC: LDS float index; STATIC with ring: index in a ring row
    float* sptr[PH::NST > 0 ? PH::NST : 1];
    int sstride[PH::NST > 0 ? PH::NST : 1];       // floats per frame (uniform)
    float* sbase[PH::NST > 0 ? PH::NST : 1];      // frame-0 address of the stored tensor (uniform)
    // wave-autonomous variant: stores go through one buffer descriptor over the whole tensor
    // (loop-invariant, in scalar registers) with a running per-lane byte offset svrun, advanced by
    // sdelta floats per step (negative in the backward loop).  A lane that stores nothing runs
    // far outside the tensor: its store is dropped by the bounds check instead of being branched
    // around, so the compiler can count the stores in flight (and the loop has no branches per
    // store).  Needs tensors below 1 GiB, which the host checks.
    unsigned svrun[PH::NST > 0 ? PH::NST : 1];
    int sdelta[PH::NST > 0 ? PH::NST : 1];
    // the same for gathers from tensors (matrix-core variant): frame-0 address of the tensor
    // (uniform) and the byte offset of the thread's element in frame 0 (idle lane: far outside)
    const float* gbase[PH::NG > 0 ? PH::NG : 1];
    unsigned gvoff[PH::NG > 0 ? PH::NG : 1];
    float inv[PH::NI > 0 ? PH::NI : 1];
    float carry[PH::NC > 0 ? PH::NC : 1];
    // wave-autonomous variant: a helper group's sums (POLLED gathers) for the NEXT step, loaded one
    // step ahead (they come from another XCD, which takes longer than a step's own exchange)
    float polled_next[PH::NG > 0 ? PH::NG : 1];
    // loader side of the static-gather ring: this thread's (static gather, item) pairs
    const float* pbase[STEP_PF_PAIRS_PER_THREAD];
    long long pstride[STEP_PF_PAIRS_PER_THREAD];
    int poff[STEP_PF_PAIRS_PER_THREAD];
    int pf_steps, pf_shift, pf_base, pairs;
    MatvecRegs mv;
    PhaseSources src;
    int n;                                        // stream of the thread's item, -1: none
};

// Loads one block of pf_steps steps of static gather values into ring half `half`.
template <class PH>
__device__ __forceinline__ void ring_fill(const PhaseRegs<PH>& r, const StepArgs& a, float* lds, int first_step, int half, int tid) {
#pragma unroll
    for (int q = 0; q < STEP_PF_PAIRS_PER_THREAD; ++q) {
        if (r.pbase[q] == nullptr) continue;
        float v[STEP_PF_MAX_STEPS];
#pragma unroll
        for (int j = 0; j < STEP_PF_MAX_STEPS; ++j) {
            v[j] = 0.0f;
            const int st = first_step + j;
            if (j < r.pf_steps && st < step_count(a)) {
                const int frame = step_frame(a, st) + r.poff[q];
                if (frame >= 0 && frame < a.T) v[j] = r.pbase[q][frame * r.pstride[q]];
            }
        }
#pragma unroll
        for (int j = 0; j < STEP_PF_MAX_STEPS; ++j)
            if (j < r.pf_steps) lds[r.pf_base + (half * r.pf_steps + j) * r.pairs + q * STEP_THREADS + tid] = v[j];
    }
}

// MODE 0: LDS variant (static gathers through the workgroup ring); 1: wave-autonomous variant
// (per-wavefront ring, own matrix-vector set-up); 2: static gathers are loaded directly.
// SH: StepShared, or a leaner table set with the members lay and iteminfo (threads beyond
// STEP_THREADS, which some variants have, own no item).
template <class PH, int NB, int MODE = 0, class SH = StepShared>
__device__ __forceinline__ void phase_setup(PhaseRegs<PH>& r, const StepArgs& a, const SH& sh, float* lds, int w, int tid) {
    const StepPhase& ph = sh.lay.ph[PH::P];
    cwords_t pw = (cwords_t)a.words + suni(ph.prog_off);
    const unsigned item = tid < STEP_THREADS ? sh.iteminfo[PH::P][tid] : 0xFFFF0000u;
    const int il = (int)(item & 0xFFFF);
    r.n = (item >> 16) == 0xFFFF ? -1 : (int)(item >> 16);
    const int G = a.G, N = a.N;
    const StepPhase& aph = sh.lay.ph[PH::ACC_PHASE];
    const int item_chunk = suni(ph.item_chunk), items = item_chunk * N;
    r.pf_steps = suni(ph.pf_steps); r.pf_base = suni(ph.pf_base); r.pairs = PH::NS * items;
    r.pf_shift = 0;
    while ((1 << r.pf_shift) < r.pf_steps) ++r.pf_shift;
#pragma unroll
    for (int g = 0; g < PH::NG; ++g) {
        cwords_t e = pw + PG_HEADER_WORDS + g * GA_WORDS;
        const int dim = e[GA_DIM];
        const int chunk = (dim + G - 1) / G, i = w * chunk + il;
        const bool active = r.n >= 0 && il < chunk && i < dim;
        r.gstride[g] = suni(N * dim);
        if (PH::gkind(g) == GA_KIND_ACC) {
            r.gptr[g] = active ? a.weights : nullptr;   // any non-null marker
            r.goff[g] = aph.acc_base + (e[GA_FRAME_OFF] * aph.cmax + il) * NB + (r.n >= 0 ? r.n : 0);
        } else if (PH::gkind(g) == GA_KIND_STATIC && (MODE == 1 || (MODE == 0 && r.pf_steps > 0))) {
            r.gptr[g] = active ? a.weights : nullptr;
            r.goff[g] = PH::sidx(g) * items + (r.n >= 0 ? r.n : 0) * item_chunk + il;
        } else {
            r.gptr[g] = active ? ((cbufs_t)a.buf_ptr)[e[GA_BUF]] + (size_t)r.n * dim + i : nullptr;
            r.goff[g] = e[GA_FRAME_OFF];
            if (MODE == 2) {
                r.gbase[g] = suni_ptr(((cbufs_t)a.buf_ptr)[e[GA_BUF]]);
                r.gvoff[g] = active ? (unsigned)((r.n * dim + i) * 4) : 0xC0000000u;
            }
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
        r.sbase[q] = suni_ptr(((cbufs_t)a.buf_ptr)[st[q * ST_WORDS + ST_BUF]]);
        r.sptr[q] = active ? r.sbase[q] + (size_t)r.n * dim + i : nullptr;
        r.sstride[q] = suni(N * dim);
    }
#pragma unroll
    for (int c = 0; c < (PH::NC > 0 ? PH::NC : 1); ++c) r.carry[c] = 0.0f;
    // ring loader pairs: pair index pi = q * 256 + tid -> (static gather si, item)
#pragma unroll
    for (int q = 0; q < STEP_PF_PAIRS_PER_THREAD; ++q) {
        r.pbase[q] = nullptr; r.pstride[q] = 0; r.poff[q] = 0;
        const int pi = q * STEP_THREADS + tid;
        if (MODE == 0 && PH::NS > 0 && r.pf_steps > 0 && pi < r.pairs) {
            const int si = pi / items, it = pi - si * items;
            const int n2 = it / item_chunk, il2 = it - n2 * item_chunk;
            cwords_t e = pw + PG_HEADER_WORDS + PH::sgather(si) * GA_WORDS;
            const int dim = e[GA_DIM];
            const int chunk = (dim + G - 1) / G, i = w * chunk + il2;
            if (il2 < chunk && i < dim) {
                r.pbase[q] = ((cbufs_t)a.buf_ptr)[e[GA_BUF]] + (size_t)n2 * dim + i;
                r.pstride[q] = (long long)N * dim; r.poff[q] = e[GA_FRAME_OFF];
            }
        }
    }
    if constexpr (MODE == 0) {   // the other variants have their own matrix-vector and ring set-up
        if (PH::HAS_TASKS) { matvec_setup<NB>(r.mv, sh, PH::P, tid); sources_setup(r.src, a, sh, PH::P); }
        if (PH::NS > 0 && r.pf_steps > 0) ring_fill<PH>(r, a, lds, 0, 0, tid);
    }
}

// Optional cycle stamps of one workgroup's steps 64..71 (8 stamps per step, written behind the
// control words) for tuning; compiled in only when RNNG_STEP_TRACE is defined for the run-time build
// (its value is the traced block index plus one).
#if defined(RNNG_STEP_TRACE)
#if !defined(RNNG_STEP_TRACE_AT)
#define RNNG_STEP_TRACE_AT 64
#endif
#define RNNG_STAMP(i)                                                                                       \
    if (blockIdx.x == RNNG_STEP_TRACE - 1 && tid == 0 && step >= RNNG_STEP_TRACE_AT && step < RNNG_STEP_TRACE_AT + 8)         \
        reinterpret_cast<unsigned long long*>(a.ctrl + 16)[(step - RNNG_STEP_TRACE_AT) * 8 + (i)] = clock64()
#else
#define RNNG_STAMP(i)
#endif

template <class PH, int NB, int NPHASES>
__device__ __forceinline__ void phase_step(PhaseRegs<PH>& r, const StepArgs& a, const StepShared& sh, float* lds,
                                           int step, int t, int tid, bool& dead) {
    float s[MAX_SLOTS];
    RNNG_STAMP(0);
    const bool ring = PH::NS > 0 && r.pf_steps > 0;
    const int js = ring ? (step & (r.pf_steps - 1)) : 0;
    const int blk = ring ? (step >> r.pf_shift) : 0;
    // 1. element-wise inputs (own units).  Values this program produced in the previous step come
    //    from registers, values that do not change during the step loop from the LDS ring (loaded a
    //    block of steps ahead); anything else is loaded coherently now and consumed after the
    //    matrix-vector part.
#pragma unroll
    for (int g = 0; g < PH::NG; ++g) {
        if (PH::gkind(g) == GA_KIND_CARRY) {
            if (step > 0) {
                s[g] = r.carry[PH::cidx(g)];
            } else {      // first step of this call: the previous frame's value, if the window has one
                const int frame = t + r.goff[g];
                s[g] = (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) ? r.gptr[g][(long long)frame * r.gstride[g]] : 0.0f;
            }
        } else if (PH::gkind(g) == GA_KIND_STATIC && ring) {
            s[g] = r.gptr[g] != nullptr ? lds[r.pf_base + ((blk & 1) * r.pf_steps + js) * r.pairs + r.goff[g]] : 0.0f;
        } else if (PH::gkind(g) != GA_KIND_ACC) {
            const int frame = t + r.goff[g];
            float v = 0.0f;
            if (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) {
                if (PH::gkind(g) == GA_KIND_STATIC) v = r.gptr[g][(long long)frame * r.gstride[g]];
                else v = load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]);
            }
            s[g] = v;
        }
    }
#pragma unroll
    for (int v = 0; v < PH::NI; ++v) s[PH::NG + v] = r.inv[v];
    RNNG_STAMP(1);
    if (PH::HAS_TASKS) {
        poll_sources(r.src, a, lds, t, tid, dead);
        RNNG_STAMP(2);
        __syncthreads();
        RNNG_STAMP(3);
        matvec_run<NB>(r.mv, lds);
        RNNG_STAMP(4);
        __syncthreads();
    }
    RNNG_STAMP(5);
#pragma unroll
    for (int g = 0; g < PH::NG; ++g)
        if (PH::gkind(g) == GA_KIND_ACC) s[g] = r.gptr[g] != nullptr ? lds[r.goff[g]] : 0.0f;
    PH::ops(s);
    RNNG_STAMP(6);
#pragma unroll
    for (int q = 0; q < PH::NST; ++q)
        if (r.sptr[q] != nullptr) store_shared(r.sptr[q] + (long long)t * r.sstride[q], s[PH::stslot(q)]);
#pragma unroll
    for (int g = 0; g < PH::NG; ++g)
        if (PH::gkind(g) == GA_KIND_CARRY) r.carry[PH::cidx(g)] = s[PH::gaux(g)];
    RNNG_STAMP(7);
    // at the first step of a block: fetch the next block of static values into the other ring half
    if (ring && js == 0 && step + r.pf_steps < step_count(a)) ring_fill<PH>(r, a, lds, step + r.pf_steps, (blk + 1) & 1, tid);
    if (NPHASES > 1 || (ring && !PH::HAS_TASKS)) __syncthreads();
}


// =============================================================================================
// Wave-autonomous variant (run-time specialised, single-phase components, few streams).
//
// Each wavefront owns UW units of every layer and is self-sufficient: its rows of the full
// weight matrices live in its vector registers (a row's contraction is spread over the 64
// lanes, F = ceil(K / 64) consecutive elements per lane), it polls the shared source vectors
// straight into registers, reduces each row with DPP adds, and runs the element-wise program
// for its own units on its first lanes.  There is no LDS staging of weights or vectors and no
// workgroup barrier inside the time loop; a workgroup is just four such wavefronts on one CU.
//
// MV is a generated descriptor:
//   static constexpr int NT (tasks), UW (units per wavefront), NSRC, RW (weight registers),
//   NREG (polled regions: single shared vectors or exchange bundles), XFR, NBS (bundle stores),
//   XF (source registers per stream), EARLY (placement of the non-shared stores);  constexpr nedges(task), esrc(task, e), F(src), K(src),
//   xoff(src), woff(ul, task, e); per region rbuf, rfoff, RK (floats per stream), RB (interleave
//   factor), rsrc(r, j) (source that reads member j, -1: none); per bundle store bs_ebuf, bs_B,
//   bs_dim, bs_member0, bs_q(bs, j) (store index of member j or -1); bundled(q).
// =============================================================================================
__device__ __forceinline__ float wave_sum_dpp(float v) {
#define RNNG_DPP(ctrl, rmask) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, rmask, 0xf, false))
    v += RNNG_DPP(0xB1, 0xf);    // quad_perm [1,0,3,2]
    v += RNNG_DPP(0x4E, 0xf);    // quad_perm [2,3,0,1]
    v += RNNG_DPP(0x141, 0xf);   // row_half_mirror
    v += RNNG_DPP(0x140, 0xf);   // row_mirror: every lane of a 16-lane row holds the row's sum
    v += RNNG_DPP(0x142, 0xa);   // row_bcast:15 into rows 1 and 3
    v += RNNG_DPP(0x143, 0xc);   // row_bcast:31 into rows 2 and 3: lane 63 holds the total
#undef RNNG_DPP
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

constexpr int WAVE_RING_STEPS = 16;
constexpr int WAVE_FMAX = 32;   // elements of one contraction per lane (K <= 2048)

template <class MV>
struct WaveRegs {
    float wr[MV::RW > 0 ? MV::RW : 1];
    // polled regions (a shared vector, or an exchange bundle of several): frame 0, floats per frame, frame offset
    const float* xsrc[MV::NREG > 0 ? MV::NREG : 1];
    long long xstride[MV::NREG > 0 ? MV::NREG : 1];
    int xfoff[MV::NREG > 0 ? MV::NREG : 1];
    // bundle stores: frame 0 of the interleaved tensor, floats per frame, this lane's byte offset in a frame
    float* bbase[MV::NBS > 0 ? MV::NBS : 1];
    int bstride[MV::NBS > 0 ? MV::NBS : 1];
    unsigned bvoff[MV::NBS > 0 ? MV::NBS : 1];      // (WAVE_NO_STORE: this lane stores nothing, as PhaseRegs::svrun)
    // every workgroup of this group runs on one XCD: tensors exchanged inside the group are
    // stored plainly (same in all lanes and workgroups of the group)
    bool local;
};

// Exchanged tensors by reader (generated MV::xmode(q) / MV::bs_xmode(b)):
//   0: polled inside this group only -> plain stores if the group sits on one XCD (a written-
//      through store is acknowledged much later, and this wavefront's next polling loads only
//      complete after the acknowledgement: loads and stores retire in issue order);
//   1: polled by other groups of a chain only (other XCDs) -> written through;
//   2: both -> plain store at once, and written through one step late, right after the next
//      step's poll, where its acknowledgement overlaps the step's arithmetic.
template <class MV>
__device__ __forceinline__ void wave_xcd_setup(WaveRegs<MV>& wv, const StepArgs& a, int group) {
    const int expect = a.xcc_expect[group];
    wv.local = suni(expect) >= 0;
    if (expect >= 0 && step_xcc_id() != expect && threadIdx.x == 0) atomicExch(a.ctrl, 2u);
}

// Part index of this workgroup in a single-component launch, or -1 if it has no part.
__device__ __forceinline__ int step_part_index(const StepArgs& a) {
    int w = blockIdx.x;
    if (a.xcd_stride > 1) {
        if (w % a.xcd_stride) return -1;
        w /= a.xcd_stride;
    }
    return w < a.G ? w : -1;
}

template <class MV, int NB>
__device__ __forceinline__ void wave_prologue(const StepArgs& a, StepShared& sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) compute_step_layout(a.words, a.desc_off, a.G, NB, a.N, sh.lay);
    const int ul = lane % MV::UW, n = lane / MV::UW;
    sh.iteminfo[0][tid] = (unsigned)(wave * MV::UW + ul) | ((unsigned)(n < a.N ? n : 0xFFFF) << 16);
    __syncthreads();
}

template <class MV>
__device__ __forceinline__ void wave_setup(WaveRegs<MV>& wv, const StepArgs& a, const StepShared& sh, int w, int tid) {
    const StepPhase& ph = sh.lay.ph[0];
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int r = 0; r < MV::NREG; ++r) {
        wv.xfoff[r] = MV::rfoff(r); wv.xstride[r] = (long long)MV::N * MV::RK(r);
        wv.xsrc[r] = ((cbufs_t)a.buf_ptr)[MV::rbuf(r)];
    }
#pragma unroll
    for (int ul = 0; ul < MV::UW; ++ul) {
#pragma unroll
        for (int task = 0; task < MV::NT; ++task) {
            const StepTask& tk = ph.task[task];
            const int chunk = suni(tk.chunk), n_out = suni(tk.n_out);
            const int ulw = wave * MV::UW + ul, u = w * chunk + ulw;
            const bool uok = ulw < chunk && u < n_out;
#pragma unroll
            for (int e = 0; e < STEP_MAX_EDGES; ++e) {
                if (e < MV::nedges(task)) {
                    const int K = suni(tk.e[e].k_len), transposed = suni(tk.e[e].transposed);
                    const float* W = a.weights + suni(tk.e[e].w_off);
                    const int F = MV::F(MV::esrc(task, e));
#pragma unroll
                    for (int f = 0; f < WAVE_FMAX; ++f) {
                        if (f < F) {
                            const int k = F * lane + f;
                            float v = 0.0f;
                            if (uok && k < K) v = transposed ? W[(size_t)k * n_out + u] : W[(size_t)u * K + k];
                            wv.wr[MV::woff(ul, task, e) + f] = v;
                        }
                    }
                }
            }
        }
    }
}

// 1: the wave-autonomous kernels are built for one store window (the launcher puts the definition
// in front of the generated source when the workspace fits)
#if !defined(RNNG_STORE_WINDOW)
#define RNNG_STORE_WINDOW 0
#endif
constexpr unsigned WAVE_NO_STORE = 0xC0000000u;       // +- 1 GiB stays outside a tensor below 1 GiB

// MV::SW: every stored tensor lies in one window of at most 2 GiB (the host checks it: the
// workspace), and all stores go through ONE descriptor over that window instead of one per
// tensor, which frees four scalar registers per stored tensor (with ten stored tensors the
// descriptors alone pushed the time loop into scalar spills, ~50 v_readlane per step).  Parked
// lanes stay outside: WAVE_NO_STORE +- 1 GiB is beyond 2 GiB.
template <class PH, class MV>
__device__ __forceinline__ void wave_store_setup(PhaseRegs<PH>& r, const StepArgs& a) {
#pragma unroll
    for (int q = 0; q < PH::NST; ++q) {
        r.sdelta[q] = a.backward ? -r.sstride[q] : r.sstride[q];
        const float* base = MV::SW ? a.store_base : r.sbase[q];
        r.svrun[q] = r.sptr[q] != nullptr ? (unsigned)(((int)(r.sptr[q] - base) + step_frame(a, 0) * r.sstride[q]) * 4) : WAVE_NO_STORE;
    }
}
template <class PH, class MV>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t wave_store_rsrc(const PhaseRegs<PH>& r, int q, const StepArgs& a) {
    if (MV::SW) return __builtin_amdgcn_make_buffer_rsrc(a.store_base, 0, (int)a.store_bytes, STEP_RSRC_FLAGS);
    return __builtin_amdgcn_make_buffer_rsrc(r.sbase[q], 0, a.T * r.sstride[q] * 4, STEP_RSRC_FLAGS);
}

// One value per lane into the current frame of stored tensor q.  mode 0: not exchanged, 1:
// exchanged, plain store, 2: exchanged, written through; back: the previous step's frame (the
// running offsets have moved on by one step already).
template <class PH, class MV>
__device__ __forceinline__ void wave_store(const PhaseRegs<PH>& r, int q, float v, int mode, const StepArgs& a, bool back = false) {
    const __amdgpu_buffer_rsrc_t rs = wave_store_rsrc<PH, MV>(r, q, a);
    const int off = (int)(back ? r.svrun[q] - (unsigned)(r.sdelta[q] * 4) : r.svrun[q]);
    if (mode == 2) __builtin_amdgcn_raw_buffer_store_b32(step_shared_bits(v), rs, off, 0, STEP_COHERENT_AUX);
    else if (mode == 1) __builtin_amdgcn_raw_buffer_store_b32(step_shared_bits(v), rs, off, 0, 0);
    else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, off, 0, 0);
}
template <class PH>
__device__ __forceinline__ void wave_store_advance(PhaseRegs<PH>& r) {
#pragma unroll
    for (int q = 0; q < PH::NST; ++q) r.svrun[q] += (unsigned)(r.sdelta[q] * 4);
}

// Bundle stores: the lane that stores member values of a bundle (same item for all members) writes
// them as one vector into the interleaved exchange tensor.
template <class PH, class MV>
__device__ __forceinline__ void wave_bundle_setup(WaveRegs<MV>& wv, const PhaseRegs<PH>& r, const StepArgs& a) {
#pragma unroll
    for (int bs = 0; bs < MV::NBS; ++bs) {
        wv.bbase[bs] = ((cbufs_t)a.buf_ptr)[MV::bs_ebuf(bs)];
        wv.bstride[bs] = MV::N * MV::bs_dim(bs) * MV::bs_B(bs);
        const int q0 = MV::bs_q(bs, 0);       // member 0 always exists
        const float* mbase = ((cbufs_t)a.buf_ptr)[MV::bs_member0(bs)];
        wv.bvoff[bs] = r.sptr[q0] != nullptr ? (unsigned)((int)(r.sptr[q0] - mbase) * MV::bs_B(bs) * 4) + (MV::SW ? (unsigned)((wv.bbase[bs] - a.store_base) * 4) : 0u)
                                             : WAVE_NO_STORE;
    }
}

// Loader side of a wavefront's private ring of STATIC gather values: pair = (static gather, item).
template <class PH, class MV, int NB>
struct WaveRing {
    static constexpr int ITEMS = MV::UW * NB;
    static constexpr int PAIRS = PH::NS * ITEMS;
    static constexpr int QN = (PAIRS + 63) / 64;
    static constexpr int QNA = QN > 0 ? QN : 1;
    static constexpr int FLOATS = WAVE_RING_STEPS * (PAIRS > 0 ? PAIRS : 1);
    const float* pbase[QN > 0 ? QN : 1];
    long long pstride[QN > 0 ? QN : 1];
    int poff[QN > 0 ? QN : 1];
};

template <class PH, class MV, int NB>
__device__ __forceinline__ void wave_ring_setup(WaveRing<PH, MV, NB>& rg, const StepArgs& a, const StepShared& sh, int w, int tid) {
    typedef WaveRing<PH, MV, NB> RG;
    const int lane = tid & 63, wave = tid >> 6;
    cwords_t pw = (cwords_t)a.words + suni(sh.lay.ph[0].prog_off);
#pragma unroll
    for (int q = 0; q < RG::QN; ++q) {
        // lanes without a pair load one valid word that nobody reads
        rg.pbase[q] = reinterpret_cast<const float*>(a.ctrl); rg.pstride[q] = 0; rg.poff[q] = 0;
        const int pi = q * 64 + lane;
        if (pi < RG::PAIRS) {
            const int si = pi / RG::ITEMS, it = pi - si * RG::ITEMS;
            const int n2 = it / MV::UW, il2 = wave * MV::UW + (it - n2 * MV::UW);
            cwords_t e = pw + PG_HEADER_WORDS + PH::sgather(si) * GA_WORDS;
            const int dim = e[GA_DIM];
            const int chunk = (dim + a.G - 1) / a.G, i = w * chunk + il2;
            if (n2 < a.N && il2 < chunk && i < dim) {
                rg.pbase[q] = ((cbufs_t)a.buf_ptr)[e[GA_BUF]] + (size_t)n2 * dim + i;
                rg.pstride[q] = (long long)a.N * dim; rg.poff[q] = e[GA_FRAME_OFF];
            }
        }
    }
}

// The ring holds the static values of the next WAVE_RING_STEPS steps, one row per step (row =
// step mod WAVE_RING_STEPS).  wave_ring_load fetches this lane's pairs for one step into
// registers, wave_ring_store puts them into that step's row; the time loop loads the row of step
// st + WAVE_RING_STEPS right after it has consumed the row of step st and stores it two steps
// later, so the load's latency never sits in front of a wait.
template <class PH, class MV, int NB, int QNA>
__device__ __forceinline__ void wave_ring_load(float (&v)[QNA],
                                               const WaveRing<PH, MV, NB>& rg, const StepArgs& a, int st) {
    typedef WaveRing<PH, MV, NB> RG;
#pragma unroll
    for (int q = 0; q < RG::QN; ++q) {
        // no branch around the load (the compiler could not count the loads and stores in flight
        // across one and would wait for all of them, the written-through stores included); steps
        // past the end and frames outside the window read a clamped frame, and wave_ring_store
        // replaces what that gave by zero: the loaded value is not touched before, so nothing
        // waits for it here
        const int stc = st < step_count(a) ? st : step_count(a) - 1;
        const int frame = step_frame(a, stc) + rg.poff[q];
        const int fc = frame < 0 ? 0 : (frame >= a.T ? a.T - 1 : frame);
        v[q] = rg.pbase[q][fc * rg.pstride[q]];
    }
}
template <class PH, class MV, int NB, int QNA>
__device__ __forceinline__ void wave_ring_store(const float (&v)[QNA], const WaveRing<PH, MV, NB>& rg, const StepArgs& a,
                                                float* ring, int st, int lane) {
    typedef WaveRing<PH, MV, NB> RG;
#pragma unroll
    for (int q = 0; q < RG::QN; ++q) {
        const int stc = st < step_count(a) ? st : step_count(a) - 1;
        const int frame = step_frame(a, stc) + rg.poff[q];
        // (lanes without a unit hold a word nobody reads; kernels with exchange zero it all the same)
        const bool valid = frame >= 0 && frame < a.T && (MV::NSRC == 0 || (rg.pstride[q] != 0 && st < step_count(a)));
        const float x = valid ? v[q] : 0.0f;
        if (q * 64 + lane < RG::PAIRS) ring[(st & (WAVE_RING_STEPS - 1)) * RG::PAIRS + q * 64 + lane] = x;
    }
    // other lanes of this wavefront read these values in later steps
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// Rows of the first WAVE_RING_STEPS steps, before the time loop.
template <class PH, class MV, int NB>
__device__ __forceinline__ void wave_ring_fill(const WaveRing<PH, MV, NB>& rg, const StepArgs& a, float* ring, int lane) {
    typedef WaveRing<PH, MV, NB> RG;
    for (int st = 0; st < WAVE_RING_STEPS; ++st) {
        float v[RG::QNA];
        wave_ring_load<PH, MV, NB, RG::QNA>(v, rg, a, st);
        wave_ring_store<PH, MV, NB, RG::QNA>(v, rg, a, ring, st, lane);
    }
}

// The workgroup's four wavefronts poll the shared source vectors together (each element is
// fetched once per workgroup, all loads of one attempt are issued before any is checked) and
// hand them to each other through a double-buffered LDS area; one workgroup barrier per step.
template <class MV, int NB>
struct GroupX {
    // LDS: one block [stream][quad][lane][4] per source (bundles are de-interleaved on the way
    // in).  Lane l multiplies the F consecutive elements F l ... F l + F - 1 of a vector; they are
    // kept as quads [f / 4][l][f % 4], so that a wavefront's 128-bit read of one quad covers 1 KiB
    // of consecutive addresses: no bank conflicts (element-major order has lanes F floats apart,
    // which for F = 8 makes every fourth lane hit the same banks and the four wavefronts' reads,
    // 64 KiB per step in charlm_n1's backward loop, take four times as long).
    static __device__ __forceinline__ constexpr int F4(int s) { return (MV::F(s) + 3) / 4 * 4; }
    static __device__ __forceinline__ constexpr int off(int s) {
        int o = 0;
        for (int i = 0; i < s; ++i) o += NB * 64 * F4(i);
        return o;
    }
    static constexpr int FLOATS = off(MV::NSRC) > 0 ? off(MV::NSRC) : 1;     // one buffer
    // LDS index of element k of source s, stream n / of value f of lane l
    static __device__ __forceinline__ int pos(int s, int n, int k) {
        const int l = k / MV::F(s), f = k - l * MV::F(s);
        return off(s) + n * 64 * F4(s) + ((f >> 2) * 64 + l) * 4 + (f & 3);
    }
    static __device__ __forceinline__ int lane_pos(int s, int n, int l, int f) { return off(s) + n * 64 * F4(s) + ((f >> 2) * 64 + l) * 4 + (f & 3); }
    static __device__ __forceinline__ constexpr int pairs_per_thread(int r) { return (NB * MV::RK(r) / 2 + STEP_THREADS - 1) / STEP_THREADS; }
    static __device__ __forceinline__ constexpr int words_per_thread(int r) { return (NB * MV::RK(r) + STEP_THREADS - 1) / STEP_THREADS; }
};
#if !defined(WAVE_RETRY_SLEEP)
#define WAVE_RETRY_SLEEP 0      // units of 64 clocks between polling attempts
#endif
constexpr int GROUP_MAX_LOADS = 16;  // per thread and region (N * K <= 4096 elements when K is odd, 8192 when even)

constexpr unsigned WAVE_POLL_OUTSIDE = 0x40000000u;

// The registers a step's polling loads land in.  A step's first attempt is issued at the end of
// the step before (right behind that step's stores), so they live across steps.
template <class MV>
struct PollRegs {
    suintx2 v64[MV::NREG > 0 ? MV::NREG : 1][GROUP_MAX_LOADS];
    unsigned v32[MV::NREG > 0 ? MV::NREG : 1][GROUP_MAX_LOADS];
};

// One polling attempt for frame t: all loads are issued back to back (device-coherent buffer
// loads; atomic loads would each be followed by a wait).  One buffer descriptor per source; a
// frame outside the window gets an empty one.  Loads beyond a descriptor's size return zero, so no
// load needs a branch around it.
template <class MV, int NB>
__device__ __forceinline__ void group_poll_issue(PollRegs<MV>& pr, const WaveRegs<MV>& wv, const StepArgs& a, int t, int tid) {
    typedef GroupX<MV, NB> GX;
    step_compiler_barrier();
#pragma unroll
    for (int s = 0; s < MV::NREG; ++s) {
        // one descriptor over the whole tensor (loop-invariant); a lane beyond the frame's vector
        // and a frame outside the window each add 1 GiB to the offset, which lands beyond the
        // tensor (below 1 GiB: the host checks it) without wrapping, so such loads return zero
        const int frame = t + wv.xfoff[s];
        const unsigned fo = (frame >= 0 && frame < a.T) ? (unsigned)(frame * (MV::N * MV::RK(s) * 4)) : WAVE_POLL_OUTSIDE;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(wv.xsrc[s]), 0, a.T * MV::N * MV::RK(s) * 4, STEP_RSRC_FLAGS);
        if ((MV::RK(s) & 1) == 0) {
#pragma unroll
            for (int j = 0; j < GROUP_MAX_LOADS; ++j) {
                const int p = tid + STEP_THREADS * j;
                const unsigned lo = 2 * p < MV::N * MV::RK(s) ? (unsigned)(p * 8) : WAVE_POLL_OUTSIDE;
                if (j < GX::pairs_per_thread(s)) pr.v64[s][j] = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(lo + fo), 0, STEP_COHERENT_AUX);
            }
        } else {
#pragma unroll
            for (int j = 0; j < GROUP_MAX_LOADS; ++j) {
                const int p = tid + STEP_THREADS * j;
                const unsigned lo = p < MV::N * MV::RK(s) ? (unsigned)(p * 4) : WAVE_POLL_OUTSIDE;
                if (j < GX::words_per_thread(s)) pr.v32[s][j] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(lo + fo), 0, STEP_COHERENT_AUX);
            }
        }
    }
    step_compiler_barrier();
}

// Hands polled values to LDS: out-of-window frames and lanes beyond the vector arrive as zeros; a
// bundle's interleaved elements [unit][B] go to the blocks of the sources that read its members.
template <class MV, int NB>
__device__ __forceinline__ void group_poll_deliver(const PollRegs<MV>& pr, float* xs, int tid) {
    typedef GroupX<MV, NB> GX;
    const auto& v64 = pr.v64;
    const auto& v32 = pr.v32;
    bool bundles = false;
#pragma unroll
    for (int r = 0; r < MV::NREG; ++r) bundles = bundles || MV::RB(r) > 1;
    if (bundles) __builtin_assume(tid >= 0 && tid < STEP_THREADS);
#pragma unroll
    for (int r = 0; r < MV::NREG; ++r) {
            const int RK = MV::RK(r), B = MV::RB(r), K = RK / B, total = MV::N * RK;      // (MV::N: the stream count the kernel is built for)
        if ((RK & 1) == 0) {
#pragma unroll
            for (int j = 0; j < GROUP_MAX_LOADS; ++j) {
                const int p = tid + STEP_THREADS * j;
                if (j < GX::pairs_per_thread(r) && 2 * p < total) {
                    int n = 0, e = 2 * p;
                    if (NB > 1) { n = e / RK; e -= n * RK; }
                    if (B == 1) {
                        if (MV::F(MV::rsrc(r, 0)) % 2 == 0) {      // both halves belong to one lane's quad
                            const sfloatx2 o = {__uint_as_float(v64[r][j].x), __uint_as_float(v64[r][j].y)};
                            *reinterpret_cast<sfloatx2*>(&xs[GX::pos(MV::rsrc(r, 0), n, e)]) = o;
                        } else {
                            xs[GX::pos(MV::rsrc(r, 0), n, e)] = __uint_as_float(v64[r][j].x);
                            xs[GX::pos(MV::rsrc(r, 0), n, e + 1)] = __uint_as_float(v64[r][j].y);
                        }
                    } else if (MV::rsrc(r, 0) >= 0 && MV::rsrc(r, 1) >= 0 && (B == 2 || (MV::rsrc(r, 2) >= 0 && MV::rsrc(r, 3) >= 0))) {
                        // every member is read here (they are equally wide, so their blocks differ
                        // by the offset only): no branch per pair, the block is a select.
                        // e = k * B + m with m even: members m and m + 1 of unit k
                        const int k = e / B, m = e - k * B, s0 = MV::rsrc(r, 0);
                        const int at = GX::pos(s0, n, k) - GX::off(s0);
                        int o0 = GX::off(s0), o1 = GX::off(MV::rsrc(r, 1));
                        if (B == 4 && m != 0) { o0 = GX::off(MV::rsrc(r, 2)); o1 = GX::off(MV::rsrc(r, 3)); }
                        xs[at + o0] = __uint_as_float(v64[r][j].x);
                        xs[at + o1] = __uint_as_float(v64[r][j].y);
                    } else {
                        const int k = e / B, m = e - k * B;
#pragma unroll
                        for (int mm = 0; mm < 4; mm += 2) {
                            if (mm < B && m == mm) {
                                if (MV::rsrc(r, mm) >= 0) xs[GX::pos(MV::rsrc(r, mm) >= 0 ? MV::rsrc(r, mm) : 0, n, k)] = __uint_as_float(v64[r][j].x);
                                if (MV::rsrc(r, mm + 1) >= 0) xs[GX::pos(MV::rsrc(r, mm + 1) >= 0 ? MV::rsrc(r, mm + 1) : 0, n, k)] = __uint_as_float(v64[r][j].y);
                            }
                        }
                    }
                    (void)K;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < GROUP_MAX_LOADS; ++j) {
                const int p = tid + STEP_THREADS * j;
                if (j < GX::words_per_thread(r) && p < total) {
                    int n = 0, k = p;
                    if (NB > 1) { n = k / RK; k -= n * RK; }
                    xs[GX::pos(MV::rsrc(r, 0), n, k)] = __uint_as_float(v32[r][j]);      // odd widths are never bundled
                }
            }
        }
    }
}

// Completes the polling of frame t, whose first attempt is already under way: the step's work
// that does not need the polled vectors (mid) runs under it, then the loads are checked and
// repeated until none holds a sentinel, and the vectors go to LDS.
// extra(false) tells whether the wavefront's other polled values (a helper group's sums, loaded by
// mid) have arrived, extra(true) loads them again: they take part in the same attempts.
template <class MV, int NB, class Mid, class Extra>
__device__ __forceinline__ void group_poll(PollRegs<MV>& pr, float* xs, const WaveRegs<MV>& wv, const StepArgs& a, int step, int t, int tid, bool& dead, Mid&& mid, Extra&& extra) {
    typedef GroupX<MV, NB> GX;
    // The range of the thread index lets the bounds tests of whole regions fold.  That pays in
    // kernels that poll bundles (two stores per pair: 1.30 -> 1.24 ms in charlm_n1's backward
    // loop); the single stores of plain regions are faster behind their tests (each store then
    // waits for its own load only: 0.83 against 0.89 ms in the forward loop), so kernels without
    // bundles are not told.
    bool bundles = false;
#pragma unroll
    for (int r = 0; r < MV::NREG; ++r) bundles = bundles || MV::RB(r) > 1;
    if (bundles) __builtin_assume(tid >= 0 && tid < STEP_THREADS);
    auto all_ok = [&](const PollRegs<MV>& q) {
        bool ok = true;
#pragma unroll
        for (int s = 0; s < MV::NREG; ++s) {
            if ((MV::RK(s) & 1) == 0) {
#pragma unroll
                for (int j = 0; j < GROUP_MAX_LOADS; ++j)
                    if (j < GX::pairs_per_thread(s)) ok = ok && q.v64[s][j].x != STEP_SENTINEL && q.v64[s][j].y != STEP_SENTINEL;
            } else {
#pragma unroll
                for (int j = 0; j < GROUP_MAX_LOADS; ++j)
                    if (j < GX::words_per_thread(s)) ok = ok && q.v32[s][j] != STEP_SENTINEL;
            }
        }
        return ok;
    };
    mid();
    int spins = 0;
    for (;;) {
        const bool ok = all_ok(pr) && extra(false);
        // one decision per wavefront (a scalar branch; per-lane loop exits cost ~25 scalar
        // instructions of mask handling per step, and a wavefront issues one instruction every
        // four clocks): a wavefront repeats all its loads while any lane holds a sentinel
        if (__builtin_amdgcn_ballot_w64(!ok) == 0 || dead) break;
        if (++spins > a.spin_limit) { dead = true; if ((tid & 63) == 0) atomicExch(a.ctrl, 1u); break; }
        __builtin_amdgcn_s_sleep(WAVE_RETRY_SLEEP);
        group_poll_issue<MV, NB>(pr, wv, a, t, tid);
        extra(true);
    }
#if defined(RNNG_STEP_TRACE)
    const int trace_step = a.backward ? a.t_end - 1 - t : t - a.t_begin;
    if (blockIdx.x == RNNG_STEP_TRACE - 1 && tid == 0 && trace_step >= RNNG_STEP_TRACE_AT && trace_step < RNNG_STEP_TRACE_AT + 8) {
        reinterpret_cast<unsigned long long*>(a.ctrl + 16)[64 + (trace_step - RNNG_STEP_TRACE_AT)] = spins;
        reinterpret_cast<unsigned long long*>(a.ctrl + 16)[72 + (trace_step - RNNG_STEP_TRACE_AT)] = clock64();
    }
#endif
    group_poll_deliver<MV, NB>(pr, xs, tid);
}

// Sums every p[v] over the 64 lanes.  Pairs of values are folded with the lane-swap
// instructions (upper / lower 32 lanes, then odd / even 16-lane rows), which halves the number
// of registers per level; the last four levels are DPP adds inside the 16-lane rows.  tot[v] is
// wave-uniform.
template <int NV>
__device__ __forceinline__ void wave_reduce_many(const float (&p)[NV], float (&tot)[NV]) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    constexpr int N32 = (NV + 1) / 2, N16 = (N32 + 1) / 2;
    float c[N32], e[N16];
#pragma unroll
    for (int i = 0; i < N32; ++i) {
        const float x = p[2 * i], y = (2 * i + 1 < NV) ? p[2 * i + 1] : p[2 * i];
        const u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
        c[i] = __uint_as_float(r.x) + __uint_as_float(r.y);     // lanes 0-31: x, lanes 32-63: y
    }
#pragma unroll
    for (int j = 0; j < N16; ++j) {
        const float x = c[2 * j], y = (2 * j + 1 < N32) ? c[2 * j + 1] : c[2 * j];
        const u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(y), false, false);
        float v = __uint_as_float(r.x) + __uint_as_float(r.y);  // rows: p[4j], p[4j+2], p[4j+1], p[4j+3]
#define RNNG_DPP(ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, false))
        v += RNNG_DPP(0xB1);
        v += RNNG_DPP(0x4E);
        v += RNNG_DPP(0x141);
        v += RNNG_DPP(0x140);
#undef RNNG_DPP
        e[j] = v;
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int i = v / 2, row = (v % 2) * 2 + (i % 2);
        tot[v] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, e[i / 2]), 16 * row));
    }
}

// Stores of values no other workgroup waits for are issued either right behind the shared stores
// (MV::EARLY: their acknowledgements overlap the exchange) or one step late, after the next step's
// poll, under the matrix-vector part; the generator picks per kernel from measurements.
template <class PH, class MV, int NSTA>
__device__ __forceinline__ void wave_flush_stores(const PhaseRegs<PH>& r, const float (&dfv)[NSTA], const StepArgs& a) {
#pragma unroll
    for (int q = 0; q < PH::NST; ++q)
        if (!PH::stshared(q) || MV::bundled(q)) wave_store<PH, MV>(r, q, dfv[q], 0, a);
}

// One vector per lane into frame t of bundle bs (descriptor over the whole interleaved tensor).
template <class MV>
__device__ __forceinline__ void wave_bundle_store(const WaveRegs<MV>& wv, int bs, const StepArgs& a, int t, const unsigned (&vb)[4], bool through) {
    const __amdgpu_buffer_rsrc_t rs = MV::SW ? __builtin_amdgcn_make_buffer_rsrc(a.store_base, 0, (int)a.store_bytes, STEP_RSRC_FLAGS)
                                             : __builtin_amdgcn_make_buffer_rsrc(wv.bbase[bs], 0, a.T * wv.bstride[bs] * 4, STEP_RSRC_FLAGS);
    const int off = (int)(wv.bvoff[bs] + (unsigned)(t * wv.bstride[bs] * 4));
    if (MV::bs_B(bs) == 4) {
        const muintx4 v4 = {vb[0], vb[1], vb[2], vb[3]};
        if (through) __builtin_amdgcn_raw_buffer_store_b128(v4, rs, off, 0, STEP_COHERENT_AUX);
        else __builtin_amdgcn_raw_buffer_store_b128(v4, rs, off, 0, 0);
    } else {
        const suintx2 v2 = {vb[0], vb[1]};
        if (through) __builtin_amdgcn_raw_buffer_store_b64(v2, rs, off, 0, STEP_COHERENT_AUX);
        else __builtin_amdgcn_raw_buffer_store_b64(v2, rs, off, 0, 0);
    }
}

// The written-through copies of the previous step's values that other groups poll as well
// (xmode 2); t_prev is that step's frame.  advanced: the running store addresses already point
// at the following frame.
template <class PH, class MV, int NSTA>
__device__ __forceinline__ void wave_store_through_late(const PhaseRegs<PH>& r, const WaveRegs<MV>& wv, const float (&dfv)[NSTA],
                                                        const StepArgs& a, int t_prev, bool advanced) {
    if (!wv.local) return;      // they were written through at once
#pragma unroll
    for (int q = 0; q < PH::NST; ++q)
        if (PH::stshared(q) && !MV::bundled(q) && MV::xmode(q) == 2) wave_store<PH, MV>(r, q, dfv[q], 2, a, advanced);
#pragma unroll
    for (int bs = 0; bs < MV::NBS; ++bs) {
        if (MV::bs_xmode(bs) != 2) continue;
        unsigned vb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) vb[j] = (j < MV::bs_B(bs) && MV::bs_q(bs, j) >= 0) ? step_shared_bits(dfv[MV::bs_q(bs, j) >= 0 ? MV::bs_q(bs, j) : 0]) : 0u;
        wave_bundle_store<MV>(wv, bs, a, t_prev, vb, true);
    }
}
template <class MV>
__device__ __forceinline__ constexpr bool wave_has_late_stores() {
    bool any = false;
    for (int q = 0; q < MAX_SLOTS; ++q) any = any || MV::xmode(q) == 2;
    for (int b = 0; b < 4; ++b) any = any || (b < MV::NBS && MV::bs_xmode(b) == 2);
    return any;
}

// PAR is the parity of `step` (the time loop is unrolled by two so that the register pair pf is
// indexed statically: a run-time index would make the compiler merge in-flight loads at the loop
// end, which costs a full memory wait per step).
// HU: 1 for a wavefront that owns units, 0 for one that only helps polling, 2: has_units_rt says
// which (0 / 1 give the unit-owning wavefronts a loop without a branch the compiler cannot see
// through: behind such a branch it cannot count the loads and stores in flight and waits for all
// of them).
// Register-carried values of a call's first step: the previous frame's, if the window has one
// (before the time loop, so that no step has a load behind a branch).
template <class PH>
__device__ __forceinline__ void wave_carry_init(PhaseRegs<PH>& r, const StepArgs& a) {
    const int t = step_frame(a, 0);
#pragma unroll
    for (int g = 0; g < PH::NG; ++g) {
        if (PH::gkind(g) == GA_KIND_CARRY) {
            const int frame = t + r.goff[g];
            r.carry[PH::cidx(g)] = (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) ? r.gptr[g][(long long)frame * r.gstride[g]] : 0.0f;
        }
        if (PH::gkind(g) == GA_KIND_POLLED) {      // the first step's: checked (and loaded again if need be) like every step's
            const int frame = t + r.goff[g];
            r.polled_next[g] = (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) ? load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]) : 0.0f;
        }
    }
}

template <class PH, class MV, int NB, int PAR, int HU, int QNA, int NSTA>
__device__ __forceinline__ void wave_step(PhaseRegs<PH>& r, const WaveRegs<MV>& wv, const WaveRing<PH, MV, NB>& rg,
                                          float (&pf)[2][QNA], float (&dfv)[NSTA], PollRegs<MV>& pr,
                                          const StepArgs& a, float* ring, float* xs_all, bool has_units_rt, int step, int t, int tid,
                                          bool& dead) {
    const bool has_units = HU == 2 ? has_units_rt : HU != 0;
    typedef WaveRing<PH, MV, NB> RG;
    typedef GroupX<MV, NB> GX;
    const int lane = tid & 63;
    float s[MAX_SLOTS];
    RNNG_STAMP(0);
    const int js = step & (WAVE_RING_STEPS - 1);
    const int ul_l = lane % MV::UW, n_l = lane / MV::UW;
    auto gathers = [&]() {
        // the row loaded two steps ago (for step - 2 + WAVE_RING_STEPS) goes into the ring now
        if (PH::NS > 0 && has_units && step > 1) wave_ring_store<PH, MV, NB, QNA>(pf[PAR], rg, a, ring, step - 2 + WAVE_RING_STEPS, lane);
#pragma unroll
        for (int g = 0; g < PH::NG; ++g) {
            if (PH::gkind(g) == GA_KIND_CARRY) {
                s[g] = r.carry[PH::cidx(g)];      // the first step's: wave_carry_init
            } else if (PH::gkind(g) == GA_KIND_STATIC) {
                // idle lanes read a valid (unused) ring entry instead of branching around the load
                const int item = (n_l * MV::UW + ul_l) < RG::ITEMS ? (n_l * MV::UW + ul_l) : 0;
                s[g] = ring[js * RG::PAIRS + PH::sidx(g) * RG::ITEMS + item];
            } else if (PH::gkind(g) == GA_KIND_FRAMES) {
                const int frame = t + r.goff[g];
                float v = 0.0f;
                if (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) v = load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]);
                s[g] = v;
            } else if (PH::gkind(g) == GA_KIND_POLLED) {
                // a helper group's sum for this frame, loaded one step ahead (the helper runs ahead; the
                // value is checked with the poll's attempts)
                s[g] = r.polled_next[g];
            }
        }
#pragma unroll
        for (int v = 0; v < PH::NI; ++v) s[PH::NG + v] = r.inv[v];
    };
    // a helper group's sums (POLLED gathers, loaded by gathers()): arrived? / load them again
    auto polled_sums = [&](bool reload) {
        bool ok = true;
#pragma unroll
        for (int g = 0; g < PH::NG; ++g) {
            if (PH::gkind(g) == GA_KIND_POLLED) {
                if (reload && has_units) {
                    const int frame = t + r.goff[g];
                    if (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) s[g] = load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]);
                }
                ok = ok && (!has_units || __float_as_uint(s[g]) != STEP_SENTINEL);
            }
        }
        return ok;
    };
    // the next step's sums go out behind this step's poll (behind the last step: a frame that nothing
    // reads).  In front of the poll they cost more than they gain: the poll's check waits for every
    // load in flight, also for these, which come from another XCD (charlm_n1 1.77 against 1.68 ms).
    auto polled_ahead = [&]() {
        if (!has_units) return;
#pragma unroll
        for (int g = 0; g < PH::NG; ++g)
            if (PH::gkind(g) == GA_KIND_POLLED) {
                const int frame = step_frame(a, step + 1) + r.goff[g];
                float v = 0.0f;
                if (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) v = load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]);
                r.polled_next[g] = v;
            }
    };
    float xr[NB][MV::XF > 0 ? MV::XF : 1];
    if (MV::NSRC == 0) { gathers(); polled_ahead(); }
    RNNG_STAMP(1);
    if (MV::NSRC > 0) {
        float* xs = xs_all + PAR * GX::FLOATS;
        if (!MV::PE) group_poll_issue<MV, NB>(pr, wv, a, t, tid);
        group_poll<MV, NB>(pr, xs, wv, a, step, t, tid, dead, gathers, polled_sums);
        polled_ahead();
        step_lds_barrier();
#if defined(RNNG_STEP_TRACE)
        if (blockIdx.x == RNNG_STEP_TRACE - 1 && tid == 0 && step >= RNNG_STEP_TRACE_AT && step < RNNG_STEP_TRACE_AT + 8) reinterpret_cast<unsigned long long*>(a.ctrl + 16)[80 + (step - RNNG_STEP_TRACE_AT)] = clock64();
#endif
        if (!has_units) {
            if (MV::PE) group_poll_issue<MV, NB>(pr, wv, a, step_frame(a, step + 1), tid);
            return;
        }
#pragma unroll
        for (int sidx = 0; sidx < MV::NSRC; ++sidx)
#pragma unroll
            for (int n = 0; n < NB; ++n)
#pragma unroll
                for (int f = 0; f < WAVE_FMAX; ++f)
                    if (f < MV::F(sidx)) xr[n][MV::xoff(sidx) + f] = xs[GX::lane_pos(sidx, n, lane, f)];
    } else if (!has_units) {
        return;
    }
    RNNG_STAMP(2);
    if (wave_has_late_stores<MV>() && step > 0) wave_store_through_late<PH, MV>(r, wv, dfv, a, step_frame(a, step - 1), MV::EARLY != 0);
    // the previous step's deferred stores, then the ring row of step + WAVE_RING_STEPS (stored next step)
    if (!MV::EARLY && step > 0) {
        wave_flush_stores<PH, MV>(r, dfv, a);
        wave_store_advance<PH>(r);
    }
    if (PH::NS > 0) wave_ring_load<PH, MV, NB, QNA>(pf[PAR], rg, a, step + WAVE_RING_STEPS);
    // rows: partial dot products, cross-lane reduction, result picked by the owning item lane
    constexpr int NV = (MV::UW * MV::NT * NB) > 0 ? (MV::UW * MV::NT * NB) : 1;
    float part[NV], tot[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) part[v] = 0.0f;
#pragma unroll
    for (int ul = 0; ul < MV::UW; ++ul) {
#pragma unroll
        for (int task = 0; task < MV::NT; ++task) {
#pragma unroll
            for (int n = 0; n < NB; ++n) {
                float p = 0.0f;
#pragma unroll
                for (int e = 0; e < STEP_MAX_EDGES; ++e) {
                    if (e < MV::nedges(task)) {
                        const int sidx = MV::esrc(task, e);
#pragma unroll
                        for (int f = 0; f < WAVE_FMAX; ++f)
                            if (f < MV::F(sidx)) p = fmaf(wv.wr[MV::woff(ul, task, e) + f], xr[n][MV::xoff(sidx) + f], p);
                    }
                }
                part[(ul * MV::NT + task) * NB + n] = p;
            }
        }
    }
    float acc[MV::NT > 0 ? MV::NT : 1];
#pragma unroll
    for (int task = 0; task < (MV::NT > 0 ? MV::NT : 1); ++task) acc[task] = 0.0f;
    if (MV::NT > 0) {
        wave_reduce_many<NV>(part, tot);
#pragma unroll
        for (int ul = 0; ul < MV::UW; ++ul)
#pragma unroll
            for (int task = 0; task < MV::NT; ++task)
#pragma unroll
                for (int n = 0; n < NB; ++n)
                    if (ul_l == ul && n_l == n) acc[task] = tot[(ul * MV::NT + task) * NB + n];
    }
    RNNG_STAMP(3);
#pragma unroll
    for (int g = 0; g < PH::NG; ++g)
        if (PH::gkind(g) == GA_KIND_ACC) s[g] = acc[PH::gaux(g)];
    // (a component without sources of its own checks a helper group's sums here; the others did in their poll)
    if (MV::NSRC == 0) {
        int spins = 0;
        while (__builtin_amdgcn_ballot_w64(!polled_sums(false)) != 0 && !dead) {
            if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
            polled_sums(true);
        }
    }
    PH::ops(s);
    RNNG_STAMP(4);
#pragma unroll
    for (int q = 0; q < PH::NST; ++q) {
        if (PH::stshared(q) && !MV::bundled(q)) {
            const bool through = MV::xmode(q) == 1 || !wv.local;
            wave_store<PH, MV>(r, q, s[PH::stslot(q)], through ? 2 : 1, a);
            if (MV::xmode(q) == 2) dfv[q] = s[PH::stslot(q)];      // written through one step late
        } else {
            dfv[q] = s[PH::stslot(q)];
        }
    }
    // bundles: one coherent vector store per lane (lanes without an item store outside the descriptor)
#pragma unroll
    for (int bs = 0; bs < MV::NBS; ++bs) {
        unsigned vb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) vb[j] = (j < MV::bs_B(bs) && MV::bs_q(bs, j) >= 0) ? step_shared_bits(s[PH::stslot(MV::bs_q(bs, j) >= 0 ? MV::bs_q(bs, j) : 0)]) : 0u;
        wave_bundle_store<MV>(wv, bs, a, t, vb, MV::bs_xmode(bs) == 1 || !wv.local);
    }
    if (MV::EARLY) {
        // the other stores right behind the shared ones: their acknowledgements overlap the exchange
        wave_flush_stores<PH, MV>(r, dfv, a);
        wave_store_advance<PH>(r);
    }
#pragma unroll
    for (int g = 0; g < PH::NG; ++g)
        if (PH::gkind(g) == GA_KIND_CARRY) r.carry[PH::cidx(g)] = s[PH::gaux(g)];
    // PE: the next step's first polling attempt goes out right behind this step's stores (after
    // the launch's last step it polls a frame nobody waits for, or none: nothing checks what it
    // returns); otherwise at the start of the next step
    if (MV::NSRC > 0 && MV::PE) group_poll_issue<MV, NB>(pr, wv, a, step_frame(a, step + 1), tid);
    RNNG_STAMP(5);
    RNNG_STAMP(6);
    RNNG_STAMP(7);
}


// =============================================================================================
// Matrix-core variant (run-time specialised, single-phase components, many streams).
//
// With N >= 9 streams a step's full connections are skinny GEMMs: acc[n][row] = sum_s sum_k
// x_s[n][k] * W_s[row][k] over the shared source tensors x_s [N][K_s], row = task * cmax + local
// unit.  Each workgroup owns a chunk of every layer's units and keeps its weight rows on chip: in
// LDS (per source one block of cmax rows for every task the source feeds; a task the source does
// not feed reads a shared row of zeros), and whole sources that do not fit there in vector
// registers (MM::REGMASK).  Per step every wavefront polls its own share of each source's columns
// (sentinel protocol) with 128-bit coherent loads that ARE the A operands of
// v_mfma_f32_16x16x4_f32: lane (m, q) of a wavefront loads x[16 mt + m][c + 4 q .. c + 4 q + 3]
// and feeds word j of it to the j-th of four multiply steps, whose B operand is word j of the
// 128-bit read W[row][c + 4 q ..] (the order in which a dot product's columns are summed is
// free).  Nothing of x passes through LDS and the wavefronts do not wait for each other inside a
// step's contraction: chunks of 16 * NW columns (16 per wavefront; NW = 4 or 8 wavefronts: what a
// workgroup can poll per microsecond grows with the wavefronts that have loads in flight, measured
// 43 / 79 / 94 GB/s with 4 / 8 / 16) are in flight in D register sets, and a chunk that comes back
// with a sentinel is loaded again by the wavefront that needs it.  With MM::XB the sources are
// the tile-blocked twins of the exchanged tensors (a wavefront's load is 1 KiB of consecutive
// addresses: 77 instead of 35 GB/s per workgroup).  One accumulator set serves all sources; the
// NW partial tiles meet in LDS, where the element-wise program runs with one thread per
// (stream, unit) on the first STEP_THREADS threads.
//
// MM is a generated descriptor:
//   static constexpr int NJ (streams per workgroup), MT (16-stream tiles), NSRC, NTU (16-row
//   tiles), D (register sets of chunks), CMAX, ACCS (row stride of an accumulator tile), NW
//   (wavefronts), NCH (chunks of all sources), CLATE (first chunk that holds the previous step's
//   own values), NRW (weight quads in registers); bool FLAT (the chunk sequence is unrolled whole),
//   XB, HELPER (a chain's helper member: its program only stores the sums of its products, which
//   another member's program polls element by element); unsigned REGMASK; constexpr K(s), ngr(s) (groups of D chunks of source s), blk(s, task)
//   (row block of the task in source s, -1: none), used(s, nt), csrc(c) / ck0(c) (source and first
//   column of chunk c), widx(c * 16 + nt) (register index of a weight quad).
// =============================================================================================

#if !defined(MSTEP_POLL_INC)
#define MSTEP_POLL_INC 2      // 0 switches the adaptive hold-off of the first loads off
#endif
#if !defined(MSTEP_RETRY_SLEEP)
#define MSTEP_RETRY_SLEEP 0      // units of 64 clocks; measured: backing off only costs time
#endif
template <int V> struct StepIntC { static constexpr int value = V; };
template <int C, int N, class F>
__device__ __forceinline__ void step_static_for(F&& f) {
    if constexpr (C < N) { f(StepIntC<C>{}); step_static_for<C + 1, N>(f); }
}

struct MLayout {
    int ok, n_src, cmax, zrow, accbase, accstride, total_floats;
    int wbase[STEP_MAX_SOURCES], wstride[STEP_MAX_SOURCES], rows[STEP_MAX_SOURCES];
    short blk[STEP_MAX_SOURCES][STEP_MAX_TASKS];     // row block of (source, task) or -1
};

// Same on host and device.  lay is the generic step layout (tasks, sources) for G workgroups.
// nw: wavefronts per workgroup (4 or 8); a chunk of a source is 16 * nw columns, 16 per wavefront.
// reg_mask: bit s set = the weight rows of source s live in vector registers, not in LDS.
RNNG_HD inline void compute_mstep_layout(const StepLayout& lay, int N, int nw, unsigned reg_mask, int lds_limit_floats, MLayout& m) {
    m.ok = 0;
    const int cw = 16 * nw;
    if (!lay.ok || lay.n_phases != 1 || lay.n_sources < 1) return;
    const StepPhase& ph = lay.ph[0];
    if (ph.item_chunk * N > STEP_THREADS) return;
    m.n_src = lay.n_sources; m.cmax = ph.cmax;
    const int npad = (N + 15) / 16 * 16;
    for (int s = 0; s < lay.n_sources; ++s)
        if (lay.src[s].k_len & 3) return;               // rows are read with 128-bit loads
    int cur = 0, wsmax = 0;
    for (int s = 0; s < lay.n_sources; ++s) {
        int nb = 0;
        for (int t = 0; t < STEP_MAX_TASKS; ++t) {
            m.blk[s][t] = -1;
            if (t >= ph.n_tasks) continue;
            for (int e = 0; e < ph.task[t].n_edges; ++e)
                if (ph.task[t].e[e].src == s && m.blk[s][t] < 0) m.blk[s][t] = (short)nb++;
        }
        m.rows[s] = nb * ph.cmax;
        m.wstride[s] = (lay.src[s].k_len + cw - 1) / cw * cw + 4;      // zero-padded to whole chunks; = 4 (mod 32): conflict-free 128-bit reads
        m.wbase[s] = cur;
        if ((reg_mask >> s) & 1) continue;
        wsmax = m.wstride[s] > wsmax ? m.wstride[s] : wsmax;
        cur += m.rows[s] * m.wstride[s];
    }
    m.zrow = cur; cur += wsmax;
    const int ntu = (ph.n_tasks * ph.cmax + 15) / 16;
    m.accstride = ntu * 16 + 4;                         // = 4 (mod 16): conflict-free tile rows
    m.accbase = cur; cur += nw * npad * m.accstride;    // one partial tile per wavefront
    if (cur > lds_limit_floats) return;
    m.total_floats = cur;
    m.ok = 1;
}

// With RNNG_STORE_WINDOW (the workspace fits 2 GiB) the element-wise loads and stores of the
// matrix-core build all go through ONE descriptor over the workspace, else through one per tensor:
// with 13 stores and 8 loads per step the descriptors' scalar work was a third of the
// element-wise part's instructions and spilled scalar registers.
struct MStore { static constexpr bool SW = RNNG_STORE_WINDOW != 0; };
// (leaner than StepShared: one phase, so that more of the 160 KiB is left for weight rows)
struct MShared { StepLayout lay; unsigned iteminfo[1][STEP_THREADS]; MLayout ml; unsigned retried[2]; };

template <class PH, class MM>
// w: index of this workgroup among the a.G * a.J workgroups of the component.
__device__ __forceinline__ void mstep_kernel_body(const StepArgs& a, MShared& ms, float* lds, int w) {
    if (w < 0 || w >= a.G * a.J) return;
    const int wj = w / a.G;      // stream group
    w -= wj * a.G;               // unit chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = a.T;
    const int n0 = wj * MM::NJ;                                            // first stream of this workgroup
    const int N = a.N - n0 < MM::NJ ? a.N - n0 : MM::NJ;                   // its streams
    MShared& sh = ms;
    constexpr int NW = MM::NW, NTHR = 64 * NW, CW = 16 * NW;      // wavefronts, threads, columns of a chunk
    if (tid == 0) { compute_step_layout(a.words, a.desc_off, a.G, 1, MM::NJ, sh.lay); compute_mstep_layout(sh.lay, MM::NJ, NW, MM::REGMASK, (int)(MSTEP_LDS_LIMIT / 4), ms.ml); }
    __syncthreads();
    const StepPhase& ph = sh.lay.ph[0];
    const MLayout& ml = ms.ml;
    if (tid < STEP_THREADS) {      // the element-wise items sit on the first STEP_THREADS threads
        const int ic = ph.item_chunk;
        const int il = tid % ic, n = tid / ic;
        sh.iteminfo[0][tid] = (unsigned)il | ((unsigned)(n < N ? n0 + n : 0xFFFF) << 16);      // global stream index
    }
    for (int i = tid; i < ml.total_floats; i += NTHR) lds[i] = 0.0f;
    if (tid < 2) ms.retried[tid] = 0u;
    __syncthreads();
    // resident weights: W_lds[s][blk(s, task) * cmax + ul][k]; edges of one task that share a
    // source add up in one row
    constexpr int CMAX = MM::CMAX;
    for (int s = 0; s < ml.n_src; ++s) {
        if ((MM::REGMASK >> s) & 1) continue;      // (in registers, below)
        const int K = sh.lay.src[s].k_len;
        for (int t = 0; t < ph.n_tasks; ++t) {
            const StepTask& task = ph.task[t];
            for (int e = 0; e < task.n_edges; ++e) {
                const StepEdge ed = task.e[e];
                if (ed.src != s) continue;
                const float* W = a.weights + ed.w_off;
                for (int i = tid; i < CMAX * K; i += NTHR) {
                    const int ul = i / K, k = i - ul * K;
                    const int u = w * task.chunk + ul;
                    float v = 0.0f;
                    if (ul < task.chunk && u < task.n_out) v = ed.transposed ? W[(size_t)k * task.n_out + u] : W[(size_t)u * K + k];
                    lds[ml.wbase[s] + (ml.blk[s][t] * CMAX + ul) * ml.wstride[s] + k] += v;
                }
                __syncthreads();
            }
        }
    }
    PhaseRegs<PH> r;
    phase_setup<PH, 1, 2>(r, a, sh, lds, w, tid);
    __syncthreads();

    constexpr int D = MM::D, NPAD = MM::MT * 16, ACCS = MM::ACCS;
    const int accbase = suni(ml.accbase);
    const int item_il = tid < STEP_THREADS ? (int)(sh.iteminfo[0][tid] & 0xFFFF) : 0;
    const int item_n = tid / suni(ph.item_chunk);                          // local stream of this thread's item
    // LDS address of the weight row behind each of this lane's tile columns, per source
    int brow[MM::NSRC][MM::NTU];
#pragma unroll
    for (int sidx = 0; sidx < MM::NSRC; ++sidx)
#pragma unroll
        for (int nt = 0; nt < MM::NTU; ++nt) {
            const int col = nt * 16 + (lane & 15);
            const int task = col / CMAX, ul = col - task * CMAX;
            int b = -1;
#pragma unroll
            for (int t2 = 0; t2 < STEP_MAX_TASKS; ++t2) if (task == t2) b = MM::blk(sidx, t2);
            brow[sidx][nt] = (b >= 0 ? suni(ml.wbase[sidx]) + (b * CMAX + ul) * suni(ml.wstride[sidx]) : suni(ml.zrow)) + 4 * (lane >> 4);
        }
    // Weight rows that do not fit LDS stay in vector registers for the whole launch (sources in
    // MM::REGMASK; only with the unrolled chunk sequence, where every register index is static):
    // for chunk c and row tile nt this lane keeps the four words it would read from LDS, i.e. the
    // B operands of the chunk's four multiply steps, W[row of (nt, lane & 15)][k0 + 16 wave +
    // 4 (lane >> 4) ...].  Edges of one task that share the source add up.
    // The workgroups of an XCD poll the same lines of its L2 at about the same time.  With the
    // unrolled chunk sequence every workgroup therefore walks a source's chunks from a place of its
    // own (rank inside the XCD; chunk c of the sequence stands for columns rot(sidx, k0) ...), which
    // spreads the requests over the L2's channels (stand-alone probe: 10 to 28 % more polled bytes
    // per microsecond).  The order of the sources stays.  Kept for components with several sources
    // (measured: charlm_n32 3.68 -> 3.54 ms per window, generalized_n64 14.22 -> 14.15); a layer
    // with one source ran 3 % slower with it (fig4_h2048_n16).
#if !defined(MSTEP_ROTATE)
#define MSTEP_ROTATE 1
#endif
    int krot[MM::NSRC];
#pragma unroll
    for (int sidx = 0; sidx < MM::NSRC; ++sidx) {
        const int nch = (MM::K(sidx) + CW - 1) / CW;
        krot[sidx] = MM::FLAT && MSTEP_ROTATE && MM::NSRC > 1 ? suni((int)((blockIdx.x >> 3) & 31) * nch / 32 * CW) : 0;
    }
    auto rot = [&](auto ss, int k0) {
        constexpr int sidx = decltype(ss)::value;
        constexpr int KP = (MM::K(sidx) + CW - 1) / CW * CW;
        const int kk = k0 + krot[sidx];
        return kk >= KP ? kk - KP : kk;
    };
    mfloatx4 wr[MM::NRW > 0 ? MM::NRW : 1];
    if constexpr (MM::NRW > 0) {
        step_static_for<0, MM::NCH>([&](auto cc) {
            constexpr int c = decltype(cc)::value, sidx = MM::csrc(c);
            const int k0 = rot(StepIntC<sidx>{}, MM::ck0(c));
            if constexpr (((MM::REGMASK >> sidx) & 1) != 0) {
                step_static_for<0, MM::NTU>([&](auto tt) {
                    constexpr int nt = decltype(tt)::value;
                    if constexpr (MM::used(sidx, nt)) {
                        const int col = nt * 16 + (lane & 15);
                        const int task = col / CMAX, ul = col - task * CMAX;
                        const int kk = k0 + wave * 16 + 4 * (lane >> 4);
                        mfloatx4 wv = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (task < ph.n_tasks) {
                            const StepTask& tk = ph.task[task];
                            const int u = w * tk.chunk + ul;
                            for (int e = 0; e < tk.n_edges; ++e) {
                                const StepEdge ed = tk.e[e];
                                if (ed.src != sidx || ul >= tk.chunk || u >= tk.n_out) continue;
                                const float* W = a.weights + ed.w_off;
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (kk + j < MM::K(sidx)) wv[j] += ed.transposed ? W[(size_t)(kk + j) * tk.n_out + u] : W[(size_t)u * MM::K(sidx) + kk + j];
                            }
                        }
                        wr[MM::widx(c * 16 + nt)] = wv;
                    }
                });
            }
        });
    }
    // this lane's A-operand element inside a chunk: stream 16 mt + (lane & 15), columns wcol ... wcol + 3;
    // its byte offset in chunk 0 of each source (a stream beyond N: outside the descriptor)
    // With tile-blocked exchange (MM::XB) the source is the tensor's twin, whose 16 x 16 tiles
    // [(unit % 16) / 4][stream % 16][unit % 4] are 1 KiB of consecutive addresses each: the
    // wavefront's load of a tile is lane l -> bytes 16 l, and the tiles of a stream tile's
    // column blocks follow each other.
    const int wcol = wave * 16 + 4 * (lane >> 4);
    int aoff[MM::NSRC][MM::MT];
#pragma unroll
    for (int sidx = 0; sidx < MM::NSRC; ++sidx)
#pragma unroll
        for (int mt = 0; mt < MM::MT; ++mt) {
            const int n = mt * 16 + (lane & 15);
            if (MM::XB) aoff[sidx][mt] = ((mt * (MM::K(sidx) / 16) + wave) * 256 + lane * 4) * 4;
            else aoff[sidx][mt] = n < N ? (n * MM::K(sidx) + wcol) * 4 : 0x7FFFFFF0;
        }

    // Stores go through one buffer descriptor per stored tensor with a running per-lane offset
    // (a lane without an element is parked outside the tensor), gathers read a harmless address
    // where a lane has nothing to load: the time loop has no load or store behind a per-lane
    // branch, so the compiler can count what is in flight instead of waiting for all of it.
    wave_store_setup<PH, MStore>(r, a);
    wave_carry_init<PH>(r, a);
    if constexpr (MStore::SW) {      // gather offsets relative to the window (parked lanes stay outside)
#pragma unroll
        for (int g = 0; g < PH::NG; ++g)
            if (PH::gkind(g) != GA_KIND_ACC && r.gvoff[g] != 0xC0000000u) r.gvoff[g] += (unsigned)((r.gbase[g] - a.store_base) * 4);
    }
    // tile-blocked exchange: the exchanged values are stored a second time, written through, into
    // the twins (the row-major copies, which nobody polls, are then stored plainly)
    const float* xbase[PH::NST > 0 ? PH::NST : 1];
    unsigned xvrun[PH::NST > 0 ? PH::NST : 1];
    if constexpr (MM::XB) {
        cwords_t pw = (cwords_t)a.words + suni(ph.prog_off);
        cwords_t st = pw + PG_HEADER_WORDS + PH::NG * GA_WORDS + PH::NI * IV_WORDS + pw[PG_NOPS] * MO_WORDS;
#pragma unroll
        for (int q = 0; q < PH::NST; ++q) {
            xbase[q] = nullptr; xvrun[q] = WAVE_NO_STORE;
            if (!PH::stshared(q) || !PH::sttwin(q)) continue;
            const int dim = suni(st[q * ST_WORDS + ST_DIM]);
            xbase[q] = suni_ptr(((cbufs_t)a.buf_ptr)[a.twin_base + suni(st[q * ST_WORDS + ST_BUF])]);
            if (r.sptr[q] != nullptr) {
                const int i = (int)(r.sptr[q] - r.sbase[q]) - r.n * dim;      // this thread's unit
                const int off = ((r.n >> 4) * (dim >> 4) + (i >> 4)) * 256 + ((((i & 15) >> 2) << 4) + (r.n & 15)) * 4 + (i & 3);
                xvrun[q] = (unsigned)((off + step_frame(a, 0) * r.sstride[q]) * 4);
                if (MStore::SW) xvrun[q] += (unsigned)((xbase[q] - a.store_base) * 4);
            }
        }
    }
    const bool wave_items = __builtin_amdgcn_ballot_w64(r.n >= 0) != 0;      // wavefronts without items skip the element-wise part
    const int item_n_safe = r.n >= 0 ? item_n : 0;
    // value of gather g (STATIC or FRAMES kind) at `frame`; zero outside the window or for an idle
    // lane (a buffer load outside the descriptor's range)
    auto gather_at = [&](auto gg, int frame) -> float {
        constexpr int g = decltype(gg)::value;
        const bool in_window = frame >= 0 && frame < T;
        const __amdgpu_buffer_rsrc_t rg = MStore::SW ? __builtin_amdgcn_make_buffer_rsrc(a.store_base, 0, (int)a.store_bytes, STEP_RSRC_FLAGS)
                                                     : __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(r.gbase[g]), 0, T * r.gstride[g] * 4, STEP_RSRC_FLAGS);
        const int off = in_window ? (int)(r.gvoff[g] + (unsigned)(frame * r.gstride[g] * 4)) : (int)WAVE_NO_STORE;
        return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rg, off, 0, PH::gkind(g) == GA_KIND_STATIC ? 0 : STEP_COHERENT_AUX));
    };

    bool dead = false;
    int pdelay = 0;
    float sn[PH::NG > 0 ? PH::NG : 1];      // STATIC inputs of the next step, loaded one step ahead
    const int nsteps = step_count(a);
    if (wave_items && nsteps > 0)
        step_static_for<0, PH::NG>([&](auto gg) {
            constexpr int g = decltype(gg)::value;
            if (PH::gkind(g) == GA_KIND_STATIC) sn[g] = gather_at(gg, step_frame(a, 0) + r.goff[g]);
        });
    for (int step = 0; step < nsteps; ++step) {
        const int t = step_frame(a, step);
        float s[MAX_SLOTS];
        RNNG_STAMP(0);
        // element-wise inputs from the thread's own earlier frames: coherent loads, issued first
        if (wave_items)
            step_static_for<0, PH::NG>([&](auto gg) {
                constexpr int g = decltype(gg)::value;
                if (PH::gkind(g) == GA_KIND_FRAMES || PH::gkind(g) == GA_KIND_POLLED) s[g] = gather_at(gg, t + r.goff[g]);
            });
        RNNG_STAMP(1);

        // one buffer descriptor per source tensor; a frame outside the window gets an empty one
        // (all its loads return zeros, which pass the sentinel check and contribute nothing)
        __amdgpu_buffer_rsrc_t rs[MM::NSRC];
#pragma unroll
        for (int sidx = 0; sidx < MM::NSRC; ++sidx) {
            const StepSource& sc = sh.lay.src[sidx];
            const int frame = t + suni(sc.frame_off);
            const bool in_window = frame >= 0 && frame < T;
            // (a twin's frame has the same size, and its stream tiles are as large as 16 rows)
            const float* g = ((cbufs_t)a.buf_ptr)[(MM::XB ? a.twin_base : 0) + suni(sc.buf)] + ((size_t)(in_window ? frame : 0) * a.N + n0) * MM::K(sidx);
            rs[sidx] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(g), 0, in_window ? N * MM::K(sidx) * 4 : 0, STEP_RSRC_FLAGS);
        }
        // A helper member has no values of its own to wait for and would otherwise poll each frame
        // of its sources while the producing member's stores are still under way, which slows that
        // member's own exchange.  It therefore starts a step only when the frame of the NEXT step
        // shows its first value: the producers have then consumed, hence seen, all of this step's
        // frame, and every load below succeeds at once.  (The last step has no next frame.)
        if constexpr (MM::HELPER) {
            if (step + 1 < nsteps) {
                const StepSource& sc = sh.lay.src[0];
                const int frame = step_frame(a, step + 1) + suni(sc.frame_off);
                if (frame >= 0 && frame < T) {
                    const float* p = ((cbufs_t)a.buf_ptr)[(MM::XB ? a.twin_base : 0) + suni(sc.buf)] + ((size_t)frame * a.N + n0) * MM::K(0);
                    int spins = 0;
                    while (__float_as_uint(load_coherent(p)) == STEP_SENTINEL && !dead) {
                        if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
                        __builtin_amdgcn_s_sleep(8);
                    }
                }
            }
        }
        // ---- chunk pipeline ----
        // The sources' columns form one sequence of chunks of CW columns (a source's last chunk
        // zero-padded).  D register sets hold D - 1 chunks in flight: while chunk c is multiplied,
        // the set of chunk c - 1 takes the loads of chunk c + D - 1 and chunk c + 1 is tested for
        // sentinels.  These three run in one basic block, so that the compiler can place the loads
        // and the test between the matrix instructions, where the wavefront would otherwise idle.
        // Short sequences (MM::FLAT) are unrolled whole, so that the chunks in flight may span any
        // number of sources; long ones run source by source in groups of D chunks (the last group
        // of a source padded with empty chunks that are skipped; loads that have nothing to fetch
        // get an offset outside the descriptor instead of a branch), which looks ahead into the
        // next source's first group only.
        muintx4 v[D][MM::MT];
        // This lane's operands of the chunk with first column k0 of source S (on: else nothing is
        // fetched).  Columns beyond K read as zeros; they exist only if K is no multiple of CW.
        auto load_chunk = [&](muintx4 (&dst)[MM::MT], const __amdgpu_buffer_rsrc_t& rsrc, const int (&base)[MM::MT], int K, bool k_ragged, int k0, bool on) {
#pragma unroll
            for (int mt = 0; mt < MM::MT; ++mt) {
                int off = base[mt] + (MM::XB ? k0 * 64 : k0 * 4);      // (blocked: k0 / 16 tiles of 1 KiB further)
                if (k_ragged) off = k0 + (MM::XB ? wave * 16 : wcol) < K ? off : 0x7FFFFFF0;
                off = on ? off : 0x7FFFFFF0;
                dst[mt] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, STEP_COHERENT_AUX);
            }
        };
        // true if some element of the chunk still shows the sentinel (same in all lanes)
        auto incomplete = [&](const muintx4 (&x)[MM::MT]) {
            unsigned m = 0;
#pragma unroll
            for (int mt = 0; mt < MM::MT; ++mt) {
                const unsigned m1 = x[mt].x > x[mt].y ? x[mt].x : x[mt].y, m2 = x[mt].z > x[mt].w ? x[mt].z : x[mt].w;
                const unsigned m3 = m1 > m2 ? m1 : m2;
                m = m > m3 ? m : m3;
            }
            return __builtin_amdgcn_ballot_w64(m == STEP_SENTINEL) != 0;
        };
        bool retried = false;
        // the retry loads into registers of its own (a reload of the pipelined set would make
        // every later use of it wait for all loads in flight)
        auto reload = [&](muintx4 (&dst)[MM::MT], auto ss, int k0) {
            constexpr int sidx = decltype(ss)::value;
            retried = true;
            muintx4 again[MM::MT];
            int spins = 0;
            for (;;) {
                if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
                __builtin_amdgcn_s_sleep(MSTEP_RETRY_SLEEP);
                step_compiler_barrier();
                load_chunk(again, rs[sidx], aoff[sidx], MM::K(sidx), MM::K(sidx) % CW != 0, k0, true);
                if (!incomplete(again)) break;
            }
#pragma unroll
            for (int mt = 0; mt < MM::MT; ++mt) dst[mt] = again[mt];
        };
        mfloatx4 acc[MM::MT][MM::NTU];
        // chunk in register set `set` (first column k0 of source sidx) times the resident weights
        auto multiply = [&](auto ss, const muintx4 (&x)[MM::MT], const mfloatx4 (&opb)[MM::NTU]) {
            constexpr int sidx = decltype(ss)::value;
#pragma unroll
            for (int mt = 0; mt < MM::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MM::NTU; ++nt)
                    if (MM::used(sidx, nt)) {
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(x[mt].x), opb[nt][0], acc[mt][nt], 0, 0, 0);
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(x[mt].y), opb[nt][1], acc[mt][nt], 0, 0, 0);
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(x[mt].z), opb[nt][2], acc[mt][nt], 0, 0, 0);
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(x[mt].w), opb[nt][3], acc[mt][nt], 0, 0, 0);
                    }
        };
        // The loads of what the other workgroups produced in the step before are held back until
        // those stores are usually visible (a first attempt that comes back with a sentinel costs a
        // whole extra round trip); chunks in front of them (MM::CLATE) are not.
        // (With the unrolled sequence, where the multiplications of the early chunks fill that time,
        // holding back measured slower than retrying: charlm_n32 forward 1.26 against 0.89 ms.)
        constexpr int POLL_INC = MM::FLAT ? 0 : MSTEP_POLL_INC;
        auto hold_off = [&]() { for (int i = 0; i < pdelay; ++i) __builtin_amdgcn_s_sleep(1); };
        if constexpr (MM::FLAT) {
            constexpr int NCH = MM::NCH;
            step_static_for<0, D - 1>([&](auto ii) {
                constexpr int i = decltype(ii)::value;
                constexpr int sx = MM::csrc(i < NCH ? i : 0);
                if (i == MM::CLATE) hold_off();
                load_chunk(v[i], rs[sx], aoff[sx], MM::K(sx), MM::K(sx) % CW != 0, rot(StepIntC<sx>{}, MM::ck0(i < NCH ? i : 0)), i < NCH);
            });
#pragma unroll
            for (int mt = 0; mt < MM::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MM::NTU; ++nt) acc[mt][nt] = mfloatx4{0.0f, 0.0f, 0.0f, 0.0f};
            bool bad = incomplete(v[0]);      // of the chunk that comes next
            step_static_for<0, NCH>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                constexpr int i = c % D, j = (c + D - 1) % D, i1 = (c + 1) % D;
                constexpr int sidx = MM::csrc(c);
                const int k0 = rot(StepIntC<sidx>{}, MM::ck0(c));
                constexpr int ca = c + D - 1 < NCH ? c + D - 1 : 0;      // the chunk D - 1 positions ahead, if any
                constexpr int sa = MM::csrc(ca);
                mfloatx4 opb[MM::NTU];
                step_static_for<0, MM::NTU>([&](auto tt) {
                    constexpr int nt = decltype(tt)::value;
                    if constexpr (MM::used(sidx, nt)) {
                        if constexpr (((MM::REGMASK >> sidx) & 1) != 0) opb[nt] = wr[MM::widx(c * 16 + nt)];
                        else opb[nt] = *reinterpret_cast<const mfloatx4*>(&lds[brow[sidx][nt] + k0 + wave * 16]);
                    }
                });
                if (bad && !dead) reload(v[i], StepIntC<sidx>{}, k0);
                if (c == 0) { RNNG_STAMP(2); }
                if (c == 1) { RNNG_STAMP(6); RNNG_STAMP(7); }
                if (c + D - 1 == MM::CLATE) hold_off();
                if (c + D - 1 < NCH) load_chunk(v[j], rs[sa], aoff[sa], MM::K(sa), MM::K(sa) % CW != 0, rot(StepIntC<sa>{}, MM::ck0(ca)), true);
                bad = c + 1 < NCH ? incomplete(v[i1]) : false;
                multiply(StepIntC<sidx>{}, v[i], opb);
            });
        } else {
        hold_off();
        step_static_for<0, D - 1>([&](auto ii) {
            constexpr int i = decltype(ii)::value;
            load_chunk(v[i], rs[0], aoff[0], MM::K(0), MM::K(0) % CW != 0, i * CW, i * CW < (MM::K(0) + CW - 1) / CW * CW);
        });
#pragma unroll
        for (int mt = 0; mt < MM::MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < MM::NTU; ++nt) acc[mt][nt] = mfloatx4{0.0f, 0.0f, 0.0f, 0.0f};
        bool bad = incomplete(v[0]);      // of the chunk that comes next

        step_static_for<0, MM::NSRC>([&](auto ss) {
            constexpr int sidx = decltype(ss)::value;
            constexpr int NGR = MM::ngr(sidx);
            constexpr int KP = (MM::K(sidx) + CW - 1) / CW * CW;              // weight rows are zero-padded up to here
            constexpr int snext = sidx + 1 < MM::NSRC ? sidx + 1 : sidx;
            constexpr int KPN = (MM::K(snext) + CW - 1) / CW * CW;
#pragma unroll 1
            for (int g = 0; g < NGR; ++g) {
                step_static_for<0, D>([&](auto ii) {
                    constexpr int i = decltype(ii)::value;
                    constexpr int j = (i + D - 1) % D;                   // register set of the chunk D - 1 positions ahead
                    constexpr int i1 = (i + 1) % D;                      // register set of the next chunk
                    const int k0 = (g * D + i) * CW;
                    // the chunk D - 1 positions ahead: in this source, or in the next one's first group
                    const int gj = i == 0 ? g : g + 1;
                    const bool same = gj < NGR;
                    const int kj = same ? (gj * D + j) * CW : j * CW;
                    const bool on = same ? kj < KP : (sidx + 1 < MM::NSRC && kj < KPN);
                    const __amdgpu_buffer_rsrc_t rn = same ? rs[sidx] : rs[snext];
                    auto ahead = [&]() {
                        if (same) load_chunk(v[j], rn, aoff[sidx], MM::K(sidx), MM::K(sidx) % CW != 0, kj, on);
                        else load_chunk(v[j], rn, aoff[snext], MM::K(snext), MM::K(snext) % CW != 0, kj, on);
                    };
                    if (k0 < KP) {
                        // the weights of this chunk (tiles the source does not feed read the zero row)
                        mfloatx4 opb[MM::NTU];
#pragma unroll
                        for (int nt = 0; nt < MM::NTU; ++nt)
                            if (MM::used(sidx, nt)) opb[nt] = *reinterpret_cast<const mfloatx4*>(&lds[brow[sidx][nt] + k0 + wave * 16]);
                        if (bad && !dead) reload(v[i], ss, k0);
                        if (sidx == 0 && i == 0 && g == 0) { RNNG_STAMP(2); }
                        if (sidx == 0 && i == 1 && g == 0) { RNNG_STAMP(6); RNNG_STAMP(7); }
                        ahead();
                        bad = incomplete(v[i1]);
                        multiply(ss, v[i], opb);
                    } else {
                        ahead();
                        bad = incomplete(v[i1]);
                    }
                });
            }
        });
        }
        // ---- hand the accumulators to the element-wise threads: one partial tile per wavefront ----
        // (the previous step's readers of the tiles are behind the barrier that ends a step)
        {
            const int tb = accbase + wave * (NPAD * ACCS);
#pragma unroll
            for (int mt = 0; mt < MM::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MM::NTU; ++nt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        lds[tb + (mt * 16 + 4 * (lane >> 4) + i) * ACCS + nt * 16 + (lane & 15)] = acc[mt][nt][i];
        }
        RNNG_STAMP(3);
        // did any wavefront have to load a chunk again?  (word `step & 1`; the other one is cleared for the next step)
        if (POLL_INC > 0 && retried && lane == 0) atomicOr(&ms.retried[step & 1], 1u);
        step_lds_barrier();
        if (POLL_INC > 0) {
            if (ms.retried[step & 1]) pdelay = pdelay + POLL_INC < 96 ? pdelay + POLL_INC : 96;
            else if ((step & 63) == 63 && pdelay > 0) --pdelay;
            if (tid == 0) ms.retried[(step + 1) & 1] = 0u;
        }
        RNNG_STAMP(4);
        // ---- element-wise program: one thread per (stream, unit) ----
        if (wave_items) {
#pragma unroll
            for (int v = 0; v < PH::NI; ++v) s[PH::NG + v] = r.inv[v];
            step_static_for<0, PH::NG>([&](auto gg) {
                constexpr int g = decltype(gg)::value;
                if (PH::gkind(g) == GA_KIND_CARRY) s[g] = r.carry[PH::cidx(g)];
                else if (PH::gkind(g) == GA_KIND_STATIC) s[g] = sn[g];
                if (PH::gkind(g) == GA_KIND_ACC) {
                    const int tb = accbase + item_n_safe * ACCS + PH::gaux(g) * CMAX + item_il;
                    float x = (lds[tb] + lds[tb + NPAD * ACCS]) + (lds[tb + 2 * NPAD * ACCS] + lds[tb + 3 * NPAD * ACCS]);
                    if constexpr (NW == 8)
                        x += (lds[tb + 4 * NPAD * ACCS] + lds[tb + 5 * NPAD * ACCS]) + (lds[tb + 6 * NPAD * ACCS] + lds[tb + 7 * NPAD * ACCS]);
                    s[g] = r.gptr[g] != nullptr ? x : 0.0f;
                }
            });
            // sums that a helper member of the launch computes ahead of this member: loaded at the
            // step's start, here they have normally arrived (the wavefront repeats while one is missing)
            step_static_for<0, PH::NG>([&](auto gg) {
                constexpr int g = decltype(gg)::value;
                if constexpr (PH::gkind(g) == GA_KIND_POLLED) {
                    int spins = 0;
                    while (__builtin_amdgcn_ballot_w64(__float_as_uint(s[g]) == STEP_SENTINEL) != 0 && !dead) {
                        if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
                        s[g] = gather_at(gg, t + r.goff[g]);
                    }
                }
            });
            PH::ops(s);
#pragma unroll
            for (int q = 0; q < PH::NST; ++q) {
                const bool twin = MM::XB && PH::stshared(q) && PH::sttwin(q);
                wave_store<PH, MStore>(r, q, s[PH::stslot(q)], PH::stshared(q) && !twin ? 2 : 0, a);
                if (twin) {
                    const __amdgpu_buffer_rsrc_t rx = MStore::SW ? __builtin_amdgcn_make_buffer_rsrc(a.store_base, 0, (int)a.store_bytes, STEP_RSRC_FLAGS)
                                                                 : __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(xbase[q]), 0, a.T * r.sstride[q] * 4, STEP_RSRC_FLAGS);
                    __builtin_amdgcn_raw_buffer_store_b32(step_shared_bits(s[PH::stslot(q)]), rx, (int)xvrun[q], 0, STEP_COHERENT_AUX);
                }
            }
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_CARRY) r.carry[PH::cidx(g)] = s[PH::gaux(g)];
            // the next step's STATIC inputs, behind this step's stores: they arrive during that
            // step's contraction (behind the last step: outside the window, nothing is loaded)
            const int t2 = a.backward ? t - 1 : t + 1;
            const bool more = step + 1 < nsteps;
            step_static_for<0, PH::NG>([&](auto gg) {
                constexpr int g = decltype(gg)::value;
                if (PH::gkind(g) == GA_KIND_STATIC) sn[g] = gather_at(gg, more ? t2 + r.goff[g] : -1);
            });
        }
        wave_store_advance<PH>(r);
        if constexpr (MM::XB) {
#pragma unroll
            for (int q = 0; q < PH::NST; ++q) xvrun[q] += (unsigned)(r.sdelta[q] * 4);
        }
        RNNG_STAMP(5);
        step_lds_barrier();   // the tiles are written again in the next step
    }
}

// =============================================================================================
// Matrix-core variant with a two-dimensional split (many streams, wide layers).
//
// In the variant above every workgroup polls every source tensor whole (N * K values per source
// and step), and with wide layers that polling is all a step waits for.  Here the G workgroups
// form G / GJ row groups of GJ workgroups.  Workgroup (gi, gj) still owns the units of chunk
// w = gi * GJ + gj for the element-wise program, but of the contraction it does column slice gj
// (K / GJ columns of every source) for the rows of ALL GJ members of its row group: it polls
// only its slice, multiplies (each wavefront four members' row tiles, operands straight from the
// polling loads as above) and stores the partial sums, written through, into
// partial[frame][member][gj][row][stream].  Then it polls the GJ partial sums of its own rows,
// adds them and runs the element-wise program.  Per step a workgroup polls N * K / GJ values per
// source (four times, once per wavefront) plus GJ * rows * N partial sums, instead of N * K.
//
// M2 is a generated descriptor:
//   static constexpr int NJ (streams), MT (16-stream tiles), NSRC, GJ, RT (rows of a member:
//   tasks * cmax <= 16), CMAX, ACCS, PT (64-column chunks of all sources' slices), DS (register
//   sets); constexpr K(s), KS(s) (columns of a slice, a multiple of 64), psrc(p) / pchunk(p)
//   (source and chunk of position p), blk(s, task).
// =============================================================================================
struct M2Layout {
    int ok, n_src, cmax, zrow, accbase, accstride, total_floats;
    int wbase[STEP_MAX_SOURCES], wstride[STEP_MAX_SOURCES], rows[STEP_MAX_SOURCES];
    short blk[STEP_MAX_SOURCES][STEP_MAX_TASKS];
};

RNNG_HD inline void compute_mstep2_layout(const StepLayout& lay, int N, int GJ, int lds_limit_floats, M2Layout& m) {
    m.ok = 0;
    if (!lay.ok || lay.n_phases != 1 || lay.n_sources < 1) return;
    const StepPhase& ph = lay.ph[0];
    if (ph.item_chunk * N > STEP_THREADS || ph.n_tasks * ph.cmax > 16) return;
    m.n_src = lay.n_sources; m.cmax = ph.cmax;
    const int npad = (N + 15) / 16 * 16;
    int cur = 0, wsmax = 0;
    for (int s = 0; s < lay.n_sources; ++s) {
        if (lay.src[s].k_len % (64 * GJ)) return;       // slices of whole 64-column chunks
        int nb = 0;
        for (int t = 0; t < STEP_MAX_TASKS; ++t) {
            m.blk[s][t] = -1;
            if (t >= ph.n_tasks) continue;
            for (int e = 0; e < ph.task[t].n_edges; ++e)
                if (ph.task[t].e[e].src == s && m.blk[s][t] < 0) m.blk[s][t] = (short)nb++;
        }
        m.rows[s] = nb * ph.cmax;
        m.wstride[s] = lay.src[s].k_len / GJ + 4;
        wsmax = m.wstride[s] > wsmax ? m.wstride[s] : wsmax;
        m.wbase[s] = cur; cur += GJ * m.rows[s] * m.wstride[s];
    }
    m.zrow = cur; cur += wsmax;
    m.accstride = 16 + 4;
    m.accbase = cur; cur += npad * m.accstride;
    if (cur > lds_limit_floats) return;
    m.total_floats = cur;
    m.ok = 1;
}

struct M2Shared { StepShared sh; M2Layout ml; };

// w: index of this workgroup among the a.G workgroups of the component.
template <class PH, class M2>
__device__ __forceinline__ void mstep2_kernel_body(const StepArgs& a, M2Shared& ms, float* lds, int w) {
    if (w < 0 || w >= a.G) return;
    constexpr int GJ = M2::GJ, RT = M2::RT, CMAX = M2::CMAX, NPAD = M2::MT * 16, ACCS = M2::ACCS, NQ = NPAD / 4;
    // A wavefront multiplies the rows of four members.  A member with few rows does not fill a
    // 16-row tile: PACK members share one (RP rows each), so the wavefront has TPW tiles.
    constexpr int RP = RT <= 4 ? 4 : RT <= 8 ? 8 : 16, PACK = 16 / RP, TT = GJ / PACK;      // TT row tiles in all
    // Work of a step = (stream tile, row tile) pairs.  With 1, 2 or 4 stream tiles a wavefront takes
    // ONE stream tile (so that no polled value is loaded by two wavefronts) and TT * MT / 4 row
    // tiles; with 3 it takes all stream tiles and a quarter of the row tiles.
    constexpr bool BY_STREAMS = M2::MT == 1 || M2::MT == 2 || M2::MT == 4;
    constexpr int MTW = BY_STREAMS ? 1 : M2::MT, WPS = BY_STREAMS ? 4 / M2::MT : 4, TPW = TT / WPS;
    static_assert(TT % WPS == 0, "row tiles must divide among the wavefronts");
    const int gi = w / GJ, gj = w - gi * GJ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mt0 = BY_STREAMS ? wave / WPS : 0, tl0 = (wave % WPS) * TPW;      // this wavefront's stream tile and first row tile
    const int T = a.T, N = a.N;
    StepShared& sh = ms.sh;
    if (tid == 0) { compute_step_layout(a.words, a.desc_off, a.G, 1, M2::NJ, sh.lay); compute_mstep2_layout(sh.lay, M2::NJ, GJ, (int)(STEP_LDS_LIMIT / 4), ms.ml); }
    __syncthreads();
    const StepPhase& ph = sh.lay.ph[0];
    const M2Layout& ml = ms.ml;
    {
        const int ic = ph.item_chunk;
        const int il = tid % ic, n = tid / ic;
        sh.iteminfo[0][tid] = (unsigned)il | ((unsigned)(n < N ? n : 0xFFFF) << 16);
    }
    for (int i = tid; i < ml.total_floats; i += STEP_THREADS) lds[i] = 0.0f;
    __syncthreads();
    // resident weights: column slice gj of the rows of every member m of this row group
    for (int s = 0; s < ml.n_src; ++s) {
        const int K = sh.lay.src[s].k_len, KS = K / GJ;
        for (int t = 0; t < ph.n_tasks; ++t) {
            const StepTask& task = ph.task[t];
            for (int e = 0; e < task.n_edges; ++e) {
                const StepEdge ed = task.e[e];
                if (ed.src != s) continue;
                const float* W = a.weights + ed.w_off;
                for (int i = tid; i < GJ * CMAX * KS; i += STEP_THREADS) {
                    const int m = i / (CMAX * KS), rem = i - m * (CMAX * KS);
                    const int ul = rem / KS, kk = rem - ul * KS;
                    const int u = (gi * GJ + m) * task.chunk + ul, k = gj * KS + kk;
                    float v = 0.0f;
                    if (ul < task.chunk && u < task.n_out) v = ed.transposed ? W[(size_t)k * task.n_out + u] : W[(size_t)u * K + k];
                    lds[ml.wbase[s] + (m * ml.rows[s] + ml.blk[s][t] * CMAX + ul) * ml.wstride[s] + kk] += v;
                }
                __syncthreads();
            }
        }
    }
    PhaseRegs<PH> r;
    phase_setup<PH, 1, 2>(r, a, sh, lds, w, tid);
    __syncthreads();

    const int accbase = suni(ml.accbase);
    const int item_il = (int)(sh.iteminfo[0][tid] & 0xFFFF);
    const int item_n = tid / suni(ph.item_chunk);
    // weight row behind this lane's tile column (member, row) in each of the wavefront's tiles
    int brow[M2::NSRC][TPW];
#pragma unroll
    for (int sidx = 0; sidx < M2::NSRC; ++sidx)
#pragma unroll
        for (int tl = 0; tl < TPW; ++tl) {
            const int col = lane & 15, m = (tl0 + tl) * PACK + col / RP, row = col % RP;
            const int task = row / CMAX, ul = row - task * CMAX;
            int b = -1;
#pragma unroll
            for (int t2 = 0; t2 < STEP_MAX_TASKS; ++t2) if (task == t2) b = M2::blk(sidx, t2);
            brow[sidx][tl] = (b >= 0 && row < RT && m < GJ ? suni(ml.wbase[sidx]) + (m * suni(ml.rows[sidx]) + b * CMAX + ul) * suni(ml.wstride[sidx]) : suni(ml.zrow)) + 4 * (lane >> 4);
        }
    // A operands: stream 16 mt + (lane & 15), columns gj * KS + 64 c + 16 kb + 4 (lane >> 4) ...
    int aoff[M2::NSRC][MTW];
#pragma unroll
    for (int sidx = 0; sidx < M2::NSRC; ++sidx)
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            const int n = (mt0 + mt) * 16 + (lane & 15);
            aoff[sidx][mt] = n < N ? (n * M2::K(sidx) + gj * M2::KS(sidx) + 4 * (lane >> 4)) * 4 : 0x7FFFFFF0;
        }
    // partial sums: [frame][workgroup][slice][row][stream]
    const long long pframe = (long long)a.G * GJ * RT * NPAD;      // floats per frame
    int poff_store[MTW][TPW];      // where this lane's four streams of (stream tile, row tile) go, bytes inside a frame
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int tl = 0; tl < TPW; ++tl) {
            const int col = lane & 15, m = (tl0 + tl) * PACK + col / RP, row = col % RP;
            poff_store[mt][tl] = (row < RT && m < GJ) ? ((((gi * GJ + m) * GJ + gj) * RT + row) * NPAD + (mt0 + mt) * 16 + 4 * (lane >> 4)) * 4 : 0x7FFFFFF0;
        }
    const int prow = tid / NQ, pnq = tid - prow * NQ;      // phase 2: this thread adds row prow, streams 4 pnq ...
    const int poff_load = prow < RT ? ((w * GJ * RT + prow) * NPAD + 4 * pnq) * 4 : 0x7FFFFFF0;      // slice j adds j * RT * NPAD * 4

    bool dead = false;
    int pdelay = 0;
    float sn[PH::NG > 0 ? PH::NG : 1];
    const int nsteps = step_count(a);
    for (int step = 0; step < nsteps; ++step) {
        const int t = step_frame(a, step);
        float s[MAX_SLOTS];
        RNNG_STAMP(0);
#pragma unroll
        for (int g = 0; g < PH::NG; ++g) {
            if (PH::gkind(g) == GA_KIND_CARRY) {
                if (step > 0) {
                    s[g] = r.carry[PH::cidx(g)];
                } else {
                    const int frame = t + r.goff[g];
                    s[g] = (r.gptr[g] != nullptr && frame >= 0 && frame < a.T) ? r.gptr[g][(long long)frame * r.gstride[g]] : 0.0f;
                }
            } else if (PH::gkind(g) == GA_KIND_STATIC && step > 0) {
                s[g] = sn[g];
            } else if (PH::gkind(g) != GA_KIND_ACC) {
                const int frame = t + r.goff[g];
                float v = 0.0f;
                if (r.gptr[g] != nullptr && frame >= 0 && frame < T) {
                    if (PH::gkind(g) == GA_KIND_STATIC) v = r.gptr[g][(long long)frame * r.gstride[g]];
                    else v = load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]);
                }
                s[g] = v;
            }
        }
#pragma unroll
        for (int v = 0; v < PH::NI; ++v) s[PH::NG + v] = r.inv[v];
        RNNG_STAMP(1);

        __amdgpu_buffer_rsrc_t rs[M2::NSRC];
#pragma unroll
        for (int sidx = 0; sidx < M2::NSRC; ++sidx) {
            const StepSource& sc = sh.lay.src[sidx];
            const int frame = t + suni(sc.frame_off);
            const bool in_window = frame >= 0 && frame < T;
            const float* g = ((cbufs_t)a.buf_ptr)[suni(sc.buf)] + (size_t)(in_window ? frame : 0) * a.N * M2::K(sidx);
            rs[sidx] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(g), 0, in_window ? N * M2::K(sidx) * 4 : 0, STEP_RSRC_FLAGS);
        }
        const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(a.partial + (long long)t * pframe, 0, (int)(pframe * 4), STEP_RSRC_FLAGS);

        // ---- phase 1: this slice's share of the row group's contraction ----
        // The 64-column chunks of all sources form one sequence of PT positions (generated:
        // M2::psrc(p), M2::pchunk(p)).  Position p lives in register set p % DS; DS - 1 positions
        // are in flight: the loads of position p + DS - 1 are issued when position p is checked
        // (into the set of position p - 1, whose multiplications have been issued).
        constexpr int PT = M2::PT, DS = M2::DS;
        muintx4 v[DS][4][MTW];
        auto load_chunk = [&](muintx4 (&dst)[4][MTW], auto ss, int c) {
            constexpr int S = decltype(ss)::value;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
                    dst[kb][mt] = __builtin_amdgcn_raw_buffer_load_b128(rs[S], aoff[S][mt] + (c * 64 + kb * 16) * 4, 0, STEP_COHERENT_AUX);
        };
        auto incomplete = [&](const muintx4 (&x)[4][MTW]) {
            unsigned m = 0;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt) {
                    const unsigned m1 = x[kb][mt].x > x[kb][mt].y ? x[kb][mt].x : x[kb][mt].y, m2 = x[kb][mt].z > x[kb][mt].w ? x[kb][mt].z : x[kb][mt].w;
                    const unsigned m3 = m1 > m2 ? m1 : m2;
                    m = m > m3 ? m : m3;
                }
            return __builtin_amdgcn_ballot_w64(m == STEP_SENTINEL) != 0;
        };
        for (int i = 0; i < pdelay; ++i) __builtin_amdgcn_s_sleep(1);
        bool retried = false;
        step_static_for<0, DS - 1>([&](auto pp) {
            constexpr int q = decltype(pp)::value;
            if constexpr (q < PT) load_chunk(v[q], StepIntC<M2::psrc(q)>{}, M2::pchunk(q));
        });
        mfloatx4 acc[MTW][TPW];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
            for (int tau = 0; tau < TPW; ++tau) acc[mt][tau] = mfloatx4{0.0f, 0.0f, 0.0f, 0.0f};
        step_static_for<0, PT>([&](auto pp) {
            constexpr int pos = decltype(pp)::value, set = pos % DS, sidx = M2::psrc(pos), c = M2::pchunk(pos);
            constexpr int q = pos + DS - 1;
            if constexpr (q < PT) load_chunk(v[q % DS], StepIntC<M2::psrc(q < PT ? q : 0)>{}, M2::pchunk(q < PT ? q : 0));
            if (incomplete(v[set]) && !dead) {
                retried = true;
                muintx4 again[4][MTW];
                int spins = 0;
                for (;;) {
                    if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
                    __builtin_amdgcn_s_sleep(MSTEP_RETRY_SLEEP);
                    step_compiler_barrier();
                    load_chunk(again, StepIntC<sidx>{}, c);
                    if (!incomplete(again)) break;
                }
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int mt = 0; mt < MTW; ++mt) v[set][kb][mt] = again[kb][mt];
            }
            if (pos == 0) { RNNG_STAMP(2); }
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int tau = 0; tau < TPW; ++tau) {
                    const mfloatx4 b = *reinterpret_cast<const mfloatx4*>(&lds[brow[sidx][tau] + c * 64 + kb * 16]);
#pragma unroll
                    for (int mt = 0; mt < MTW; ++mt) {
                        acc[mt][tau] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[set][kb][mt].x), b[0], acc[mt][tau], 0, 0, 0);
                        acc[mt][tau] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[set][kb][mt].y), b[1], acc[mt][tau], 0, 0, 0);
                        acc[mt][tau] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[set][kb][mt].z), b[2], acc[mt][tau], 0, 0, 0);
                        acc[mt][tau] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[set][kb][mt].w), b[3], acc[mt][tau], 0, 0, 0);
                    }
                }
        });
        // the partial sums of (member, row, four streams) to their owners, written through
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
            for (int tau = 0; tau < TPW; ++tau) {
                const muintx4 o = {step_shared_bits(acc[mt][tau][0]), step_shared_bits(acc[mt][tau][1]), step_shared_bits(acc[mt][tau][2]), step_shared_bits(acc[mt][tau][3])};
                __builtin_amdgcn_raw_buffer_store_b128(o, rp, poff_store[mt][tau], 0, STEP_COHERENT_AUX);
            }
        // STATIC inputs of the next step
        if (step + 1 < nsteps) {
            const int t2 = a.backward ? t - 1 : t + 1;
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_STATIC) {
                    const int frame = t2 + r.goff[g];
                    float x = 0.0f;
                    if (r.gptr[g] != nullptr && frame >= 0 && frame < T) x = r.gptr[g][(long long)frame * r.gstride[g]];
                    sn[g] = x;
                }
        }
        RNNG_STAMP(3);
        // ---- phase 2: add the GJ partial sums of this workgroup's own rows ----
        {
            muintx4 q[GJ];
            int spins = 0;
            for (;;) {
                step_compiler_barrier();
#pragma unroll
                for (int j = 0; j < GJ; ++j) q[j] = __builtin_amdgcn_raw_buffer_load_b128(rp, poff_load + j * RT * NPAD * 4, 0, STEP_COHERENT_AUX);
                unsigned m = 0;
#pragma unroll
                for (int j = 0; j < GJ; ++j) {
                    const unsigned m1 = q[j].x > q[j].y ? q[j].x : q[j].y, m2 = q[j].z > q[j].w ? q[j].z : q[j].w;
                    const unsigned m3 = m1 > m2 ? m1 : m2;
                    m = m > m3 ? m : m3;
                }
                if (__builtin_amdgcn_ballot_w64(m == STEP_SENTINEL) == 0 || dead) break;
                if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
                __builtin_amdgcn_s_sleep(MSTEP_RETRY_SLEEP);
            }
            float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int j = 0; j < GJ; ++j) {
                sum[0] += __uint_as_float(q[j].x); sum[1] += __uint_as_float(q[j].y);
                sum[2] += __uint_as_float(q[j].z); sum[3] += __uint_as_float(q[j].w);
            }
            if (prow < RT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) lds[accbase + (4 * pnq + e) * ACCS + prow] = sum[e];
            }
        }
        if (__syncthreads_or(retried ? 1 : 0)) pdelay = pdelay + MSTEP_POLL_INC < 96 ? pdelay + MSTEP_POLL_INC : 96;
        else if ((step & 63) == 63 && pdelay > 0) --pdelay;
        RNNG_STAMP(4);
        // ---- element-wise program: one thread per (stream, unit) ----
        if (r.n >= 0) {
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_ACC) {
                    float x = 0.0f;
                    if (r.gptr[g] != nullptr) x = lds[accbase + item_n * ACCS + PH::gaux(g) * CMAX + item_il];
                    s[g] = x;
                }
            PH::ops(s);
#pragma unroll
            for (int q = 0; q < PH::NST; ++q) {
                if (r.sptr[q] == nullptr) continue;
                if (PH::stshared(q)) store_shared(r.sptr[q] + (long long)t * r.sstride[q], s[PH::stslot(q)]);
                else store_plain(r.sptr[q] + (long long)t * r.sstride[q], s[PH::stslot(q)]);
            }
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_CARRY) r.carry[PH::cidx(g)] = s[PH::gaux(g)];
        }
        RNNG_STAMP(5);
        step_lds_barrier();   // the tile is written again in the next step
    }
}

// =============================================================================================
// Streaming variant (run-time specialised, single-phase components, few streams, wide layers).
//
// From about 2,000 units on, the full weight matrices inside a recurrent node no longer fit the
// registers and LDS of the chip (an LSTM layer of 4,096 cells has 256 MiB of them), so a time step
// really is what the roofline model of the sequential part says: every weight is read from memory
// once per step.  Each workgroup owns a chunk of every layer's units, as in the other variants, and
// each of its four wavefronts owns UW of them.  A wavefront's work per step is a set of row
// segments, one per (unit, task, edge): the weight row W_e[u][0 .. K_e) against source vector
// x_src(e).  All segments advance together through the columns in chunks of 256 (lane l takes the
// four columns 256 j + 4 l ...: a wavefront's load covers 1 KiB of consecutive addresses), PD chunks
// ahead, so that NSEG * PD 128-bit loads per lane are in flight (tens of KiB per compute unit, which
// is what it takes to keep the memory system busy); the loads of a step's first PD chunks are issued
// before the step's exchange, because the weights do not depend on it.  The source vectors are
// polled into LDS by the whole workgroup (sentinel protocol, all loads of an attempt in flight
// together) and read from there once per (source, stream, chunk) for all segments.  Transposed
// connections (the backward direction) read a transposed copy of the matrix, made once per window,
// so that both directions stream rows.
//
// SS is a generated descriptor:
//   static constexpr int NB (streams, padded), CMAX (units per workgroup), UW (units per
//   wavefront), NT (tasks), NSRC, NSEG, PD, JMAX (256-column chunks of the longest row), NACC
//   (= UW * NT), XF (floats of the LDS source area), ACCS (row stride of the accumulator area),
//   PQ (128-bit polling loads per thread over all sources);
//   constexpr seg_ul(i), seg_task(i), seg_edge(i), seg_src(i), seg_tr(i) (reads the transposed copy), K(s), KP(s) (padded to 256),
//   xoff(s), pq0(s) / pqn(s) (first polling register and count of source s).
// =============================================================================================
struct SShared { StepShared sh; };

template <class PH, class SS>
__device__ __forceinline__ void sstep_kernel_body(const StepArgs& a, SShared& ms, float* lds, int w) {
    if (w < 0 || w >= a.G) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = a.T, N = a.N;
    StepShared& sh = ms.sh;
    if (tid == 0) compute_step_layout(a.words, a.desc_off, a.G, 1, N, sh.lay);
    __syncthreads();
    const StepPhase& ph = sh.lay.ph[0];
    {
        const int ic = ph.item_chunk;
        const int il = tid % ic, n = tid / ic;
        sh.iteminfo[0][tid] = (unsigned)il | ((unsigned)(n < N ? n : 0xFFFF) << 16);
    }
    constexpr int NB = SS::NB, UW = SS::UW, NT = SS::NT, NSEG = SS::NSEG, PD = SS::PD, JMAX = SS::JMAX, NACC = SS::NACC;
    constexpr int ACCBASE = SS::XF, ACCS = SS::ACCS;
    for (int i = tid; i < SS::XF + NB * ACCS; i += STEP_THREADS) lds[i] = 0.0f;
    __syncthreads();
    PhaseRegs<PH> r;
    phase_setup<PH, 1, 2>(r, a, sh, lds, w, tid);
    const int item_il = (int)(sh.iteminfo[0][tid] & 0xFFFF);
    const int item_n = tid / suni(ph.item_chunk);

    // this lane's byte offset in each segment's matrix at column chunk 0 (a segment without a unit
    // behind it stays outside the descriptor: its loads return zeros)
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.weights), 0, (int)a.weight_bytes, STEP_RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rwt = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.weights_t), 0, (int)a.weight_bytes, STEP_RSRC_FLAGS);
    constexpr int JR = (JMAX + PD - 1) / PD * PD;      // chunk positions of a step (whole rounds of the PD register sets)
    unsigned voff[NSEG];
#pragma unroll
    for (int i = 0; i < NSEG; ++i) {
        const StepTask& tk = ph.task[SS::seg_task(i)];
        const StepEdge ed = tk.e[SS::seg_edge(i)];
        const int chunk = suni(tk.chunk), n_out = suni(tk.n_out);
        const int ulw = wave * UW + SS::seg_ul(i), u = w * chunk + ulw;
        const bool ok = ulw < chunk && u < n_out;
        voff[i] = ok ? (unsigned)(((long long)suni(ed.w_off) + (long long)u * suni(ed.k_len) + 4 * lane) * 4) : 0xC0000000u;
    }
    // weights of chunk j of every segment; columns beyond a row's end read as zero
    auto load_chunk = [&](mfloatx4 (&dst)[NSEG], int j) {
#pragma unroll
        for (int i = 0; i < NSEG; ++i) {
            const int K = SS::K(SS::seg_src(i));
            unsigned off = voff[i] + (unsigned)(j * 1024);
            if (K % 256 != 0) off = (256 * j + 4 * lane < K) ? off : 0xC0000000u;
            else if (JR * 256 != K) off = (256 * j < K) ? off : 0xC0000000u;
            const muintx4 v = SS::seg_tr(i) ? __builtin_amdgcn_raw_buffer_load_b128(rwt, (int)off, 0, 0)
                                            : __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0);
            dst[i] = mfloatx4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        }
    };

    bool dead = false;
    float sn[PH::NG > 0 ? PH::NG : 1];
    const int nsteps = step_count(a);
    mfloatx4 wq[PD][NSEG];
    if (nsteps > 0) step_static_for<0, PD>([&](auto pp) { constexpr int p = decltype(pp)::value; if (p < JMAX) load_chunk(wq[p], p); });
    for (int step = 0; step < nsteps; ++step) {
        const int t = step_frame(a, step);
        float s[MAX_SLOTS];
        RNNG_STAMP(0);
#pragma unroll
        for (int g = 0; g < PH::NG; ++g) {
            if (PH::gkind(g) == GA_KIND_CARRY) {
                if (step > 0) {
                    s[g] = r.carry[PH::cidx(g)];
                } else {
                    const int frame = t + r.goff[g];
                    s[g] = (r.gptr[g] != nullptr && frame >= 0 && frame < T) ? r.gptr[g][(long long)frame * r.gstride[g]] : 0.0f;
                }
            } else if (PH::gkind(g) == GA_KIND_STATIC && step > 0) {
                s[g] = sn[g];
            } else if (PH::gkind(g) != GA_KIND_ACC) {
                const int frame = t + r.goff[g];
                float v = 0.0f;
                if (r.gptr[g] != nullptr && frame >= 0 && frame < T) {
                    if (PH::gkind(g) == GA_KIND_STATIC) v = r.gptr[g][(long long)frame * r.gstride[g]];
                    else v = load_coherent(r.gptr[g] + (long long)frame * r.gstride[g]);
                }
                s[g] = v;
            }
        }
#pragma unroll
        for (int v = 0; v < PH::NI; ++v) s[PH::NG + v] = r.inv[v];
        RNNG_STAMP(1);

        // ---- the exchange: the source vectors of this step into LDS ----
        {
            __amdgpu_buffer_rsrc_t rs[SS::NSRC];
#pragma unroll
            for (int sidx = 0; sidx < SS::NSRC; ++sidx) {
                const StepSource& sc = sh.lay.src[sidx];
                const int frame = t + suni(sc.frame_off);
                const bool in_window = frame >= 0 && frame < T;
                const float* g = ((cbufs_t)a.buf_ptr)[suni(sc.buf)] + (size_t)(in_window ? frame : 0) * N * SS::K(sidx);
                rs[sidx] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(g), 0, in_window ? N * SS::K(sidx) * 4 : 0, STEP_RSRC_FLAGS);
            }
            muintx4 pv[SS::PQ > 0 ? SS::PQ : 1];
            int spins = 0;
            for (;;) {
                step_compiler_barrier();
                unsigned m = 0;
#pragma unroll
                for (int sidx = 0; sidx < SS::NSRC; ++sidx)
#pragma unroll
                    for (int q = 0; q < SS::pqn(sidx); ++q)
                        pv[SS::pq0(sidx) + q] = __builtin_amdgcn_raw_buffer_load_b128(rs[sidx], (tid + STEP_THREADS * q) * 16, 0, STEP_COHERENT_AUX);
#pragma unroll
                for (int q = 0; q < SS::PQ; ++q) {
                    const unsigned m1 = pv[q].x > pv[q].y ? pv[q].x : pv[q].y, m2 = pv[q].z > pv[q].w ? pv[q].z : pv[q].w;
                    const unsigned m3 = m1 > m2 ? m1 : m2;
                    m = m > m3 ? m : m3;
                }
                if (__builtin_amdgcn_ballot_w64(m == STEP_SENTINEL) == 0 || dead) break;
                if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
            }
            // [stream][column] per source, rows padded to whole chunks (the padding stays zero)
#pragma unroll
            for (int sidx = 0; sidx < SS::NSRC; ++sidx)
#pragma unroll
                for (int q = 0; q < SS::pqn(sidx); ++q) {
                    const int e4 = (tid + STEP_THREADS * q) * 4;      // element index in the frame [N][K]
                    if (e4 < N * SS::K(sidx)) {
                        const int n = e4 / SS::K(sidx), k = e4 - n * SS::K(sidx);
                        const muintx4 v = pv[SS::pq0(sidx) + q];
                        *reinterpret_cast<mfloatx4*>(&lds[SS::xoff(sidx) + n * SS::KP(sidx) + k]) =
                            mfloatx4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
                    }
                }
        }
        step_lds_barrier();
        RNNG_STAMP(2);

        // ---- the contraction: all segments advance together, PD chunks of loads ahead ----
        float part[NACC][NB];
#pragma unroll
        for (int i = 0; i < NACC; ++i)
#pragma unroll
            for (int n = 0; n < NB; ++n) part[i][n] = 0.0f;
        auto consume = [&](const mfloatx4 (&wv)[NSEG], int j) {
#pragma unroll
            for (int sidx = 0; sidx < SS::NSRC; ++sidx) {
                if (SS::KP(sidx) != JR * 256 && 256 * j >= SS::KP(sidx)) continue;
#pragma unroll
                for (int n = 0; n < NB; ++n) {
                    const mfloatx4 x = *reinterpret_cast<const mfloatx4*>(&lds[SS::xoff(sidx) + n * SS::KP(sidx) + 256 * j + 4 * lane]);
#pragma unroll
                    for (int i = 0; i < NSEG; ++i)
                        if (SS::seg_src(i) == sidx) {
                            float& p = part[SS::seg_ul(i) * NT + SS::seg_task(i)][n];
                            p = fmaf(wv[i].x, x.x, p); p = fmaf(wv[i].y, x.y, p); p = fmaf(wv[i].z, x.z, p); p = fmaf(wv[i].w, x.w, p);
                        }
                }
            }
        };
#pragma unroll 1
        for (int jj = 0; jj < JR; jj += PD) {
            step_static_for<0, PD>([&](auto pp) {
                constexpr int p = decltype(pp)::value;
                consume(wq[p], jj + p);
                // the same register set takes chunk jj + p + PD; past the row's end the next step's first chunks
                const int jn = jj + p + PD;
                load_chunk(wq[p], jn < JR ? jn : jn - JR);
            });
        }
        // (chunks JMAX .. JR - 1, if any, were loaded as zeros; the last PD loads are the next step's first chunks)
        float tot[NACC * NB];
        {
            float flat[NACC * NB];
#pragma unroll
            for (int i = 0; i < NACC; ++i)
#pragma unroll
                for (int n = 0; n < NB; ++n) flat[i * NB + n] = part[i][n];
            wave_reduce_many<NACC * NB>(flat, tot);
        }
        if (lane == 0) {
#pragma unroll
            for (int ul = 0; ul < UW; ++ul)
#pragma unroll
                for (int task = 0; task < NT; ++task)
#pragma unroll
                    for (int n = 0; n < NB; ++n)
                        if (wave * UW + ul < SS::CMAX) lds[ACCBASE + n * ACCS + task * SS::CMAX + wave * UW + ul] = tot[(ul * NT + task) * NB + n];
        }
        // STATIC inputs of the next step
        if (step + 1 < nsteps) {
            const int t2 = a.backward ? t - 1 : t + 1;
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_STATIC) {
                    const int frame = t2 + r.goff[g];
                    float x = 0.0f;
                    if (r.gptr[g] != nullptr && frame >= 0 && frame < T) x = r.gptr[g][(long long)frame * r.gstride[g]];
                    sn[g] = x;
                }
        }
        RNNG_STAMP(3);
        step_lds_barrier();
        RNNG_STAMP(4);
        // ---- element-wise program: one thread per (stream, unit) ----
        if (r.n >= 0) {
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_ACC) s[g] = r.gptr[g] != nullptr ? lds[ACCBASE + item_n * ACCS + PH::gaux(g) * SS::CMAX + item_il] : 0.0f;
            PH::ops(s);
#pragma unroll
            for (int q = 0; q < PH::NST; ++q) {
                if (r.sptr[q] == nullptr) continue;
                if (PH::stshared(q)) store_shared(r.sptr[q] + (long long)t * r.sstride[q], s[PH::stslot(q)]);
                else store_plain(r.sptr[q] + (long long)t * r.sstride[q], s[PH::stslot(q)]);
            }
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_CARRY) r.carry[PH::cidx(g)] = s[PH::gaux(g)];
        }
        RNNG_STAMP(5);
        step_lds_barrier();   // the source and accumulator areas are written again in the next step
    }
}


// =============================================================================================
// Streaming matrix-core variant (run-time specialised, single-phase components, many streams, wide
// layers): the matrix-core variant above with the weights read from memory every step instead of
// kept in LDS.  Lane (c, q) of a wavefront loads, per chunk (16 columns per wavefront) and 16-row tile, the four
// weights W[row c][k0 + 16 wave + 4 q ...] with one 128-bit load (B operands) next to the polling
// load of the four source values of stream c (A operands); D register sets hold the operands of D
// chunks, so that (MT + NTU) * (D - 1) loads per lane are in flight.  The weight loads of a step's
// first chunks are issued before the hold-off of the polling loads: they do not depend on the
// exchange.  With more (stream, unit) items than threads the element-wise program runs in IPT
// passes of SPP streams each (the accumulator tiles hold all streams).
//
// SM is a generated descriptor:
//   static constexpr int NJ (streams), MT, NSRC, NTU, D, CMAX, ACCS, NW (wavefronts: 8, or 4 where the
//   operand registers of 8 do not fit), TR (1: the matrices are read from the transposed copy), IPT,
//   SPP, XB (exchange through the tile-blocked twins); constexpr K(s), ngr(s), edge(s, task) (edge of the task
//   that reads source s, -1: none), used(s, nt).
// =============================================================================================
template <class PH, class SM>
__device__ __forceinline__ void smstep_kernel_body(const StepArgs& a, SShared& ms, float* lds, int w) {
    if (w < 0 || w >= a.G) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = a.T, N = a.N;
    StepShared& sh = ms.sh;
    constexpr int IPT = SM::IPT, SPP = SM::SPP, NW = SM::NW, NTHR = 64 * NW, CW = 16 * NW;      // wavefronts, threads, columns of a chunk
    if (tid == 0) compute_step_layout(a.words, a.desc_off, a.G, 1, SPP < SM::NJ ? SPP : SM::NJ, sh.lay);
    __syncthreads();
    const StepPhase& ph = sh.lay.ph[0];
    if (tid < STEP_THREADS) {      // the element-wise items sit on the first STEP_THREADS threads
        const int ic = ph.item_chunk;
        const int il = tid % ic, n = tid / ic;
        sh.iteminfo[0][tid] = (unsigned)il | ((unsigned)(n < N && n < SPP ? n : 0xFFFF) << 16);
    }
    constexpr int CMAX = SM::CMAX, D = SM::D, NPAD = SM::MT * 16, ACCS = SM::ACCS;
    for (int i = tid; i < NW * NPAD * ACCS; i += NTHR) lds[i] = 0.0f;
    __syncthreads();
    PhaseRegs<PH> r;
    phase_setup<PH, 1, 2>(r, a, sh, lds, w, tid);
    const int item_il = tid < STEP_THREADS ? (int)(sh.iteminfo[0][tid] & 0xFFFF) : 0;
    const int item_n = tid / suni(ph.item_chunk);
    // floats between the same item of consecutive passes, per gather / store (SPP streams further on)
    int gpass[PH::NG > 0 ? PH::NG : 1], spass[PH::NST > 0 ? PH::NST : 1];
#pragma unroll
    for (int g = 0; g < PH::NG; ++g) gpass[g] = SPP * (r.gstride[g] / N);
#pragma unroll
    for (int q = 0; q < PH::NST; ++q) spass[q] = SPP * (r.sstride[q] / N);

    const __amdgpu_buffer_rsrc_t rwb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(SM::TR ? a.weights_t : a.weights), 0, (int)a.weight_bytes, STEP_RSRC_FLAGS);
    const int wcol = wave * 16 + 4 * (lane >> 4);
    // byte offset of this lane's B operand in chunk 0, per source and row tile (no row behind the
    // lane's tile column, or the task does not read the source: outside the descriptor)
    unsigned boff[SM::NSRC][SM::NTU];
#pragma unroll
    for (int sidx = 0; sidx < SM::NSRC; ++sidx)
#pragma unroll
        for (int nt = 0; nt < SM::NTU; ++nt) {
            const int col = nt * 16 + (lane & 15);
            const int task = col / CMAX, ul = col - task * CMAX;
            unsigned off = 0xC0000000u;
#pragma unroll
            for (int t2 = 0; t2 < STEP_MAX_TASKS; ++t2)
                if (task == t2 && SM::edge(sidx, t2) >= 0) {
                    const StepTask& tk = ph.task[t2];
                    const int u = w * tk.chunk + ul;
                    if (ul < tk.chunk && u < tk.n_out)
                        off = (unsigned)(((long long)tk.e[SM::edge(sidx, t2) >= 0 ? SM::edge(sidx, t2) : 0].w_off + (long long)u * SM::K(sidx) + wcol) * 4);
                }
            boff[sidx][nt] = off;
        }
    // (SM::XB: the sources are the tile-blocked twins of the exchanged tensors, as in the variant with
    // on-chip weights: a wavefront's load of a 16 x 16 tile is 1 KiB of consecutive addresses)
    int aoff[SM::NSRC][SM::MT];
#pragma unroll
    for (int sidx = 0; sidx < SM::NSRC; ++sidx)
#pragma unroll
        for (int mt = 0; mt < SM::MT; ++mt) {
            const int n = mt * 16 + (lane & 15);
            if (SM::XB) aoff[sidx][mt] = ((mt * (SM::K(sidx) / 16) + wave) * 256 + lane * 4) * 4;
            else aoff[sidx][mt] = n < N ? (n * SM::K(sidx) + wcol) * 4 : 0x7FFFFFF0;
        }
    // the twin's element of this thread's item (pass 0) per exchanged store, frame 0
    float* xptr[PH::NST > 0 ? PH::NST : 1];
    if constexpr (SM::XB) {
        cwords_t pw = (cwords_t)a.words + suni(ph.prog_off);
        cwords_t st = pw + PG_HEADER_WORDS + PH::NG * GA_WORDS + PH::NI * IV_WORDS + pw[PG_NOPS] * MO_WORDS;
#pragma unroll
        for (int q = 0; q < PH::NST; ++q) {
            xptr[q] = nullptr;
            if (!PH::stshared(q) || r.sptr[q] == nullptr) continue;
            const int dim = suni(st[q * ST_WORDS + ST_DIM]);
            const int i = (int)(r.sptr[q] - r.sbase[q]) - r.n * dim;      // this thread's unit
            xptr[q] = ((cbufs_t)a.buf_ptr)[a.twin_base + suni(st[q * ST_WORDS + ST_BUF])] +
                      ((r.n >> 4) * (dim >> 4) + (i >> 4)) * 256 + ((((i & 15) >> 2) << 4) + (r.n & 15)) * 4 + (i & 3);
        }
    }

    bool dead = false;
    int pdelay = 0;
    float sn[IPT][PH::NG > 0 ? PH::NG : 1];
    float carry[IPT][PH::NC > 0 ? PH::NC : 1];
#pragma unroll
    for (int p = 0; p < IPT; ++p)
#pragma unroll
        for (int c = 0; c < (PH::NC > 0 ? PH::NC : 1); ++c) carry[p][c] = 0.0f;
    const int nsteps = step_count(a);
    for (int step = 0; step < nsteps; ++step) {
        const int t = step_frame(a, step);
        RNNG_STAMP(0);
        __amdgpu_buffer_rsrc_t rs[SM::NSRC];
#pragma unroll
        for (int sidx = 0; sidx < SM::NSRC; ++sidx) {
            const StepSource& sc = sh.lay.src[sidx];
            const int frame = t + suni(sc.frame_off);
            const bool in_window = frame >= 0 && frame < T;
            const float* g = ((cbufs_t)a.buf_ptr)[(SM::XB ? a.twin_base : 0) + suni(sc.buf)] + (size_t)(in_window ? frame : 0) * N * SM::K(sidx);
            rs[sidx] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(g), 0, in_window ? N * SM::K(sidx) * 4 : 0, STEP_RSRC_FLAGS);
        }
        muintx4 v[D][SM::MT];
        mfloatx4 wb[D][SM::NTU];
        auto load_a = [&](muintx4 (&dst)[SM::MT], const __amdgpu_buffer_rsrc_t& rsrc, const int (&base)[SM::MT], int K, bool k_ragged, int k0, bool on) {
#pragma unroll
            for (int mt = 0; mt < SM::MT; ++mt) {
                int off = base[mt] + (SM::XB ? k0 * 64 : k0 * 4);
                if (k_ragged) off = k0 + (SM::XB ? wave * 16 : wcol) < K ? off : 0x7FFFFFF0;
                off = on ? off : 0x7FFFFFF0;
                dst[mt] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, STEP_COHERENT_AUX);
            }
        };
        auto load_b = [&](mfloatx4 (&dst)[SM::NTU], const unsigned (&base)[SM::NTU], int K, bool k_ragged, int k0, bool on) {
#pragma unroll
            for (int nt = 0; nt < SM::NTU; ++nt) {
                unsigned off = base[nt] + (unsigned)(k0 * 4);
                if (k_ragged) off = k0 + wcol < K ? off : 0xC0000000u;
                off = on ? off : 0xC0000000u;
                const muintx4 x = __builtin_amdgcn_raw_buffer_load_b128(rwb, (int)off, 0, 0);
                dst[nt] = mfloatx4{__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
            }
        };
        auto incomplete = [&](const muintx4 (&x)[SM::MT]) {
            unsigned m = 0;
#pragma unroll
            for (int mt = 0; mt < SM::MT; ++mt) {
                const unsigned m1 = x[mt].x > x[mt].y ? x[mt].x : x[mt].y, m2 = x[mt].z > x[mt].w ? x[mt].z : x[mt].w;
                const unsigned m3 = m1 > m2 ? m1 : m2;
                m = m > m3 ? m : m3;
            }
            return __builtin_amdgcn_ballot_w64(m == STEP_SENTINEL) != 0;
        };
        // the weights of the first chunks do not wait for the exchange
        step_static_for<0, D - 1>([&](auto ii) {
            constexpr int i = decltype(ii)::value;
            load_b(wb[i], boff[0], SM::K(0), SM::K(0) % CW != 0, i * CW, i * CW < (SM::K(0) + CW - 1) / CW * CW);
        });
        for (int i = 0; i < pdelay; ++i) __builtin_amdgcn_s_sleep(1);
        bool retried = false;
        step_static_for<0, D - 1>([&](auto ii) {
            constexpr int i = decltype(ii)::value;
            load_a(v[i], rs[0], aoff[0], SM::K(0), SM::K(0) % CW != 0, i * CW, i * CW < (SM::K(0) + CW - 1) / CW * CW);
        });
        mfloatx4 acc[SM::MT][SM::NTU];
#pragma unroll
        for (int mt = 0; mt < SM::MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < SM::NTU; ++nt) acc[mt][nt] = mfloatx4{0.0f, 0.0f, 0.0f, 0.0f};
        bool bad = incomplete(v[0]);

        step_static_for<0, SM::NSRC>([&](auto ss) {
            constexpr int sidx = decltype(ss)::value;
            constexpr int NGR = SM::ngr(sidx);
            constexpr int KP = (SM::K(sidx) + CW - 1) / CW * CW;
            constexpr int snext = sidx + 1 < SM::NSRC ? sidx + 1 : sidx;
            constexpr int KPN = (SM::K(snext) + CW - 1) / CW * CW;
#pragma unroll 1
            for (int g = 0; g < NGR; ++g) {
                step_static_for<0, D>([&](auto ii) {
                    constexpr int i = decltype(ii)::value;
                    constexpr int j = (i + D - 1) % D;
                    constexpr int i1 = (i + 1) % D;
                    const int k0 = (g * D + i) * CW;
                    const int gj = i == 0 ? g : g + 1;
                    const bool same = gj < NGR;
                    const int kj = same ? (gj * D + j) * CW : j * CW;
                    const bool on = same ? kj < KP : (sidx + 1 < SM::NSRC && kj < KPN);
                    auto ahead = [&]() {
                        if (same) {
                            load_b(wb[j], boff[sidx], SM::K(sidx), SM::K(sidx) % CW != 0, kj, on);
                            load_a(v[j], rs[sidx], aoff[sidx], SM::K(sidx), SM::K(sidx) % CW != 0, kj, on);
                        } else {
                            load_b(wb[j], boff[snext], SM::K(snext), SM::K(snext) % CW != 0, kj, on);
                            load_a(v[j], rs[snext], aoff[snext], SM::K(snext), SM::K(snext) % CW != 0, kj, on);
                        }
                    };
                    if (k0 < KP) {
                        if (bad && !dead) {
                            retried = true;
                            muintx4 again[SM::MT];
                            int spins = 0;
                            for (;;) {
                                if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicExch(a.ctrl, 1u); break; }
                                __builtin_amdgcn_s_sleep(MSTEP_RETRY_SLEEP);
                                step_compiler_barrier();
                                load_a(again, rs[sidx], aoff[sidx], SM::K(sidx), SM::K(sidx) % CW != 0, k0, true);
                                if (!incomplete(again)) break;
                            }
#pragma unroll
                            for (int mt = 0; mt < SM::MT; ++mt) v[i][mt] = again[mt];
                        }
                        if (sidx == 0 && i == 0 && g == 0) { RNNG_STAMP(2); }
                        // the operands of this chunk, before the set of the chunk before it is loaded again
                        mfloatx4 opb[SM::NTU];
#pragma unroll
                        for (int nt = 0; nt < SM::NTU; ++nt) opb[nt] = wb[i][nt];
                        ahead();
                        bad = incomplete(v[i1]);
#pragma unroll
                        for (int mt = 0; mt < SM::MT; ++mt)
#pragma unroll
                            for (int nt = 0; nt < SM::NTU; ++nt)
                                if (SM::used(sidx, nt)) {
                                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[i][mt].x), opb[nt][0], acc[mt][nt], 0, 0, 0);
                                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[i][mt].y), opb[nt][1], acc[mt][nt], 0, 0, 0);
                                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[i][mt].z), opb[nt][2], acc[mt][nt], 0, 0, 0);
                                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(v[i][mt].w), opb[nt][3], acc[mt][nt], 0, 0, 0);
                                }
                    } else {
                        ahead();
                        bad = incomplete(v[i1]);
                    }
                });
            }
        });
        // ---- hand the accumulators to the element-wise threads: one partial tile per wavefront ----
        {
            const int tb = wave * (NPAD * ACCS);
#pragma unroll
            for (int mt = 0; mt < SM::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < SM::NTU; ++nt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        lds[tb + (mt * 16 + 4 * (lane >> 4) + i) * ACCS + nt * 16 + (lane & 15)] = acc[mt][nt][i];
        }
        RNNG_STAMP(3);
        if (__syncthreads_or(retried ? 1 : 0)) pdelay = pdelay + MSTEP_POLL_INC < 96 ? pdelay + MSTEP_POLL_INC : 96;
        else if ((step & 63) == 63 && pdelay > 0) --pdelay;
        RNNG_STAMP(4);
        // ---- element-wise program: IPT passes, one thread per (stream, unit) in each ----
        // (not unrolled: interleaved passes would keep several slot files in registers)
#pragma unroll 1
        for (int p = 0; p < IPT; ++p) {
            const int pn = item_n + p * SPP;      // the pass's stream
            if (r.n < 0 || pn >= N) continue;
            float s[MAX_SLOTS];
#pragma unroll
            for (int g = 0; g < PH::NG; ++g) {
                if (PH::gkind(g) == GA_KIND_ACC) {
                    float x = 0.0f;
                    if (r.gptr[g] != nullptr) {
                        const int tb = pn * ACCS + PH::gaux(g) * CMAX + item_il;
                        x = (lds[tb] + lds[tb + NPAD * ACCS]) + (lds[tb + 2 * NPAD * ACCS] + lds[tb + 3 * NPAD * ACCS]);
                        if constexpr (NW == 8)
                            x += (lds[tb + 4 * NPAD * ACCS] + lds[tb + 5 * NPAD * ACCS]) + (lds[tb + 6 * NPAD * ACCS] + lds[tb + 7 * NPAD * ACCS]);
                    }
                    s[g] = x;
                } else if (PH::gkind(g) == GA_KIND_CARRY && step > 0 && IPT == 1) {
                    s[g] = carry[p][PH::cidx(g)];
                } else if (PH::gkind(g) == GA_KIND_STATIC && step > 0 && IPT == 1) {
                    s[g] = sn[p][g];
                } else {
                    // (with several passes a step is long, and values kept per pass would cost the
                    // registers that eight wavefronts need: everything is loaded where it is used,
                    // also what the thread itself stored in the step before)
                    const int frame = t + r.goff[g];
                    float x = 0.0f;
                    if (r.gptr[g] != nullptr && frame >= 0 && frame < T) {
                        const float* src = r.gptr[g] + (long long)frame * r.gstride[g] + (long long)p * gpass[g];
                        x = PH::gkind(g) == GA_KIND_STATIC ? *src : load_coherent(src);
                    }
                    s[g] = x;
                }
            }
#pragma unroll
            for (int q = 0; q < PH::NI; ++q) s[PH::NG + q] = r.inv[q];
            PH::ops(s);
#pragma unroll
            for (int q = 0; q < PH::NST; ++q) {
                if (r.sptr[q] == nullptr) continue;
                float* dst = r.sptr[q] + (long long)t * r.sstride[q] + (long long)p * spass[q];
                if (PH::stshared(q) && SM::XB) {
                    // (SPP streams further on = SPP / 16 stream tiles = the same distance as in the row-major tensor)
                    store_plain(dst, s[PH::stslot(q)]);
                    store_shared(xptr[q] + (long long)t * r.sstride[q] + (long long)p * spass[q], s[PH::stslot(q)]);
                } else if (PH::stshared(q)) store_shared(dst, s[PH::stslot(q)]);
                else store_plain(dst, s[PH::stslot(q)]);
            }
#pragma unroll
            for (int g = 0; g < PH::NG; ++g)
                if (PH::gkind(g) == GA_KIND_CARRY && IPT == 1) carry[p][PH::cidx(g)] = s[PH::gaux(g)];
            // STATIC inputs of the next step
            if (step + 1 < nsteps && IPT == 1) {
                const int t2 = a.backward ? t - 1 : t + 1;
#pragma unroll
                for (int g = 0; g < PH::NG; ++g)
                    if (PH::gkind(g) == GA_KIND_STATIC) {
                        const int frame = t2 + r.goff[g];
                        float x = 0.0f;
                        if (r.gptr[g] != nullptr && frame >= 0 && frame < T) x = r.gptr[g][(long long)frame * r.gstride[g] + (long long)p * gpass[g]];
                        sn[p][g] = x;
                    }
            }
        }
        RNNG_STAMP(5);
        step_lds_barrier();   // the tiles are written again in the next step
    }
}

}  // namespace rnng
