// Persistent recurrent-step kernel: one launch runs all T sequential steps of one recurrent
// node in one direction (paper Section 3.1: inside a recurrent node the frames are stepped one
// after another; per step the delayed connections come first, then the delay-0 part level by
// level; the backward pass runs the same scheme in reverse).
//
// G workgroups each own a chunk of every layer's units and keep their rows (forward) or
// columns (backward) of every full weight matrix inside the recurrent node resident in LDS for
// all T steps.  The only data that crosses workgroups is the source vector of those full
// connections (e.g. the block output h(t-1)).  There is no grid barrier: the shared vectors
// are pre-filled with a sentinel bit pattern, producers overwrite each element exactly once
// with a device-scope store, and consumers poll the elements they need until none holds the
// sentinel.  Every wait is bounded by a spin limit; on expiry an error word is set and the
// kernel runs to its end without waiting again, so the grid always drains.
#include "interp.h"
#include "kernels.h"
#include "step_layout.h"

namespace rnng {
namespace {

constexpr unsigned SENTINEL = 0xFFFFFFFFu;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

struct StepArgs {
    PlanView pv;
    const float* weights;
    unsigned* ctrl;          // [0]: set to 1 when a wait ran into the spin limit
    int desc_off, T, N, backward, G, xcd_stride, spin_limit;
};

__device__ __forceinline__ void store_shared(float* p, float v) {
    unsigned b = __float_as_uint(v);
    if (b == SENTINEL) b = 0x7FC00000u;    // a NaN result must not look like "not yet written"
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
                if (lo != SENTINEL && hi != SENTINEL) break;
                if (dead) break;
                if (++spins > spin_limit) { dead = true; atomicExch(ctrl, 1u); break; }
            }
            const int n = (2 * p) / K, k = 2 * p - n * K;
            floatx2 o = {__uint_as_float(lo), __uint_as_float(hi)};
            *reinterpret_cast<floatx2*>(&x[n * k_pad + k]) = o;
        }
    } else {
        for (int p = tid; p < total; p += STEP_THREADS) {
            const unsigned* src = reinterpret_cast<const unsigned*>(g) + p;
            unsigned v;
            int spins = 0;
            for (;;) {
                v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v != SENTINEL) break;
                if (dead) break;
                if (++spins > spin_limit) { dead = true; atomicExch(ctrl, 1u); break; }
            }
            const int n = p / K, k = p - n * K;
            x[n * k_pad + k] = __uint_as_float(v);
        }
    }
}

template <int NB>
__global__ __launch_bounds__(STEP_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void recurrent_step_kernel(StepArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ StepLayout lay;
    __shared__ unsigned short tinfo[STEP_MAX_PHASES][STEP_THREADS];   // task of the thread's matrix-vector slot
    __shared__ unsigned iteminfo[STEP_MAX_PHASES][STEP_THREADS];      // element-wise item: local unit | stream << 16

    int w = blockIdx.x;
    if (a.xcd_stride > 1) {
        if (w % a.xcd_stride) return;      // workgroups are dealt round-robin to the XCDs: keep one XCD's share
        w /= a.xcd_stride;
    }
    if (w >= a.G) return;
    const int tid = threadIdx.x;
    const int T = a.T, N = a.N, G = a.G;
    const PlanView pv = a.pv;

    if (tid == 0) compute_step_layout(pv.words, a.desc_off, G, NB, N, lay);
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
        tinfo[p][tid] = tk;
        const int il = tid % ph.item_chunk, n = tid / ph.item_chunk;
        iteminfo[p][tid] = (unsigned)il | ((unsigned)(n < N ? n : 0xFFFF) << 16);
    }
    __syncthreads();

    // Resident weights: lane-major float4 blocks, zero beyond a row's length or a layer's width.
    for (int p = 0; p < n_phases; ++p) {
        const StepPhase& ph = lay.ph[p];
        const int tk = tinfo[p][tid];
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
            for (int j = 0; j < Jt; ++j) {
                const int k0 = 4 * (sl + ph.L * j);
                floatx4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (uok) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int k = k0 + c;
                        if (k < ed.k_len) v[c] = ed.transposed ? W[(size_t)k * task.n_out + u] : W[(size_t)u * ed.k_len + k];
                    }
                }
                *reinterpret_cast<floatx4*>(&lds[ph.w_base[e] + (j * STEP_THREADS + tid) * 4]) = v;
            }
        }
    }
    __syncthreads();

    float s[MAX_SLOTS];
    bool dead = false;
    int acc_phase = 0;
    for (int step = 0; step < T; ++step) {
        const int t = a.backward ? T - 1 - step : step;
        for (int p = 0; p < n_phases; ++p) {
            const StepPhase& ph = lay.ph[p];
            const ProgramView pg(pv.words + uni(ph.prog_off));
            const unsigned item = iteminfo[p][tid];
            const int n = (int)(item >> 16);
            const bool has_item = n != 0xFFFF;
            const UnitMap um{w, G, (int)(item & 0xFFFF)};
            const int n_tasks = uni(ph.n_tasks);

            // 1. element-wise inputs of this step (own units only): issued now, consumed after the
            //    matrix-vector part, so their latency overlaps the wait for the shared vectors
            if (has_item) {
#pragma unroll
                for (int g = 0; g < STEP_MAX_GATHERS; ++g) {
                    if (g < pg.n_gather) {
                        const int32_t* e = pg.ga + g * GA_WORDS;
                        if (uni(e[GA_KIND]) == GA_KIND_FRAMES) {
                            const int dim = uni(e[GA_DIM]);
                            bool active;
                            const int i = um.unit(dim, active);
                            const int frame = t + uni(e[GA_FRAME_OFF]);
                            float v = 0.0f;
                            if (active && frame >= 0 && frame < T)
                                v = load_coherent(pv.buf_ptr[uni(e[GA_BUF])] + ((size_t)frame * N + n) * dim + i);
                            s[g] = v;
                        }
                    }
                }
                if (n_phases > 1 || step == 0) load_invariants(s, pg, a.weights, um);
            }

            if (n_tasks > 0) {
                acc_phase = p;
                // 2. shared source vectors first used in this phase
                for (int q = 0; q < lay.n_sources; ++q) {
                    const StepSource& sc = lay.src[q];
                    if (sc.first_phase != p) continue;
                    const int frame = t + sc.frame_off;
                    float* x = lds + sc.x_base;
                    if (frame < 0 || frame >= T) {
                        for (int i = tid; i < N * sc.k_len; i += STEP_THREADS) { const int nn = i / sc.k_len; x[nn * sc.k_pad + i - nn * sc.k_len] = 0.0f; }
                    } else {
                        poll_source(x, pv.buf_ptr[sc.buf] + (size_t)frame * N * sc.k_len, N, sc.k_len, sc.k_pad, tid,
                                    a.spin_limit, dead, a.ctrl);
                    }
                }
                __syncthreads();
                // 3. matrix-vector products from LDS-resident weights
                const int tk = tinfo[p][tid];
                if (tk != 0xFFFF) {
                    const StepTask& task = ph.task[tk];
                    const int L = ph.L, sl = tid & (L - 1);
                    float part[NB];
#pragma unroll
                    for (int nn = 0; nn < NB; ++nn) part[nn] = 0.0f;
                    const int n_edges = task.n_edges;
                    for (int e = 0; e < n_edges; ++e) {
                        const int k_len = task.e[e].k_len;
                        const StepSource& sc = lay.src[task.e[e].src];
                        const int xb = sc.x_base + 4 * sl, kp = sc.k_pad;
                        const int Jt = (k_len + 4 * L - 1) / (4 * L);
                        const float* wp = lds + ph.w_base[e] + tid * 4;
                        for (int j = 0; j < Jt; ++j) {
                            const floatx4 w4 = *reinterpret_cast<const floatx4*>(wp + j * STEP_THREADS * 4);
#pragma unroll
                            for (int nn = 0; nn < NB; ++nn) {
                                const floatx4 x4 = *reinterpret_cast<const floatx4*>(lds + xb + nn * kp + 4 * L * j);
                                part[nn] += w4.x * x4.x + w4.y * x4.y + w4.z * x4.z + w4.w * x4.w;
                            }
                        }
                    }
                    for (int off = L >> 1; off > 0; off >>= 1) {
#pragma unroll
                        for (int nn = 0; nn < NB; ++nn) part[nn] += __shfl_xor(part[nn], off, 64);
                    }
                    if (sl == 0) {
                        const int slot = tid / L;
#pragma unroll
                        for (int nn = 0; nn < NB; ++nn) lds[ph.acc_base + slot * NB + nn] = part[nn];
                    }
                }
                __syncthreads();
            }

            // 4. accumulators -> slots, straight-line program, stores
            if (has_item) {
                const StepPhase& aph = lay.ph[acc_phase];
                const int acc_base = aph.acc_base, cmax = aph.cmax;
#pragma unroll
                for (int g = 0; g < STEP_MAX_GATHERS; ++g) {
                    if (g < pg.n_gather) {
                        const int32_t* e = pg.ga + g * GA_WORDS;
                        if (uni(e[GA_KIND]) == GA_KIND_ACC) {
                            bool active;
                            um.unit(uni(e[GA_DIM]), active);
                            s[g] = active ? lds[acc_base + (uni(e[GA_FRAME_OFF]) * cmax + um.il) * NB + n] : 0.0f;
                        }
                    }
                }
                run_ops(s, pg);
                run_stores(s, pg, pv, um, N, t, n, [](float* p, float v) { store_shared(p, v); });
            }
            if (n_phases > 1) __syncthreads();
        }
    }
}

__global__ __launch_bounds__(256) void fill_bits_kernel(unsigned* __restrict__ p, long long n, unsigned v) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += 256LL * gridDim.x) p[i] = v;
}

}  // namespace

int step_nb_for(int N) { return N <= 1 ? 1 : N <= 2 ? 2 : N <= 4 ? 4 : N <= 8 ? 8 : 0; }

bool plan_step_launch(const int32_t* words, int desc_off, int N, int force_G, StepLaunchPlan& out) {
    const int NB = step_nb_for(N);
    out.ok = false;
    if (NB == 0) return false;
    StepLayout lay;
    const int candidates[6] = {32, 16, 8, 64, 128, 256};
    for (int c = 0; c < 6; ++c) {
        const int G = force_G > 0 ? force_G : candidates[c];
        compute_step_layout(words, desc_off, G, NB, N, lay);
        const size_t bytes = (size_t)lay.total_floats * 4;
        if (lay.ok && bytes <= STEP_LDS_LIMIT) {
            out.ok = true; out.G = G; out.NB = NB; out.lds_bytes = bytes;
            out.xcd_stride = G <= 32 ? 8 : 1;
            return true;
        }
        if (force_G > 0) break;
    }
    return false;
}

hipError_t launch_recurrent_steps(const PlanView& pv, const StepLaunchPlan& lp, int desc_off, const float* weights,
                                  unsigned* ctrl, int T, int N, bool backward, int spin_limit, hipStream_t stream) {
    StepArgs a;
    a.pv = pv; a.weights = weights; a.ctrl = ctrl; a.desc_off = desc_off; a.T = T; a.N = N; a.backward = backward ? 1 : 0;
    a.G = lp.G; a.xcd_stride = lp.xcd_stride; a.spin_limit = spin_limit;
    const dim3 grid(lp.G * lp.xcd_stride), block(STEP_THREADS);
    hipError_t e = hipSuccess;
#define RNNG_LAUNCH(NBV)                                                                                              \
    do {                                                                                                              \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&recurrent_step_kernel<NBV>),                           \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)STEP_LDS_LIMIT);                      \
        if (e != hipSuccess) return e;                                                                                \
        hipLaunchKernelGGL((recurrent_step_kernel<NBV>), grid, block, lp.lds_bytes, stream, a);                       \
    } while (0)
    switch (lp.NB) {
        case 1: RNNG_LAUNCH(1); break;
        case 2: RNNG_LAUNCH(2); break;
        case 4: RNNG_LAUNCH(4); break;
        case 8: RNNG_LAUNCH(8); break;
        default: return hipErrorInvalidValue;
    }
#undef RNNG_LAUNCH
    return hipGetLastError();
}

hipError_t launch_fill_sentinel(float* p, int64_t n, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    long long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_bits_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, reinterpret_cast<unsigned*>(p),
                       (long long)n, SENTINEL);
    return hipGetLastError();
}

}  // namespace rnng
