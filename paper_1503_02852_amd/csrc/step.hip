// Persistent recurrent-step kernel, ahead-of-time build: the element-wise programs are
// interpreted from the plan words (any component, any number of phases).  The shared device
// code and the description of the scheme are in step_device.h; jit.cpp builds the same kernel
// with a component's programs emitted as straight-line code.
#include "interp.h"
#include "kernels.h"
#include "step_device.h"

namespace rnng {
namespace {

template <int NB>
__global__ __launch_bounds__(STEP_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void recurrent_step_kernel(StepArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ StepShared sh;
    const int w = step_prologue<NB>(a, sh, lds);
    if (w < 0) return;
    const int tid = threadIdx.x;
    const int T = a.T, N = a.N, G = a.G;
    const StepLayout& lay = sh.lay;
    const int n_phases = suni(lay.n_phases);
    PlanView pv;
    pv.buf_ptr = a.buf_ptr; pv.buf_dim = nullptr; pv.words = a.words;

    float s[MAX_SLOTS];
    bool dead = false;
    int acc_phase = 0;
    const int nsteps = step_count(a);
    for (int step = 0; step < nsteps; ++step) {
        const int t = step_frame(a, step);
        for (int p = 0; p < n_phases; ++p) {
            const StepPhase& ph = lay.ph[p];
            const ProgramView pg(a.words + suni(ph.prog_off));
            const unsigned item = sh.iteminfo[p][tid];
            const int n = (int)(item >> 16);
            const bool has_item = n != 0xFFFF;
            const UnitMap um{w, G, (int)(item & 0xFFFF)};
            const int n_tasks = suni(ph.n_tasks);

            // 1. element-wise inputs of this step (own units only): issued now, consumed after the
            //    matrix-vector part, so their latency overlaps the wait for the shared vectors
            if (has_item) {
#pragma unroll
                for (int g = 0; g < STEP_MAX_GATHERS; ++g) {
                    if (g < pg.n_gather) {
                        cwords_t e = pg.ga + g * GA_WORDS;
                        if (e[GA_KIND] != GA_KIND_ACC) {
                            const int dim = e[GA_DIM];
                            bool active;
                            const int i = um.unit(dim, active);
                            const int frame = t + e[GA_FRAME_OFF];
                            float v = 0.0f;
                            if (active && frame >= 0 && frame < T)
                                v = load_coherent(((cbufs_t)a.buf_ptr)[e[GA_BUF]] + ((size_t)frame * N + n) * dim + i);
                            s[g] = v;
                        }
                    }
                }
                if (n_phases > 1 || step == 0) load_invariants(s, pg, a.weights, um);
            }

            if (n_tasks > 0) {
                acc_phase = p;
                poll_phase_sources(a, sh, lds, p, t, tid, dead);
                __syncthreads();
                MatvecRegs mr;
                matvec_setup<NB>(mr, sh, p, tid);
                matvec_run<NB>(mr, lds);
                __syncthreads();
            }

            // 4. accumulators -> slots, program, stores
            if (has_item) {
                const StepPhase& aph = lay.ph[acc_phase];
                const int acc_base = aph.acc_base, cmax = aph.cmax;
#pragma unroll
                for (int g = 0; g < STEP_MAX_GATHERS; ++g) {
                    if (g < pg.n_gather) {
                        cwords_t e = pg.ga + g * GA_WORDS;
                        if (e[GA_KIND] == GA_KIND_ACC) {
                            bool active;
                            um.unit(e[GA_DIM], active);
                            s[g] = active ? lds[acc_base + (e[GA_FRAME_OFF] * cmax + um.il) * NB + n] : 0.0f;
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

// blockIdx.y: the range
__global__ __launch_bounds__(256) void fill_ranges_kernel(const FillRanges r, unsigned v) {
    unsigned* __restrict__ p = reinterpret_cast<unsigned*>(r.p[blockIdx.y]);
    const long long n = r.n[blockIdx.y];
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

namespace {
__global__ __launch_bounds__(STEP_THREADS) void xcc_probe_kernel(unsigned* out) {
    if (threadIdx.x == 0) out[blockIdx.x] = (unsigned)step_xcc_id();
}
}  // namespace

hipError_t launch_xcc_probe(unsigned* out, int n_blocks, hipStream_t stream) {
    hipLaunchKernelGGL(xcc_probe_kernel, dim3(n_blocks), dim3(STEP_THREADS), 0, stream, out);
    return hipGetLastError();
}

void fill_step_args(StepArgs& a, const PlanView& pv, const StepLaunchPlan& lp, int desc_off, const float* weights,
                    unsigned* ctrl, int T, int N, bool backward, int spin_limit, int t_begin, int t_end) {
    a.t_begin = t_begin; a.t_end = t_end; a.J = 1;
    a.buf_ptr = pv.buf_ptr; a.words = pv.words; a.weights = weights; a.ctrl = ctrl; a.desc_off = desc_off;
    a.T = T; a.N = N; a.backward = backward ? 1 : 0; a.G = lp.G; a.xcd_stride = lp.xcd_stride; a.spin_limit = spin_limit;
    a.n_groups = 0; a.partial = nullptr; a.store_base = nullptr; a.store_bytes = 0; a.weights_t = nullptr; a.weight_bytes = 0; a.twin_base = 0;
    for (int g = 0; g < STEP_MAX_GROUPS; ++g) { a.grp_desc_off[g] = 0; a.grp_G[g] = 0; a.grp_J[g] = 1; a.grp_first[g] = 0; a.xcc_expect[g] = -1; }
}

hipError_t launch_recurrent_steps(const PlanView& pv, const StepLaunchPlan& lp, int desc_off, const float* weights,
                                  unsigned* ctrl, int T, int N, bool backward, int spin_limit, int t_begin, int t_end,
                                  hipStream_t stream) {
    StepArgs a;
    fill_step_args(a, pv, lp, desc_off, weights, ctrl, T, N, backward, spin_limit, t_begin, t_end);
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
                       (long long)n, STEP_SENTINEL);
    return hipGetLastError();
}

hipError_t launch_fill_sentinel_ranges(const FillRanges& r, hipStream_t stream) {
    if (r.count <= 0) return hipSuccess;
    if (r.count > FILL_MAX_RANGES) return hipErrorInvalidValue;
    long long most = 0;
    for (int i = 0; i < r.count; ++i) most = r.n[i] > most ? r.n[i] : most;
    if (most <= 0) return hipSuccess;
    long long blocks = (most + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_ranges_kernel, dim3((unsigned)blocks, (unsigned)r.count), dim3(256), 0, stream, r, STEP_SENTINEL);
    return hipGetLastError();
}

}  // namespace rnng
