// Device-side interpreter of node programs (see program.h for the encoding).
//
// All control flow depends only on program words, which are forced into scalar registers, so
// the slot file is indexed with uniform indices and stays in vector registers.
#pragma once
#include <hip/hip_runtime.h>

#include "program.h"

namespace rnng {

__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + __expf(-x)); }
// tanh without cancellation near 0: t = e^{-2|x|}; tanh|x| = (1 - t) / (1 + t).
__device__ __forceinline__ float tanh_f(float x) {
    const float ax = fabsf(x);
    const float t = __expf(-2.0f * ax);
    const float r = (1.0f - t) / (1.0f + t);
    return copysignf(r, x);
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Ownership of units: workgroup part `w` of `G` owns units [w * chunk, (w + 1) * chunk) of a
// layer of width dim, chunk = ceil(dim / G).  A thread works on local unit il of every layer.
struct UnitMap {
    int w, G, il;
    __device__ __forceinline__ int unit(int dim, bool& active) const {
        const int chunk = (dim + G - 1) / G;
        const int i = w * chunk + il;
        active = il < chunk && i < dim;
        return i;
    }
};

struct ProgramView {
    cwords_t ga; cwords_t iv; cwords_t mo; cwords_t st;
    int n_gather, n_inv, n_ops, n_stores;
    __device__ __forceinline__ explicit ProgramView(const int32_t* gp) {
        cwords_t p = (cwords_t)gp;
        n_gather = uni(p[PG_NGATHER]); n_inv = uni(p[PG_NINV]); n_ops = uni(p[PG_NOPS]); n_stores = uni(p[PG_NSTORES]);
        ga = p + PG_HEADER_WORDS; iv = ga + n_gather * GA_WORDS; mo = iv + n_inv * IV_WORDS; st = mo + n_ops * MO_WORDS;
    }
};

// slots [n_gather, n_gather + n_inv): diagonal weights and biases (independent of t and n).
__device__ __forceinline__ void load_invariants(float (&s)[MAX_SLOTS], const ProgramView& pg,
                                                const float* __restrict__ weights, const UnitMap& um) {
    for (int v = 0; v < pg.n_inv; ++v) {
        cwords_t e = pg.iv + v * IV_WORDS;
        bool active;
        const int i = um.unit(uni(e[IV_DIM]), active);
        s[pg.n_gather + v] = active ? weights[uni(e[IV_W_OFF]) + i] : 0.0f;
    }
}

// slots [0, n_gather): values of frame tensors at (t + frame_off, n, i); AccFn supplies the
// matrix-vector accumulator entries: acc(buffer id, dim, n, i, il).
template <class AccFn>
__device__ __forceinline__ void load_gathers(float (&s)[MAX_SLOTS], const ProgramView& pg, const PlanView& pv,
                                             const UnitMap& um, int T, int N, int t, int n, AccFn acc, bool with_acc) {
    for (int g = 0; g < pg.n_gather; ++g) {
        cwords_t e = pg.ga + g * GA_WORDS;
        const int dim = uni(e[GA_DIM]), buf = uni(e[GA_BUF]);
        bool active;
        const int i = um.unit(dim, active);
        if (uni(e[GA_KIND]) == GA_KIND_ACC) {
            if (with_acc) s[g] = active ? acc(buf, dim, n, i, um.il) : 0.0f;
        } else {
            const int frame = t + uni(e[GA_FRAME_OFF]);
            float v = 0.0f;
            if (active && frame >= 0 && frame < T) v = ((cbufs_t)pv.buf_ptr)[buf][((size_t)frame * N + n) * dim + i];
            s[g] = v;
        }
    }
}

// Only the accumulator slots (used when the other gathers were issued earlier).
template <class AccFn>
__device__ __forceinline__ void load_accumulators(float (&s)[MAX_SLOTS], const ProgramView& pg, const UnitMap& um,
                                                  int n, AccFn acc) {
    for (int g = 0; g < pg.n_gather; ++g) {
        cwords_t e = pg.ga + g * GA_WORDS;
        if (uni(e[GA_KIND]) != GA_KIND_ACC) continue;
        const int dim = uni(e[GA_DIM]);
        bool active;
        const int i = um.unit(dim, active);
        s[g] = active ? acc(uni(e[GA_BUF]), dim, n, i, um.il) : 0.0f;
    }
}

__device__ __forceinline__ void run_ops(float (&s)[MAX_SLOTS], const ProgramView& pg) {
    for (int p = 0; p < pg.n_ops; ++p) {
        const int packed = uni(pg.mo[p * MO_WORDS + MO_PACKED]);
        const int opc = packed & 0xFF, d = (packed >> 8) & 0xFF, a = (packed >> 16) & 0xFF, b = (packed >> 24) & 0xFF;
        const float va = s[a];
        float r;
        switch (opc) {
            case MOP_MOV: r = va; break;
            case MOP_ADD: r = va + s[b]; break;
            case MOP_MUL: r = va * s[b]; break;
            case MOP_FMA: r = fmaf(va, s[b], s[uni(pg.mo[p * MO_WORDS + MO_C])]); break;
            case MOP_SIG: r = sigmoid_f(va); break;
            case MOP_TANH: r = tanh_f(va); break;
            case MOP_DSIG: { const float y = s[b]; r = va * y * (1.0f - y); break; }
            case MOP_DTANH: { const float y = s[b]; r = va * (1.0f - y * y); break; }
            case MOP_RELU: r = fmaxf(va, 0.0f); break;
            case MOP_DRELU: r = s[b] > 0.0f ? va : 0.0f; break;
            case MOP_MAX: r = fmaxf(va, s[b]); break;
            case MOP_GE: r = va >= s[b] ? 1.0f : 0.0f; break;
            case MOP_GT: r = va > s[b] ? 1.0f : 0.0f; break;
            default: r = 0.0f; break;
        }
        s[d] = r;
    }
}

// StoreFn(ptr, value) performs the store (plain, or with a wider visibility scope).
template <class StoreFn>
__device__ __forceinline__ void run_stores(const float (&s)[MAX_SLOTS], const ProgramView& pg, const PlanView& pv,
                                           const UnitMap& um, int N, int t, int n, StoreFn store) {
    for (int q = 0; q < pg.n_stores; ++q) {
        cwords_t e = pg.st + q * ST_WORDS;
        const int dim = uni(e[ST_DIM]);
        bool active;
        const int i = um.unit(dim, active);
        if (active) store(((cbufs_t)pv.buf_ptr)[uni(e[ST_BUF])] + ((size_t)t * N + n) * dim + i, s[uni(e[ST_SLOT])]);
    }
}

}  // namespace rnng
