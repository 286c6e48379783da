// Device-side interpreter of node programs (see program.h for the encoding).
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

// Value of one factor for (frame t, stream n, unit i).  `words` points at the factor.
__device__ __forceinline__ float factor_value(const PlanView& pv, const int32_t* __restrict__ f,
                                              const float* __restrict__ weights, const float* slots,
                                              int T, int N, int t, int n, int i) {
    float v;
    const int slot = f[FACTOR_SLOT];
    if (slot >= 0) {
        v = slots[slot];
    } else {
        const int frame = t + f[FACTOR_FRAME_OFF];
        if (frame < 0 || frame >= T) return 0.0f;
        const int buf = f[FACTOR_BUF];
        v = pv.buf_ptr[buf][((size_t)frame * N + n) * pv.buf_dim[buf] + i];
    }
    const int w_off = f[FACTOR_W_OFF];
    if (w_off >= 0) v *= weights[w_off + i];
    return v;
}

// Evaluates every NodeOp of a program for one (t, n, i).  Control flow depends only on the
// program words, so it is uniform across a wavefront; lanes with i >= dim of an op idle.
__device__ __forceinline__ void run_node_program(const PlanView& pv, const int32_t* __restrict__ prog,
                                                 const float* __restrict__ weights,
                                                 int T, int N, int t, int n, int i) {
    float slots[MAX_SLOTS];
    const int n_ops = prog[PROG_NOPS];
    const int32_t* w = prog + PROG_HEADER_WORDS;
    for (int o = 0; o < n_ops; ++o) {
        const int dim = w[OP_DIM];
        const int n_terms = w[OP_NTERMS];
        const bool active = i < dim;
        float v = 0.0f;
        if (active) {
            const int pre = w[OP_PRE_BUF], bias = w[OP_BIAS_OFF], acc = w[OP_ACC_BUF];
            if (pre >= 0) v += pv.buf_ptr[pre][((size_t)t * N + n) * dim + i];
            if (bias >= 0) v += weights[bias + i];
            if (acc >= 0) v += pv.buf_ptr[acc][(size_t)n * dim + i];
        }
        const int32_t* tw = w + OP_HEADER_WORDS;
        for (int q = 0; q < n_terms; ++q) {
            const int nf = tw[0];
            ++tw;
            float prod = 1.0f;
            for (int j = 0; j < nf; ++j) {
                if (active) prod *= factor_value(pv, tw, weights, slots, T, N, t, n, i);
                tw += FACTOR_WORDS;
            }
            v += prod;
        }
        if (active) {
            const int post = w[OP_POST];
            if (post == POST_SIGMOID) v = sigmoid_f(v);
            else if (post == POST_TANH) v = tanh_f(v);
            else if (post >= POST_DSIGMOID) {
                const int db = w[OP_DERIV_BUF];
                const float y = pv.buf_ptr[db][((size_t)t * N + n) * dim + i];
                v *= (post == POST_DSIGMOID) ? y * (1.0f - y) : (1.0f - y * y);
            }
            pv.buf_ptr[w[OP_OUT_BUF]][((size_t)t * N + n) * dim + i] = v;
        }
        const int os = w[OP_OUT_SLOT];
        if (os >= 0) slots[os] = v;
        w = tw;
    }
}

}  // namespace rnng
