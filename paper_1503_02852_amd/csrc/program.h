// Encoding of the element-wise node programs and matrix-vector task lists that the host
// planner emits and the HIP kernels interpret.  Plain int32 words in device memory.
//
// A "buffer" is a [T][N][dim] float tensor (node activations y_k, node state gradients
// dE/ds_k) or a one-frame [N][dim] scratch tensor (matrix-vector accumulators); kernels get
// a table of base pointers and widths indexed by buffer id.
//
// NodeOp (one per node and direction), evaluated for every (frame t, stream n, unit i < dim):
//     v = [pre_buf(t,n,i)] + [weights[bias_off + i]] + [acc_buf(n,i)] + sum over terms
//     term   = product over its factors
//     factor = value(buf, t + frame_off, n, i) * [weights[w_off + i]]
//              value is taken from register slot `slot` if slot >= 0 (a result of an earlier
//              NodeOp of the same program invocation), is 0 if the frame lies outside the window
//     out    = post(v):  forward: v, sigmoid(v), tanh(v)
//                        backward: v * y(1-y) or v * (1-y^2) with y = deriv_buf(t,n,i)
//     out is stored to out_buf(t,n,i) and kept in register slot out_slot.
// This covers the additive layer (sum of weighted activations), the multiplicative layer (one
// term with one factor per incoming connection), and in the backward direction the delta of a
// node as the sum over its outgoing connections of W^T eps, where eps for a multiplicative
// destination carries the product of the destination's other incoming connection outputs
// (paper Section 2.1 forward equations and Section 2.2 delta / epsilon equations).
#pragma once
#include <cstdint>

namespace rnng {

enum { POST_NONE = 0, POST_SIGMOID = 1, POST_TANH = 2, POST_DSIGMOID = 3, POST_DTANH = 4 };

enum {
    OP_POST = 0, OP_DIM, OP_OUT_BUF, OP_PRE_BUF, OP_BIAS_OFF, OP_ACC_BUF, OP_DERIV_BUF,
    OP_OUT_SLOT, OP_NTERMS, OP_HEADER_WORDS
};
enum { FACTOR_BUF = 0, FACTOR_FRAME_OFF, FACTOR_W_OFF, FACTOR_SLOT, FACTOR_WORDS };

// Node program: [n_ops, max_dim, ops...]; op = header, then per term [n_factors, factors...].
enum { PROG_NOPS = 0, PROG_MAXDIM, PROG_HEADER_WORDS };

// Matrix-vector task list: [n_tasks, tasks...]; task = [n_out, acc_buf, n_edges, edges...];
// edge = [w_off, k_len, transposed, src_buf, frame_off].
//   not transposed: acc[n][u] += sum_k W[u][k] * src(t + frame_off, n, k)       W is [n_out][k_len]
//   transposed:     acc[n][u] += sum_k W[k][u] * src(t + frame_off, n, k)       W is [k_len][n_out]
enum { MV_NOUT = 0, MV_ACC_BUF, MV_NEDGES, MV_HEADER_WORDS };
enum { MVE_W_OFF = 0, MVE_KLEN, MVE_TRANSPOSED, MVE_SRC_BUF, MVE_FRAME_OFF, MVE_WORDS };

// Column-sum task (gradients of diagonal weights and biases):
//   grads[out_off + i] = sum over t, n of the product of the factors.   [dim, out_off, n_factors, factors...]
enum { CS_DIM = 0, CS_OUT_OFF, CS_NFACTORS, CS_HEADER_WORDS };

constexpr int MAX_SLOTS = 32;

// Device view of the plan tables.
struct PlanView {
    float* const* buf_ptr;    // [n_bufs] base pointers
    const int32_t* buf_dim;   // [n_bufs] widths
    const int32_t* words;     // program words
};

}  // namespace rnng
