// Encoding of the element-wise node programs and matrix-vector task lists that the host
// planner emits and the HIP kernels interpret.  Plain int32 words in device memory.
//
// A "buffer" is a [T][N][dim] float tensor (node activations y_k, node state gradients
// dE/ds_k, batched pre-activations) or a one-frame [N][dim] tensor (matrix-vector
// accumulators); kernels get a table of base pointers and widths indexed by buffer id.
//
// A node program evaluates, for one (frame t, stream n, unit i), all layers of one phase of a
// component in one direction.  It is straight-line code over a small register file of slots:
//   gather   slot g      <- buffer(t + frame_off, n, i), 0 outside the window   (loads, hoistable)
//   inv      next slots  <- weights[w_off + i]  (diagonal weights, biases; do not depend on t)
//   ops      slot dst    <- op(slot a, slot b, slot c)
//   stores   buffer(t, n, i) <- slot
// which covers the additive layer (sum of weighted activations, Section 2.1), the
// multiplicative layer (product of the incoming connection outputs), the activation functions,
// and in the backward direction delta_k = (sum over outgoing connections of W^T eps) * f'(s_k)
// with eps of a multiplicative destination carrying the product of that destination's other
// incoming connection outputs (Section 2.2).
#pragma once
#if !defined(__HIPCC_RTC__)
#include <cstdint>
#else
typedef signed int int32_t;   // the run-time compiler has no <cstdint>
#endif

namespace rnng {

enum {
    MOP_MOV = 0,    // d = a
    MOP_ADD = 1,    // d = a + b
    MOP_MUL = 2,    // d = a * b
    MOP_FMA = 3,    // d = a * b + c
    MOP_SIG = 4,    // d = 1 / (1 + exp(-a))
    MOP_TANH = 5,   // d = tanh(a)
    MOP_DSIG = 6,   // d = a * b * (1 - b)
    MOP_DTANH = 7,  // d = a * (1 - b * b)
    MOP_ZERO = 8,   // d = 0
    MOP_RELU = 9,   // d = max(a, 0)
    MOP_DRELU = 10, // d = b > 0 ? a : 0
    MOP_MAX = 11,   // d = max(a, b)
    MOP_GE = 12,    // d = a >= b ? 1 : 0
    MOP_GT = 13     // d = a > b ? 1 : 0
};

// Program header, then gather entries, inv entries, ops, stores.
enum { PG_NGATHER = 0, PG_NINV, PG_NOPS, PG_NSTORES, PG_MAXDIM, PG_NSLOTS, PG_HEADER_WORDS = 8 };
enum { GA_BUF = 0, GA_FRAME_OFF, GA_DIM, GA_KIND, GA_AUX, GA_WORDS };
// Gather kinds.  FRAMES, STATIC and CARRY all mean "buffer(t + frame_off, n, i)"; the distinction
// only tells a step kernel how it may obtain the value:
//   FRAMES  written by the same component during the step loop: load it coherently, this step
//   ACC     matrix-vector accumulator (frame_off = index of the task in its phase)
//   STATIC  not written during this component's step loop before it is read (outputs of earlier
//           components, forward activations in the backward pass, batched pre-activations): may
//           be loaded early and cached
//   CARRY   the value this same program computed in the previous step (aux = its result slot):
//           may be kept in a register instead of being re-loaded
//   POLLED  written by another component of the same launch, element by element for this frame
//           (a sum that a helper member of a chain computes ahead of time): load it coherently
//           and repeat while it shows the sentinel
enum { GA_KIND_FRAMES = 0, GA_KIND_ACC = 1, GA_KIND_STATIC = 2, GA_KIND_CARRY = 3, GA_KIND_POLLED = 4 };
enum { IV_W_OFF = 0, IV_DIM, IV_WORDS };
enum { MO_PACKED = 0, MO_C, MO_WORDS };                         // packed = opcode | dst << 8 | a << 16 | b << 24
enum { ST_BUF = 0, ST_SLOT, ST_DIM, ST_FLAGS, ST_WORDS };         // flags bit 0: other workgroups poll this buffer

constexpr int MAX_SLOTS = 32;     // a 32-float slot file stays in vector registers (indexed with uniform indices)

inline int program_words(const int32_t* p) {
    return PG_HEADER_WORDS + p[PG_NGATHER] * GA_WORDS + p[PG_NINV] * IV_WORDS + p[PG_NOPS] * MO_WORDS +
           p[PG_NSTORES] * ST_WORDS;
}

// Matrix-vector task list: [n_tasks, tasks...]; task = [n_out, acc_buf, n_edges, edges...];
// edge = [w_off, k_len, transposed, src_buf, frame_off].
//   not transposed: acc[n][u] += sum_k W[u][k] * src(t + frame_off, n, k)       W is [n_out][k_len]
//   transposed:     acc[n][u] += sum_k W[k][u] * src(t + frame_off, n, k)       W is [k_len][n_out]
enum { MV_NOUT = 0, MV_ACC_BUF, MV_NEDGES, MV_HEADER_WORDS };
enum { MVE_W_OFF = 0, MVE_KLEN, MVE_TRANSPOSED, MVE_SRC_BUF, MVE_FRAME_OFF, MVE_WORDS };

// Column-sum task (gradients of diagonal weights and biases):
//   grads[out_off + i] = sum over t, n of the product of the factors;
//   factor = buffer(t + frame_off, n, i) * [weights[w_off + i]].
//   [dim, out_off, n_factors, factors...], factor = [buf, frame_off, w_off]
enum { CS_DIM = 0, CS_OUT_OFF, CS_NFACTORS, CS_HEADER_WORDS };
enum { CF_BUF = 0, CF_FRAME_OFF, CF_W_OFF, CF_CMP, CF_WORDS };     // CF_CMP 1 / 2: this factor and the next one stand for [this >= next] / [this > next]

// Plan words and the buffer table never change while a kernel runs: device code reads them
// through the constant address space, which makes uniform reads scalar loads.
#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC_RTC__)
#define RNNG_CONST_AS __attribute__((address_space(4)))
#else
#define RNNG_CONST_AS
#endif
typedef const RNNG_CONST_AS int32_t* cwords_t;
typedef float* const RNNG_CONST_AS* cbufs_t;

// Device view of the plan tables.
struct PlanView {
    float* const* buf_ptr;    // [n_bufs] base pointers
    const int32_t* buf_dim;   // [n_bufs] widths
    const int32_t* words;     // program words
};

}  // namespace rnng
