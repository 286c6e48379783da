/*
 * rnngraph -- forward pass and backpropagation through time for generalized LSTM-like RNN
 * graphs (Hwang & Sung, "Single Stream Parallelization of Generalized LSTM-Like RNNs on a
 * GPU") on one AMD MI355X (gfx950).
 *
 * A network is a directed graph (paper Section 2.1): a node is a layer, an edge is a
 * connection m with a weight W_m and a delay d_m >= 0 that carries the source layer's
 * activation of frame t - d_m to the destination layer at frame t.  The library analyses the
 * graph (Section 3.1: strongly connected components become sequentially stepped "recurrent
 * nodes", everything else is worked on for all frames of the window at once) and runs the
 * forward pass and BPTT (Section 2.2) for N weight-sharing streams (Section 3.2).
 *
 * Conventions
 *  - Every function returns 0 on success or a negative rnn_status; rnn_last_error() gives a
 *    thread-local message.  Nothing throws across this boundary.
 *  - "d_" pointers are DEVICE pointers owned by the caller (weights, inputs, targets,
 *    workspace, gradients).  All other pointers are HOST pointers.  The library owns only
 *    host-side plan memory inside rnn_graph.
 *  - Calls that take a stream are asynchronous on that HIP stream (hipStream_t passed as
 *    void*; NULL = the default stream).
 *  - Frames x streams x units tensors are time-major row-major: element (t, n, i) of a node of
 *    width dim lives at ((t * N + n) * dim + i), t in [0, T), n in [0, N).
 *  - A fresh window (rnn_forward) starts from zero activations; a window moved ahead with
 *    rnn_shift_window starts from the activations the earlier frames left (Section 3.2).  Error
 *    terms from frames after the window are zero, and errors are back-propagated through the
 *    window's own frames only (Section 2.2: "while t > t0'").
 *  - All arithmetic is fp32.  Gradients are dE_total/dW, summed (not averaged) over frames
 *    and streams, E_total = sum over frames, streams and output nodes of E(t) (-ln y_target
 *    or 1/2 |d - y|^2, by the output node's criterion).
 */
#ifndef RNNGRAPH_H
#define RNNGRAPH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rnn_graph rnn_graph; /* opaque */

enum rnn_status {
    RNN_OK = 0,
    RNN_ERR_INVALID_ARGUMENT = -1, /* NULL pointer, bad size, bad index */
    RNN_ERR_INVALID_GRAPH = -2,    /* the node / edge list violates a rule listed at rnn_graph_create */
    RNN_ERR_WORKSPACE = -3,        /* workspace NULL, misaligned or too small */
    RNN_ERR_SEQUENCE = -4,         /* rnn_bptt before rnn_forward, rnn_grads before rnn_bptt */
    RNN_ERR_DEVICE = -5,           /* a HIP call failed, a specialised kernel could not be built, loaded or launched, or a
                                      kernel reported a wait that ran into its limit or a workgroup placement other than
                                      the one observed for the device */
    RNN_ERR_NO_MEMORY = -6
};

/* Node (layer) kinds: Section 2.1 defines additive layers (sum of the incoming connection
 * outputs, then an activation function) and multiplicative layers (element-wise product), and
 * allows other aggregation functions; RNN_NODE_MAX takes the element-wise maximum of the incoming
 * connection outputs (its error terms go to the connection that holds the maximum, to the one
 * with the lowest edge index if several do). */
enum { RNN_NODE_INPUT = 0, RNN_NODE_ADD = 1, RNN_NODE_MUL = 2, RNN_NODE_MAX = 3 };
/* Activation functions f_k (Section 2.1 leaves them open); softmax is allowed on output nodes
 * only and is paired with the cross-entropy criterion, the case for which Section 2.2 writes the
 * output delta out.  RNN_ACT_RELU is the rectifier max(0, s); its derivative at s = 0 counts as 0. */
enum { RNN_ACT_LINEAR = 0, RNN_ACT_SIGMOID = 1, RNN_ACT_TANH = 2, RNN_ACT_SOFTMAX = 3, RNN_ACT_RELU = 4 };
/* Values of rnn_node_desc.is_output.  In Section 2.2 the initial delta of an output layer
 * depends on the error criterion E(t) and on the layer's activation function.
 * RNN_OUT_CROSS_ENTROPY: additive softmax layer, class-index targets,
 * E(t) = -ln y_target, delta = d - y;  RNN_OUT_SQUARED_ERROR (the MSE criterion that Section 4
 * names): additive layer with linear, sigmoid, tanh or rectifier activation, dense targets,
 * E(t) = 1/2 sum_j (d_j - y_j)^2, delta_j = (d_j - y_j) f'(s_j). */
enum { RNN_OUT_NONE = 0, RNN_OUT_CROSS_ENTROPY = 1, RNN_OUT_SQUARED_ERROR = 2 };
/* Weight kinds: full matrix [n_dst x n_src] (row-major, z = W y), diagonal (a vector, used for
 * peepholes) and identity (no parameters), cf. the Fig. 1 caption. */
enum { RNN_W_FULL = 0, RNN_W_DIAG = 1, RNN_W_IDENTITY = 2 };
/* Edge classes of the intra-stream schedule (Section 3.1). */
enum { RNN_EDGE_BATCHED = 0, RNN_EDGE_STEP_DELAYED = 1, RNN_EDGE_STEP_DELAY0 = 2 };

typedef struct { int32_t kind, act, dim, has_bias, is_output; } rnn_node_desc;
typedef struct { int32_t src, dst, delay, wkind; } rnn_edge_desc;

/* Builds the schedule for a graph given as a node list and an edge list (Section 2.1).
 * HOST arrays, copied.  *out receives a handle to be released with rnn_graph_destroy.
 * RNN_ERR_INVALID_GRAPH if: a node id is out of range; dim <= 0; an unknown kind / act / wkind;
 * an identity or diagonal edge joins nodes of different width; delay < 0; an edge enters an
 * input node; a non-input node has no incoming edge; an input node has a bias, an activation or
 * is an output; softmax on a node that is not a cross-entropy output, a cross-entropy output
 * that is not additive-softmax, a squared-error output that is not additive or has softmax;
 * an output node with outgoing edges; has_bias on a multiplicative or maximum node; there is no output
 * node; or the delay-0 edges contain a cycle (Section 3.1 needs the per-step remainder to be a
 * DAG). */
int rnn_graph_create(const rnn_node_desc* nodes, int32_t n_nodes,
                     const rnn_edge_desc* edges, int32_t n_edges, rnn_graph** out);
void rnn_graph_destroy(rnn_graph* g);

/* The intra-stream schedule of Section 3.1 in canonical form (HOST int32 arrays supplied by
 * the caller; the first four have n_nodes entries, edge_class has n_edges; any may be NULL):
 *   node_comp[v]      index of v's strongly connected component; components are numbered by
 *                     increasing (comp_level, smallest node id in the component)
 *   node_level[v]     level of v inside one time step of its recurrent node: 0 if v has no
 *                     delay-0 in-edge from its own component, else 1 + max over those sources;
 *                     0 for nodes outside recurrent components
 *   comp_level[v]     longest-path level of v's component in the condensation DAG
 *   comp_recurrent[v] 1 if v's component is a recurrent node (more than one node, or a self-loop)
 *   edge_class[m]     RNN_EDGE_BATCHED (source and destination in different components: worked
 *                     on for all frames at once), RNN_EDGE_STEP_DELAYED (same component,
 *                     delay >= 1: computed first in each step), RNN_EDGE_STEP_DELAY0 (same
 *                     component, delay 0: part of the per-step DAG)
 *   *n_comps          number of components */
int rnn_graph_schedule(const rnn_graph* g, int32_t* node_comp, int32_t* node_level,
                       int32_t* comp_level, int32_t* comp_recurrent, int32_t* edge_class,
                       int32_t* n_comps);

/* Flat parameter layout shared by the weight and the gradient buffer.  rnn_param_count is the
 * buffer length in floats (it includes alignment padding between blocks; padding entries are
 * never read and receive zero gradient).  A full edge occupies len = n_dst * n_src floats at
 * off, row-major [n_dst][n_src]; a diagonal edge len = dim; an identity edge len = 0; a bias
 * len = dim (0 if the node has none). */
int64_t rnn_param_count(const rnn_graph* g);
int rnn_edge_param_offset(const rnn_graph* g, int32_t edge, int64_t* off, int64_t* len);
int rnn_bias_param_offset(const rnn_graph* g, int32_t node, int64_t* off, int64_t* len);

/* Bytes of DEVICE workspace needed for a window of T frames and N streams: the plan tables, 1 KiB
 * of control words (E_total, error flags) and, per node, activations and error terms for every
 * frame of the window plus d_max history frames in front of it (d_max = the longest delay of any
 * connection), which hold what the frames before the window left.  Negative rnn_status on error. */
int64_t rnn_workspace_bytes(const rnn_graph* g, int32_t T, int32_t N);

/* Forward pass over one window (Section 2.1 equations on the Section 3.1 schedule).
 *   d_weights  DEVICE, rnn_param_count floats.
 *   d_inputs   HOST array with one DEVICE pointer per input node, in increasing node id, each
 *              a [T][N][dim] float tensor.  The tensors are read in place by rnn_forward,
 *              rnn_bptt and rnn_grads and must stay unchanged until rnn_grads has completed.
 *   d_workspace DEVICE, 256-byte aligned, at least rnn_workspace_bytes(g, T, N); it holds the
 *              window's state between rnn_forward, rnn_bptt and rnn_grads.
 * One graph handle serves one window at a time.  All work is queued on hip_stream; the first
 * forward call of a process on a device also runs a short probe kernel and waits for it (it
 * records on which XCD the workgroups of a launch land: recurrent layers whose workgroups share
 * an XCD then exchange their state through that XCD's L2; RNNG_XCD_LOCAL=0 in the environment
 * switches that off), later calls do not synchronise. */
int rnn_forward(rnn_graph* g, const float* d_weights, const float* const* d_inputs,
                int32_t T, int32_t N, void* d_workspace, int64_t ws_bytes, void* hip_stream);

/* Forward pass over frames [t_begin, t_end) of a window of T frames (Section 3.2, BPTT(h; h'):
 * the forward pass advances by h' new frames while the backward pass covers the last h frames).
 * Frames [0, t_begin) must already hold the results of earlier calls on the same workspace with
 * the same T and N (RNN_ERR_SEQUENCE otherwise): delayed connections read them as y(t - d), so a
 * window computed in pieces equals the window computed at once.  Arguments as in rnn_forward,
 * which is rnn_forward_range(.., 0, T, ..).  A call with t_begin = 0 starts a fresh window: zero
 * state in front of it, control words cleared.  rnn_bptt needs the whole window computed. */
int rnn_forward_range(rnn_graph* g, const float* d_weights, const float* const* d_inputs,
                      int32_t T, int32_t N, int32_t t_begin, int32_t t_end,
                      void* d_workspace, int64_t ws_bytes, void* hip_stream);

/* One-hot input layer (the 38,000-word input of Section 4): declares that input number `input`
 * (position in increasing node id among the input nodes) is given as class indices instead of a
 * dense tensor: d_indices is a DEVICE int32 [T][N] array, frame (t, n) of the node is the unit
 * vector of class d_indices[t][n] (-1: the zero vector).  It must stay valid and unchanged from
 * rnn_forward until rnn_grads has completed.  The full connections leaving the node become column
 * gathers (forward) and scatter-adds (weight gradients) instead of GEMMs over a one-hot matrix;
 * the node may only have full out-connections.  d_inputs[input] of rnn_forward is then ignored
 * (may be NULL) and rnn_output of the node yields NULL.  d_indices = NULL returns to dense input. */
int rnn_set_onehot_input(rnn_graph* g, int32_t input, const int32_t* d_indices);

/* Moves the window `frames` frames ahead in time (Section 3.2): every node's activations of
 * frame t + frames become those of frame t, for t < T - frames; the last `frames` frames are then
 * undefined until rnn_forward_range(.., T - frames, T, ..) has computed them from the caller's
 * equally shifted input tensors.  1 <= frames < T; needs a completely computed window.
 * The d_max frames in front of the new window start are kept as history (for an input node with a
 * delayed or element-wise out-connection the library keeps its own copy, so the caller may
 * overwrite its tensors right away): delayed connections read them in the forward pass, and in
 * the backward pass the connection outputs z_n(t) of multiplicative layers and the weight-gradient
 * terms eps_m(t) y_k(t - d_m)^T of the window's first frames use them, as the last two equations
 * of Section 2.2 say (only the back-propagation of delta and epsilon stops at the window start).
 * For a one-hot input given as class indices the library likewise keeps the indices of the history
 * frames. */
int rnn_shift_window(rnn_graph* g, int32_t frames, void* hip_stream);

/* DEVICE view of node's activations y [T][N][dim] inside the workspace of the last rnn_forward
 * (for an input node: the caller's own input tensor). */
int rnn_output(const rnn_graph* g, int32_t node, const float** d_y);

/* Backward pass (Section 2.2: output delta from the error criterion, delta and epsilon
 * back-propagated through the reversed schedule) for the window of the last rnn_forward.
 *   d_targets  HOST array with one DEVICE pointer per output node, in increasing node id.
 *              Cross-entropy output: an int32 [T][N] tensor of class indices; -1 means "no error
 *              at this frame"; an index not below the layer's width leaves its frame out and
 *              raises a flag that rnn_check and rnn_grads(loss) report as
 *              RNN_ERR_INVALID_ARGUMENT.  Squared-error output: a float [T][N][dim] tensor of
 *              target vectors; an element that is NaN carries no error.
 * d_weights must hold the same values as in rnn_forward. */
int rnn_bptt(rnn_graph* g, const float* d_weights, const void* const* d_targets, void* hip_stream);

/* DEVICE view of dE_total/ds_k [T][N][dim] (the paper's -delta_k) after rnn_bptt; not defined
 * for input nodes. */
int rnn_state_grad(const rnn_graph* g, int32_t node, const float** d_ds);

/* Weight gradients (last equation of Section 2.2, summed over the N streams as in Section 3.2).
 *   d_grads  DEVICE, rnn_param_count floats, overwritten with dE_total/dW in the parameter layout.
 *   loss     HOST double or NULL; if given the call synchronises the stream, stores E_total and
 *            reports the window's error flags like rnn_check. */
int rnn_grads(rnn_graph* g, float* d_grads, double* loss, void* hip_stream);

/* on != 0: every gradient element has one writer and a fixed order of additions, so rnn_grads
 * returns the same bits from run to run (the weight-gradient and column sums are then not split
 * over workgroups that add atomically: slower where a sum is long and its matrix small).  Off by
 * default.  E_total is a double sum of per-workgroup parts whose order is not fixed either way. */
int rnn_set_deterministic(rnn_graph* g, int32_t on);

/* Waits for hip_stream and reports what the kernels of the current window have flagged since its
 * rnn_forward (or rnn_forward_range(.., 0, ..)): RNN_ERR_DEVICE if a recurrent step kernel gave up
 * a bounded wait or found itself on another XCD than observed (the window's activations and
 * gradients are then invalid), RNN_ERR_INVALID_ARGUMENT for a target index out of range, else
 * RNN_OK.  The asynchronous calls cannot report these themselves: callers that never pass `loss`
 * to rnn_grads call this once per window, or every so many windows. */
int rnn_check(rnn_graph* g, void* hip_stream);

/* The recurrent-step kernel is specialised at run time for each recurrent node's element-wise
 * step program (compiled with hiprtc on first use, cached per process by program structure).
 * rnn_specialise compiles the kernels this graph needs for N streams ahead of the first window;
 * it needs no GPU.  Returns the number of kernels compiled or found in the cache (0 if N is
 * served by kernels that are not specialised), or RNN_ERR_DEVICE with the compiler log as
 * message.  Only where the run-time compiler cannot be loaded at all (no libhiprtc.so), or with
 * RNNG_JIT=0 in the environment, the interpreting build of the same kernel takes over; a
 * specialised kernel that fails to compile, load or launch is an error of the call that needs it,
 * never a silent change of build (rnn_step_build in rnngraph_aux.h tells which build ran). */
int rnn_specialise(rnn_graph* g, int32_t N);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): rnn_forward with the workspace in a device array that
 * is part of the library image (RNN_STATIC_WORKSPACE_BYTES per GPU, held from the time the library
 * is loaded until the process ends), and the output layers' activations copied to the caller.
 *   d_inputs   as in rnn_forward.
 *   d_outputs  HOST array with one DEVICE pointer per output node, in increasing node id, each a
 *              [T][N][dim] float tensor that receives the node's activations y.
 * The call allocates nothing on the device and loads no code: every kernel it needs must already
 * be loaded, which one earlier rnn_forward of the same graph handle and N on this device (on a
 * workspace of the caller's) has done; else RNN_ERR_SEQUENCE.  RNN_ERR_WORKSPACE if the window
 * needs more than RNN_STATIC_WORKSPACE_BYTES (rnn_workspace_bytes tells), RNN_ERR_SEQUENCE if
 * kernel-class timing is switched on (it creates events).  Afterwards the handle's window lives in
 * the static array: rnn_output, rnn_bptt, rnn_grads work on it as after rnn_forward.  All calls
 * on one GPU share that GPU's array, which keeps the last call's contents (the call clears what
 * must start at zero): calls that overlap on one GPU, from any handle or stream, race. */
#define RNN_STATIC_WORKSPACE_BYTES (32 * 1024 * 1024)
int rnn_forward_static(rnn_graph* g, const float* d_weights, const float* const* d_inputs, float* const* d_outputs,
                       int32_t T, int32_t N, void* hip_stream);

/* Message for the last error on this thread (never NULL). */
const char* rnn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RNNGRAPH_H */
