// Execution plan built once per graph by the host planner.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "graph.h"
#include "program.h"

namespace rnng {

// One A*B product that contributes to a GEMM destination.
struct GemmPairPlan {
    int a_buf;          // buffer id of A ([frames][k] tensor)
    int b_buf;          // buffer id of B, or -1 if B is a weight block
    int64_t b_w_off;    // weight offset of B (if b_buf < 0)
    int k_len;          // contraction length (units); for weight-gradient GEMMs: unused (frames)
    int delay;          // frame shift between the destination rows and A's rows
};

// Forward: C = y_dst [frames][n] = sum_p y_src_p(t - d_p) W_p^T.
// Backward: C = dE/dy_src [frames][n] = sum_p ds_dst_p(t + d_p) W_p.
struct GemmProblemPlan {
    int c_buf;
    int n;              // columns of C
    std::vector<GemmPairPlan> pairs;
};

// Weight gradient of one full edge: G[n_dst][n_src] = sum_t ds_dst(t)^T y_src(t - d).
struct GradGemmPlan {
    int64_t w_off; int n_dst, n_src, dst_buf, src_buf, delay;
};

struct PhasePlan {
    int mv_off = -1;     // word offset of the matrix-vector task list (-1: none)
    int prog_off = -1;   // word offset of the node program
    int max_dim = 0;
    int mv_max_out = 0;  // largest n_out over the tasks
    int n_mv_tasks = 0;
};

struct CompPlan {
    bool recurrent = false;
    int softmax_node = -1;                  // exec node id if this component is a softmax output node
    int sqerr_node = -1;                    // exec node id if this component is a squared-error output node
    std::vector<GemmProblemPlan> fwd_gemms, bwd_gemms;
    std::vector<PhasePlan> fwd_phases, bwd_phases;   // bwd_phases already in execution order
    bool has_fwd_program = false, has_bwd_program = false;
    int fwd_desc_off = -1, bwd_desc_off = -1;  // step descriptors: [n_phases, (mv_off, prog_off)...]
    // buffers that workgroups of the persistent step kernel read from each other (sources of
    // full connections inside the recurrent node); they are pre-filled with a sentinel
    std::vector<int> fwd_shared_bufs, bwd_shared_bufs;
    int64_t step_weight_floats = 0;         // weights of all full connections inside the component
    int chain = -1;                         // index into Plan::chains if the component is a chain member
    bool helper = false;                    // a helper member of a chain launch (ChainPlan::fwd_split / bwd_split)
};

// Consecutive recurrent components first..last whose step loops can run side by side in one
// kernel launch: members[i] is component first + i lowered with the full connections between
// chain members taken into the step loop (read with the sentinel protocol like a component's own
// delayed connections) instead of into a GEMM over all frames.
//
// fwd_split / bwd_split (empty if not built) are second lowerings of the two launches, in which
// the products of the connections between members are not added to the contraction of the member
// they lead into (a step of that member is bound by its arithmetic, while compute units idle): a
// helper member per such member (helper = true: a step program without recurrence, one direction
// only) computes them from the other member's values as soon as those appear and stores the sums
// into a tensor of its own (Plan::fbuf forward, Plan::hbuf backward), which the member's program
// reads element by element (GA_KIND_POLLED).  Order forward: the first component, then helper and
// split lowering of each later one; backward: the last component, then helper and split lowering
// of each earlier one.
struct ChainPlan {
    int first = 0, last = 0;
    std::vector<CompPlan> members;
    std::vector<CompPlan> fwd_split, bwd_split;
};

// Exchange bundle: up to four equally wide tensors that one step program stores and other
// workgroups poll (an LSTM's four gate deltas in the backward loop).  The wave-autonomous step
// kernel writes them with ONE coherent store per lane into the interleaved tensor `ebuf`
// ([frame][stream][unit][B]) and polls that instead of the members: every additional coherent
// store per step costs about a quarter of a microsecond of exchange time.  Other kernels ignore
// bundles and use the member tensors.
struct BundlePlan {
    int ebuf = -1, B = 0, dim = 0;
    int members[4] = {-1, -1, -1, -1};      // buffer ids; -1: padding lane (stored as zero)
};

struct Plan {
    // original graph and its canonical schedule (what rnn_graph_schedule exports)
    std::vector<GNode> nodes; std::vector<GEdge> edges; Schedule sched;
    // execution graph: full edges into multiplicative nodes are routed through a synthetic
    // linear additive node, so that every full edge ends in an additive node
    std::vector<GNode> xnodes; std::vector<GEdge> xedges; std::vector<int> xedge_param; Schedule xsched;
    // parameter layout (original indexing)
    std::vector<int64_t> edge_off, edge_len, bias_off, bias_len; int64_t n_params = 0;
    // buffers: y of exec node k -> k; ds of k -> K + k; matrix-vector accumulator of k -> 2K + k;
    // batched pre-activation of k kept apart from y_k -> 3K + k, likewise for ds_k -> 4K + k
    // (used when y_k / ds_k is read by other workgroups during the step loop); the sums that a
    // chain's helper member hands to the backward program of k -> 5K + k, to the forward program -> 6K + k
    int n_bufs = 0;
    std::vector<int> buf_dim;
    std::vector<char> buf_alloc;            // 0 not in the workspace, 1 [T][N][dim], 2 [N][dim], 3 a tile-blocked twin (below)
    // Tile-blocked twins.  A many-stream step kernel polls an exchanged tensor in tiles of 16
    // streams x 16 units, and a wavefront's load is served at full rate only if its 1 KiB lies at
    // consecutive addresses (measured: 77 GB/s per workgroup against 35 GB/s for 16 rows of 64
    // bytes).  Every tensor b that workgroups of a single-phase recurrent component exchange, and
    // whose width is a multiple of 16, therefore has a twin with the id twin_base + b:
    // [frame][stream / 16][unit / 16][(unit % 16) / 4][stream % 16][unit % 4], allocated for
    // windows whose stream count is a multiple of 16.  The producing kernel stores each value
    // twice (row-major for everyone else, blocked for the pollers).
    int twin_base = -1;
    std::vector<CompPlan> comps;
    std::vector<ChainPlan> chains;
    std::vector<BundlePlan> bundles;
    std::vector<int> bundle_of;             // per buffer id: index into bundles or -1
    std::vector<GradGemmPlan> grad_gemms;
    int colsum_off = -1, n_colsum = 0, colsum_max_dim = 0;
    std::vector<int32_t> words;             // all programs
    std::vector<int> input_nodes, output_nodes;   // original ids, increasing
    // History: every tensor of the window is stored with `hist` frames in front of the window's
    // first frame (hist = the longest delay of any connection).  They hold the activations that the
    // frames before the window left (zero for a fresh window), so that delayed connections, the
    // epsilon of multiplicative layers and the weight-gradient sums of the window's first frames
    // read the real y(t - d) (Section 2.2, last two equations; Section 3.2, BPTT(h; h')).
    int hist = 0;
    // Input nodes are read in place from the caller's tensors, which have no history frames.  An
    // input with a delayed or an element-wise (identity / diagonal) out-connection is copied into a
    // workspace tensor of its own (with history) instead; the others are read by GEMMs only, which
    // take the caller's rows directly.
    std::vector<char> input_staged;               // per exec node id
    std::vector<char> input_delayed;              // per exec node id: an input node with a delayed out-connection

    int ybuf(int k) const { return k; }
    int dbuf(int k) const { return (int)xnodes.size() + k; }
    int abuf(int k) const { return 2 * (int)xnodes.size() + k; }
    int pbuf(int k) const { return 3 * (int)xnodes.size() + k; }
    int qbuf(int k) const { return 4 * (int)xnodes.size() + k; }
    int hbuf(int k) const { return 5 * (int)xnodes.size() + k; }
    int fbuf(int k) const { return 6 * (int)xnodes.size() + k; }
};

// Returns false and a reason on an invalid graph.
bool build_plan(const std::vector<GNode>& nodes, const std::vector<GEdge>& edges, Plan& plan, std::string& err);

}  // namespace rnng
