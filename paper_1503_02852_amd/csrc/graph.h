// Host-side graph description and the intra-stream schedule analyser (integers only).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace rnng {

struct GNode { int kind, act, dim, has_bias, is_output; };
struct GEdge { int src, dst, delay, wkind; };

enum { NODE_INPUT = 0, NODE_ADD = 1, NODE_MUL = 2, NODE_MAX = 3 };
enum { ACT_LINEAR = 0, ACT_SIGMOID = 1, ACT_TANH = 2, ACT_SOFTMAX = 3, ACT_RELU = 4 };
enum { OUT_NONE = 0, OUT_CROSS_ENTROPY = 1, OUT_SQUARED_ERROR = 2 };      // GNode::is_output
enum { W_FULL = 0, W_DIAG = 1, W_IDENTITY = 2 };
enum { EDGE_BATCHED = 0, EDGE_STEP_DELAYED = 1, EDGE_STEP_DELAY0 = 2 };

// Canonical schedule (paper Section 3.1): strongly connected components, which of them are
// recurrent nodes, longest-path levels of the condensation, levels inside a time step, and
// the class of every edge.
struct Schedule {
    int n_comps = 0;
    std::vector<int> node_comp;        // per node: component index (canonical numbering)
    std::vector<int> node_level;       // per node: level inside one time step
    std::vector<int> comp_level;       // per component
    std::vector<int> comp_recurrent;   // per component
    std::vector<int> edge_class;       // per edge
    std::vector<std::vector<int>> comp_nodes;  // per component: member nodes, increasing id
};

// Returns an empty string if the node / edge list is a valid network, else the reason.
std::string validate_graph(const std::vector<GNode>& nodes, const std::vector<GEdge>& edges);

// Tarjan's SCC algorithm (iterative) + canonical levelling.  Returns false (and a reason)
// if the delay-0 edges contain a cycle.
bool analyse_graph(const std::vector<GNode>& nodes, const std::vector<GEdge>& edges,
                   Schedule& out, std::string& err);

}  // namespace rnng
