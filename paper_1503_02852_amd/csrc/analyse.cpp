// Graph validation and the intra-stream schedule analyser (paper Section 3.1).
//
// Strongly connected components are found with Tarjan's algorithm (the paper names it and
// notes that it yields the components in reverse topological order of the condensation).
// A component with more than one node, or with a self-loop, is a "recurrent node"; all other
// nodes form a DAG that is worked on for every frame of the window at once.  Inside a
// recurrent node one time step computes the delayed connections first and the remaining
// delay-0 part in topological order; that order is exported as per-node levels.
#include "graph.h"

#include <algorithm>
#include <sstream>

namespace rnng {

std::string validate_graph(const std::vector<GNode>& nodes, const std::vector<GEdge>& edges) {
    std::ostringstream e;
    const int K = (int)nodes.size();
    if (K == 0) return "graph has no nodes";
    std::vector<int> n_in(K, 0), n_out(K, 0);
    int n_outputs = 0;
    for (int k = 0; k < K; ++k) {
        const GNode& n = nodes[k];
        if (n.kind < NODE_INPUT || n.kind > NODE_MAX) { e << "node " << k << ": unknown kind " << n.kind; return e.str(); }
        if (n.act < ACT_LINEAR || n.act > ACT_RELU) { e << "node " << k << ": unknown activation " << n.act; return e.str(); }
        if (n.dim <= 0) { e << "node " << k << ": dim must be positive"; return e.str(); }
        if (n.kind == NODE_INPUT && (n.has_bias || n.is_output || n.act != ACT_LINEAR)) {
            e << "node " << k << ": an input node has no bias, no activation and is not an output"; return e.str();
        }
        if ((n.kind == NODE_MUL || n.kind == NODE_MAX) && n.has_bias) { e << "node " << k << ": a multiplicative or maximum node has no bias"; return e.str(); }
        if (n.is_output < OUT_NONE || n.is_output > OUT_SQUARED_ERROR) { e << "node " << k << ": unknown output kind " << n.is_output; return e.str(); }
        if (n.is_output == OUT_CROSS_ENTROPY) {
            ++n_outputs;
            if (n.kind != NODE_ADD || n.act != ACT_SOFTMAX) {
                e << "node " << k << ": a cross-entropy output node must be additive with softmax activation"; return e.str();
            }
        } else if (n.is_output == OUT_SQUARED_ERROR) {
            ++n_outputs;
            if (n.kind != NODE_ADD || n.act == ACT_SOFTMAX) {
                e << "node " << k << ": a squared-error output node must be additive with linear, sigmoid, tanh or rectifier activation"; return e.str();
            }
        } else if (n.act == ACT_SOFTMAX) {
            e << "node " << k << ": softmax is allowed on output nodes only"; return e.str();
        }
    }
    if (n_outputs == 0) return "graph has no output node";
    for (size_t m = 0; m < edges.size(); ++m) {
        const GEdge& ed = edges[m];
        if (ed.src < 0 || ed.src >= K || ed.dst < 0 || ed.dst >= K) { e << "edge " << m << ": node id out of range"; return e.str(); }
        if (ed.delay < 0) { e << "edge " << m << ": negative delay"; return e.str(); }
        if (ed.wkind < W_FULL || ed.wkind > W_IDENTITY) { e << "edge " << m << ": unknown weight kind " << ed.wkind; return e.str(); }
        if (ed.wkind != W_FULL && nodes[ed.src].dim != nodes[ed.dst].dim) {
            e << "edge " << m << ": identity / diagonal edge joins nodes of different width"; return e.str();
        }
        if (nodes[ed.dst].kind == NODE_INPUT) { e << "edge " << m << ": enters an input node"; return e.str(); }
        if (nodes[ed.src].is_output) { e << "edge " << m << ": leaves an output node"; return e.str(); }
        ++n_in[ed.dst]; ++n_out[ed.src];
    }
    for (int k = 0; k < K; ++k)
        if (nodes[k].kind != NODE_INPUT && n_in[k] == 0) { e << "node " << k << ": non-input node without incoming edge"; return e.str(); }
    return "";
}

namespace {

// Iterative Tarjan.  comp_of[v] = index in emission order (reverse topological).
int tarjan_scc(int K, const std::vector<std::vector<int>>& succ, std::vector<int>& comp_of) {
    std::vector<int> index(K, -1), low(K, 0), it(K, 0);
    std::vector<char> on_stack(K, 0);
    std::vector<int> stack, call;
    comp_of.assign(K, -1);
    int counter = 0, n_comps = 0;
    for (int root = 0; root < K; ++root) {
        if (index[root] >= 0) continue;
        call.push_back(root);
        index[root] = low[root] = counter++;
        stack.push_back(root); on_stack[root] = 1;
        while (!call.empty()) {
            int v = call.back();
            if (it[v] < (int)succ[v].size()) {
                int w = succ[v][it[v]++];
                if (index[w] < 0) {
                    index[w] = low[w] = counter++;
                    stack.push_back(w); on_stack[w] = 1;
                    call.push_back(w);
                } else if (on_stack[w]) {
                    low[v] = std::min(low[v], index[w]);
                }
            } else {
                call.pop_back();
                if (!call.empty()) low[call.back()] = std::min(low[call.back()], low[v]);
                if (low[v] == index[v]) {
                    for (;;) {
                        int w = stack.back(); stack.pop_back(); on_stack[w] = 0;
                        comp_of[w] = n_comps;
                        if (w == v) break;
                    }
                    ++n_comps;
                }
            }
        }
    }
    return n_comps;
}

}  // namespace

bool analyse_graph(const std::vector<GNode>& nodes, const std::vector<GEdge>& edges,
                   Schedule& out, std::string& err) {
    const int K = (int)nodes.size();
    const int M = (int)edges.size();
    std::vector<std::vector<int>> succ(K);
    for (const GEdge& e : edges) succ[e.src].push_back(e.dst);
    std::vector<int> raw;
    const int C = tarjan_scc(K, succ, raw);

    // Recurrent flag and condensation levels.  Tarjan emits a component only after every
    // component reachable from it, so walking the emission order backwards visits sources
    // before destinations.
    std::vector<int> size(C, 0), rec(C, 0), level(C, 0), min_id(C, K);
    for (int v = 0; v < K; ++v) { ++size[raw[v]]; min_id[raw[v]] = std::min(min_id[raw[v]], v); }
    for (int c = 0; c < C; ++c) rec[c] = size[c] > 1;
    for (const GEdge& e : edges) if (e.src == e.dst) rec[raw[e.src]] = 1;
    std::vector<std::vector<int>> comp_in(C);   // per component: source components of entering edges
    for (const GEdge& e : edges)
        if (raw[e.src] != raw[e.dst]) comp_in[raw[e.dst]].push_back(raw[e.src]);
    for (int c = C - 1; c >= 0; --c)
        for (int s : comp_in[c]) level[c] = std::max(level[c], level[s] + 1);

    // Canonical numbering by (level, smallest member id).
    std::vector<int> order(C);
    for (int c = 0; c < C; ++c) order[c] = c;
    std::sort(order.begin(), order.end(), [&](int a, int b) {
        return level[a] != level[b] ? level[a] < level[b] : min_id[a] < min_id[b];
    });
    std::vector<int> renum(C);
    for (int i = 0; i < C; ++i) renum[order[i]] = i;

    out.n_comps = C;
    out.node_comp.assign(K, 0);
    out.comp_level.assign(C, 0);
    out.comp_recurrent.assign(C, 0);
    out.comp_nodes.assign(C, {});
    for (int v = 0; v < K; ++v) { out.node_comp[v] = renum[raw[v]]; out.comp_nodes[renum[raw[v]]].push_back(v); }
    for (int c = 0; c < C; ++c) { out.comp_level[renum[c]] = level[c]; out.comp_recurrent[renum[c]] = rec[c]; }

    out.edge_class.assign(M, EDGE_BATCHED);
    for (int m = 0; m < M; ++m) {
        const GEdge& e = edges[m];
        if (out.node_comp[e.src] == out.node_comp[e.dst])
            out.edge_class[m] = e.delay >= 1 ? EDGE_STEP_DELAYED : EDGE_STEP_DELAY0;
    }

    // Levels inside a time step: longest path over delay-0 edges within a component (Kahn).
    // The same sweep over ALL delay-0 edges detects delay-0 cycles anywhere in the graph.
    std::vector<int> indeg(K, 0);
    std::vector<std::vector<int>> succ0(K);
    for (const GEdge& e : edges) if (e.delay == 0) { ++indeg[e.dst]; succ0[e.src].push_back(e.dst); }
    std::vector<int> ready;
    for (int v = 0; v < K; ++v) if (indeg[v] == 0) ready.push_back(v);
    size_t done = 0;
    std::vector<int> topo;
    while (done < ready.size()) {
        int v = ready[done++];
        topo.push_back(v);
        for (int w : succ0[v]) if (--indeg[w] == 0) ready.push_back(w);
    }
    if ((int)topo.size() != K) { err = "the delay-0 edges contain a cycle"; return false; }
    out.node_level.assign(K, 0);
    std::vector<std::vector<int>> in0(K);   // delay-0 in-edges from the same component
    for (int m = 0; m < M; ++m)
        if (out.edge_class[m] == EDGE_STEP_DELAY0) in0[edges[m].dst].push_back(edges[m].src);
    for (int v : topo)
        for (int s : in0[v]) out.node_level[v] = std::max(out.node_level[v], out.node_level[s] + 1);
    return true;
}

}  // namespace rnng
