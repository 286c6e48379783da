// Host planner: turns the analysed graph into GEMM problem lists, matrix-vector task lists
// and element-wise node programs, following the paper's intra-stream schedule (Section 3.1):
// per component in topological order, edges that enter the component from outside are worked
// on for all frames at once; inside a recurrent node every time step first takes the delayed
// connections and then the delay-0 part level by level.  The backward direction uses the
// reversed order (Section 3.1, last sentences) with the delta / epsilon equations of Section 2.2.
#include "plan.h"

#include <algorithm>
#include <map>

namespace rnng {

namespace {

constexpr int64_t PARAM_ALIGN = 64;   // floats; keeps every weight block 256-byte aligned

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct FactorH { int buf, frame_off, w_off, slot; };
struct TermH { std::vector<FactorH> f; };
struct OpH {
    int post = POST_NONE, dim = 0, out_buf = -1, pre_buf = -1, bias_off = -1, acc_buf = -1,
        deriv_buf = -1, out_slot = -1;
    std::vector<TermH> terms;
};
struct MvEdgeH { int w_off, k_len, transposed, src_buf, frame_off; };
struct MvTaskH { int n_out, acc_buf; std::vector<MvEdgeH> edges; };

int emit_program(std::vector<int32_t>& w, const std::vector<OpH>& ops, int& max_dim) {
    int off = (int)w.size();
    max_dim = 0;
    for (const OpH& o : ops) max_dim = std::max(max_dim, o.dim);
    w.push_back((int)ops.size());
    w.push_back(max_dim);
    for (const OpH& o : ops) {
        int32_t h[OP_HEADER_WORDS];
        h[OP_POST] = o.post; h[OP_DIM] = o.dim; h[OP_OUT_BUF] = o.out_buf; h[OP_PRE_BUF] = o.pre_buf;
        h[OP_BIAS_OFF] = o.bias_off; h[OP_ACC_BUF] = o.acc_buf; h[OP_DERIV_BUF] = o.deriv_buf;
        h[OP_OUT_SLOT] = o.out_slot; h[OP_NTERMS] = (int)o.terms.size();
        w.insert(w.end(), h, h + OP_HEADER_WORDS);
        for (const TermH& t : o.terms) {
            w.push_back((int)t.f.size());
            for (const FactorH& f : t.f) { w.push_back(f.buf); w.push_back(f.frame_off); w.push_back(f.w_off); w.push_back(f.slot); }
        }
    }
    return off;
}

int emit_matvecs(std::vector<int32_t>& w, const std::vector<MvTaskH>& tasks, int& max_out) {
    int off = (int)w.size();
    max_out = 0;
    w.push_back((int)tasks.size());
    for (const MvTaskH& t : tasks) {
        max_out = std::max(max_out, t.n_out);
        w.push_back(t.n_out); w.push_back(t.acc_buf); w.push_back((int)t.edges.size());
        for (const MvEdgeH& e : t.edges) {
            w.push_back(e.w_off); w.push_back(e.k_len); w.push_back(e.transposed); w.push_back(e.src_buf); w.push_back(e.frame_off);
        }
    }
    return off;
}

}  // namespace

bool build_plan(const std::vector<GNode>& nodes, const std::vector<GEdge>& edges, Plan& P, std::string& err) {
    err = validate_graph(nodes, edges);
    if (!err.empty()) return false;
    P.nodes = nodes; P.edges = edges;
    if (!analyse_graph(nodes, edges, P.sched, err)) return false;
    const int K0 = (int)nodes.size(), M0 = (int)edges.size();
    for (int k = 0; k < K0; ++k) {
        if (nodes[k].kind == NODE_INPUT) P.input_nodes.push_back(k);
        if (nodes[k].is_output) P.output_nodes.push_back(k);
    }

    // ---- parameter layout: edges in index order, then biases in node order ----
    P.edge_off.assign(M0, 0); P.edge_len.assign(M0, 0); P.bias_off.assign(K0, 0); P.bias_len.assign(K0, 0);
    int64_t cur = 0;
    for (int m = 0; m < M0; ++m) {
        const GEdge& e = edges[m];
        int64_t len = e.wkind == W_FULL ? (int64_t)nodes[e.dst].dim * nodes[e.src].dim : e.wkind == W_DIAG ? nodes[e.dst].dim : 0;
        P.edge_off[m] = cur; P.edge_len[m] = len;
        cur = align_up(cur + len, PARAM_ALIGN);
    }
    for (int k = 0; k < K0; ++k) {
        int64_t len = nodes[k].has_bias ? nodes[k].dim : 0;
        P.bias_off[k] = cur; P.bias_len[k] = len;
        cur = align_up(cur + len, PARAM_ALIGN);
    }
    P.n_params = cur;
    if (cur >= (int64_t(1) << 31)) { err = "parameter count exceeds 2^31 - 1"; return false; }

    // ---- execution graph: route full edges into multiplicative nodes through a linear node ----
    P.xnodes = nodes;
    for (int m = 0; m < M0; ++m) {
        const GEdge& e = edges[m];
        if (e.wkind == W_FULL && nodes[e.dst].kind == NODE_MUL) {
            int s = (int)P.xnodes.size();
            P.xnodes.push_back(GNode{NODE_ADD, ACT_LINEAR, nodes[e.dst].dim, 0, 0});
            P.xedges.push_back(GEdge{e.src, s, e.delay, W_FULL}); P.xedge_param.push_back(m);
            P.xedges.push_back(GEdge{s, e.dst, 0, W_IDENTITY}); P.xedge_param.push_back(-1);
        } else {
            P.xedges.push_back(e); P.xedge_param.push_back(m);
        }
    }
    if (!analyse_graph(P.xnodes, P.xedges, P.xsched, err)) return false;
    const int K = (int)P.xnodes.size(), M = (int)P.xedges.size();
    const std::vector<GNode>& xn = P.xnodes;
    const std::vector<GEdge>& xe = P.xedges;
    const Schedule& S = P.xsched;
    P.n_bufs = 3 * K;
    P.buf_dim.assign(P.n_bufs, 0);
    for (int k = 0; k < K; ++k) P.buf_dim[P.ybuf(k)] = P.buf_dim[P.dbuf(k)] = P.buf_dim[P.abuf(k)] = xn[k].dim;

    std::vector<std::vector<int>> in_e(K), out_e(K);
    for (int m = 0; m < M; ++m) { in_e[xe[m].dst].push_back(m); out_e[xe[m].src].push_back(m); }
    auto w_off_of = [&](int m) -> int { return xe[m].wkind == W_DIAG ? (int)P.edge_off[P.xedge_param[m]] : -1; };
    auto full_off = [&](int m) -> int64_t { return P.edge_off[P.xedge_param[m]]; };

    P.comps.assign(S.n_comps, CompPlan());
    for (int c = 0; c < S.n_comps; ++c) {
        CompPlan& cp = P.comps[c];
        cp.recurrent = S.comp_recurrent[c] != 0;
        std::vector<int> members;
        for (int k : S.comp_nodes[c]) if (xn[k].kind != NODE_INPUT) members.push_back(k);
        if (members.empty()) continue;
        std::sort(members.begin(), members.end(), [&](int a, int b) {
            return S.node_level[a] != S.node_level[b] ? S.node_level[a] < S.node_level[b] : a < b;
        });

        // phases: a delay-0 full edge inside the component separates its source and destination
        std::map<int, int> phase;
        int n_phases = 1;
        for (int k : members) {
            int p = 0;
            for (int m : in_e[k])
                if (S.edge_class[m] == EDGE_STEP_DELAY0) p = std::max(p, phase[xe[m].src] + (xe[m].wkind == W_FULL ? 1 : 0));
            phase[k] = p; n_phases = std::max(n_phases, p + 1);
        }

        // ---- forward ----
        for (int k : members) {
            GemmProblemPlan gp; gp.c_buf = P.ybuf(k); gp.n = xn[k].dim;
            for (int m : in_e[k])
                if (xe[m].wkind == W_FULL && S.edge_class[m] == EDGE_BATCHED)
                    gp.pairs.push_back(GemmPairPlan{P.ybuf(xe[m].src), -1, full_off(m), xn[xe[m].src].dim, xe[m].delay});
            if (!gp.pairs.empty()) cp.fwd_gemms.push_back(gp);
            if (xn[k].act == ACT_SOFTMAX) cp.softmax_node = k;
        }
        for (int p = 0; p < n_phases; ++p) {
            std::vector<int> np;
            for (int k : members) if (phase[k] == p) np.push_back(k);
            if ((int)np.size() > MAX_SLOTS) { err = "a recurrent node has too many layers in one step phase"; return false; }
            std::map<int, int> slot;
            for (size_t i = 0; i < np.size(); ++i) slot[np[i]] = (int)i;
            std::vector<MvTaskH> tasks; std::vector<OpH> ops;
            for (int k : np) {
                OpH o; o.dim = xn[k].dim; o.out_buf = P.ybuf(k); o.out_slot = slot[k];
                o.post = xn[k].act == ACT_SIGMOID ? POST_SIGMOID : xn[k].act == ACT_TANH ? POST_TANH : POST_NONE;
                if (xn[k].has_bias) o.bias_off = (int)P.bias_off[k];
                MvTaskH task; task.n_out = xn[k].dim; task.acc_buf = P.abuf(k);
                TermH product;
                for (int m : in_e[k]) {
                    const GEdge& e = xe[m];
                    if (e.wkind == W_FULL) {
                        if (S.edge_class[m] == EDGE_BATCHED) o.pre_buf = P.ybuf(k);
                        else task.edges.push_back(MvEdgeH{(int)full_off(m), xn[e.src].dim, 0, P.ybuf(e.src), -e.delay});
                        continue;
                    }
                    FactorH f{P.ybuf(e.src), -e.delay, w_off_of(m), -1};
                    if (e.delay == 0 && slot.count(e.src) && slot[e.src] < slot[k]) f.slot = slot[e.src];
                    if (xn[k].kind == NODE_MUL) product.f.push_back(f);
                    else { TermH t; t.f.push_back(f); o.terms.push_back(t); }
                }
                if (xn[k].kind == NODE_MUL) o.terms.push_back(product);
                if (!task.edges.empty()) { o.acc_buf = task.acc_buf; tasks.push_back(task); }
                ops.push_back(o);
            }
            PhasePlan ph;
            if (!tasks.empty()) { ph.mv_off = emit_matvecs(P.words, tasks, ph.mv_max_out); ph.n_mv_tasks = (int)tasks.size(); }
            ph.prog_off = emit_program(P.words, ops, ph.max_dim);
            cp.fwd_phases.push_back(ph);
        }
        cp.has_fwd_program = true;

        // ---- backward ----
        if (cp.softmax_node >= 0) continue;   // output delta comes from the softmax / cross-entropy kernel
        for (int j : members) {
            GemmProblemPlan gp; gp.c_buf = P.dbuf(j); gp.n = xn[j].dim;
            for (int m : out_e[j])
                if (xe[m].wkind == W_FULL && S.edge_class[m] == EDGE_BATCHED)
                    gp.pairs.push_back(GemmPairPlan{P.dbuf(xe[m].dst), -1, full_off(m), xn[xe[m].dst].dim, xe[m].delay});
            if (!gp.pairs.empty()) cp.bwd_gemms.push_back(gp);
        }
        for (int p = n_phases - 1; p >= 0; --p) {
            std::vector<int> np;
            for (int k : members) if (phase[k] == p) np.push_back(k);
            std::reverse(np.begin(), np.end());
            std::map<int, int> slot;
            for (size_t i = 0; i < np.size(); ++i) slot[np[i]] = (int)i;
            std::vector<MvTaskH> tasks; std::vector<OpH> ops;
            for (int j : np) {
                OpH o; o.dim = xn[j].dim; o.out_buf = P.dbuf(j); o.out_slot = slot[j];
                if (xn[j].act == ACT_SIGMOID) { o.post = POST_DSIGMOID; o.deriv_buf = P.ybuf(j); }
                else if (xn[j].act == ACT_TANH) { o.post = POST_DTANH; o.deriv_buf = P.ybuf(j); }
                MvTaskH task; task.n_out = xn[j].dim; task.acc_buf = P.abuf(j);
                for (int m : out_e[j]) {
                    const GEdge& e = xe[m];
                    const int k = e.dst;
                    if (e.wkind == W_FULL) {
                        if (S.edge_class[m] == EDGE_BATCHED) o.pre_buf = P.dbuf(j);
                        else task.edges.push_back(MvEdgeH{(int)full_off(m), xn[k].dim, 1, P.dbuf(k), e.delay});
                        continue;
                    }
                    TermH t;
                    FactorH f{P.dbuf(k), e.delay, w_off_of(m), -1};
                    if (e.delay == 0 && slot.count(k) && slot[k] < slot[j]) f.slot = slot[k];
                    t.f.push_back(f);
                    if (xn[k].kind == NODE_MUL)
                        for (int m2 : in_e[k])
                            if (m2 != m) t.f.push_back(FactorH{P.ybuf(xe[m2].src), e.delay - xe[m2].delay, w_off_of(m2), -1});
                    o.terms.push_back(t);
                }
                if (!task.edges.empty()) { o.acc_buf = task.acc_buf; tasks.push_back(task); }
                ops.push_back(o);
            }
            PhasePlan ph;
            if (!tasks.empty()) { ph.mv_off = emit_matvecs(P.words, tasks, ph.mv_max_out); ph.n_mv_tasks = (int)tasks.size(); }
            ph.prog_off = emit_program(P.words, ops, ph.max_dim);
            cp.bwd_phases.push_back(ph);
        }
        cp.has_bwd_program = true;
    }

    // ---- weight gradients ----
    for (int m = 0; m < M; ++m)
        if (xe[m].wkind == W_FULL)
            P.grad_gemms.push_back(GradGemmPlan{full_off(m), xn[xe[m].dst].dim, xn[xe[m].src].dim,
                                                P.dbuf(xe[m].dst), P.ybuf(xe[m].src), xe[m].delay});
    P.colsum_off = (int)P.words.size();
    P.n_colsum = 0;
    auto emit_colsum = [&](int dim, int out_off, const std::vector<FactorH>& fs) {
        P.words.push_back(dim); P.words.push_back(out_off); P.words.push_back((int)fs.size());
        for (const FactorH& f : fs) { P.words.push_back(f.buf); P.words.push_back(f.frame_off); P.words.push_back(f.w_off); P.words.push_back(f.slot); }
        ++P.n_colsum; P.colsum_max_dim = std::max(P.colsum_max_dim, dim);
    };
    for (int m = 0; m < M; ++m) {
        if (xe[m].wkind != W_DIAG) continue;
        const GEdge& e = xe[m];
        std::vector<FactorH> fs;
        fs.push_back(FactorH{P.dbuf(e.dst), 0, -1, -1});
        fs.push_back(FactorH{P.ybuf(e.src), -e.delay, -1, -1});
        if (xn[e.dst].kind == NODE_MUL)
            for (int m2 : in_e[e.dst])
                if (m2 != m) fs.push_back(FactorH{P.ybuf(xe[m2].src), -xe[m2].delay, w_off_of(m2), -1});
        emit_colsum(xn[e.dst].dim, (int)full_off(m), fs);
    }
    for (int k = 0; k < K0; ++k)
        if (nodes[k].has_bias) emit_colsum(nodes[k].dim, (int)P.bias_off[k], {FactorH{P.dbuf(k), 0, -1, -1}});
    return true;
}

}  // namespace rnng
