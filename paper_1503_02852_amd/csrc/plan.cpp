// Host planner: turns the analysed graph into GEMM problem lists, matrix-vector task lists
// and element-wise node programs, following the paper's intra-stream schedule (Section 3.1):
// per component in topological order, edges that enter the component from outside are worked
// on for all frames at once; inside a recurrent node every time step first takes the delayed
// connections and then the delay-0 part level by level.  The backward direction uses the
// reversed order (Section 3.1, last sentences) with the delta / epsilon equations of Section 2.2.
#include "plan.h"
#include "step_layout.h"

#include <algorithm>
#include <array>
#include <map>

namespace rnng {

namespace {

constexpr int64_t PARAM_ALIGN = 64;   // floats; keeps every weight block 256-byte aligned

int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// cmp 1 / 2: this factor and the next one of the term stand for [this >= next] / [this > next]
// (1 or 0), the routing of a maximum node's error terms
struct FactorH { int buf, frame_off, w_off, slot; int cmp = 0; };
struct TermH { std::vector<FactorH> f; };
enum { POST_NONE = 0, POST_SIGMOID = 1, POST_TANH = 2, POST_DSIGMOID = 3, POST_DTANH = 4, POST_RELU = 5, POST_DRELU = 6 };
struct OpH {
    int post = POST_NONE, dim = 0, out_buf = -1, pre_buf = -1, bias_off = -1, acc_buf = -1, acc_task = 0,
        deriv_buf = -1, out_slot = -1, polled_buf = -1;
    bool new_program = false;   // must not share a program with the operation before it
    bool pre_static = false;    // pre_buf was written before the step loop (batched GEMM), not by an earlier part
    bool partial_out = false;   // out_buf holds a partial sum, not the layer's value
    bool agg_max = false;       // the terms are aggregated by their maximum, not their sum (maximum node, forward)
    std::vector<TermH> terms;
};
struct MvEdgeH { int w_off, k_len, transposed, src_buf, frame_off; };
struct MvTaskH { int n_out, acc_buf; std::vector<MvEdgeH> edges; };

// Lowers a list of node operations (each a sum of products of factors, then an activation or
// a derivative factor) to the straight-line slot program described in program.h.
// What a program's loads may assume about its component's step loop.
struct EmitCtx {
    const std::vector<char>* written = nullptr;   // per buffer: written during this component's step loop
    const std::vector<char>* shared = nullptr;    // per buffer: read by other workgroups during the step loop
    int step_dir = 0;                             // -1 forward, +1 backward: frame offset of "the previous step"; 0: not stepped
};

struct Lowering {
    std::vector<std::array<int, 4>> gathers;   // buf, frame_off, dim, kind
    std::vector<std::array<int, 2>> invs;      // w_off, dim
    int gather_slot(int buf, int frame_off, int dim, int kind) {
        for (size_t i = 0; i < gathers.size(); ++i)
            if (gathers[i][0] == buf && gathers[i][1] == frame_off && gathers[i][3] == kind) return (int)i;
        gathers.push_back({buf, frame_off, dim, kind});
        return (int)gathers.size() - 1;
    }
    int inv_index(int w_off, int dim) {
        for (size_t i = 0; i < invs.size(); ++i) if (invs[i][0] == w_off) return (int)i;
        invs.push_back({w_off, dim});
        return (int)invs.size() - 1;
    }
};

// Returns the word offset of the program, or -1 (with err set) if it needs too many slots.
int emit_program(std::vector<int32_t>& w, const std::vector<OpH>& all_ops, int first, int last,
                 const std::vector<int>& buf_dim, int& max_dim, bool dry_run, const EmitCtx* ctx = nullptr) {
    // results of operations outside [first, last) are read back from their buffers
    std::vector<OpH> ops(all_ops.begin() + first, all_ops.begin() + last);
    for (OpH& o : ops)
        for (TermH& t : o.terms)
            for (FactorH& f : t.f) f.slot = (f.slot >= first && f.slot < last) ? f.slot - first : -1;
    Lowering L;
    // pass 1: collect loads so that their slots are known before any op is emitted
    for (const OpH& o : ops) {
        if (o.pre_buf >= 0) L.gather_slot(o.pre_buf, 0, o.dim, GA_KIND_FRAMES);
        if (o.bias_off >= 0) L.inv_index(o.bias_off, o.dim);
        if (o.acc_buf >= 0) L.gather_slot(o.acc_buf, o.acc_task, o.dim, GA_KIND_ACC);
        if (o.polled_buf >= 0) L.gather_slot(o.polled_buf, 0, o.dim, GA_KIND_POLLED);
        for (const TermH& t : o.terms)
            for (const FactorH& f : t.f) {
                if (f.slot < 0) L.gather_slot(f.buf, f.frame_off, buf_dim[f.buf], GA_KIND_FRAMES);
                if (f.w_off >= 0 || f.w_off <= -1000) L.inv_index(f.w_off, buf_dim[f.buf]);
            }
        if (o.deriv_buf >= 0) L.gather_slot(o.deriv_buf, 0, o.dim, GA_KIND_FRAMES);
    }
    bool has_cmp = false;
    for (const OpH& o : ops) for (const TermH& t : o.terms) for (const FactorH& f : t.f) has_cmp = has_cmp || f.cmp != 0;
    const int ng = (int)L.gathers.size(), ni = (int)L.invs.size();
    // temporaries: the running product; with comparisons also their running product and two operands
    const int res0 = ng + ni, tmp = res0 + (int)ops.size(), tmp_mask = tmp + 1, tmp_a = tmp + 2, tmp_b = tmp + 3;
    const int n_slots = tmp + (has_cmp ? 4 : 1);
    if (n_slots > MAX_SLOTS || ng > STEP_MAX_GATHERS) return -1;
    if (dry_run) return 0;
    std::vector<std::array<int, 2>> mops;      // packed, c
    std::vector<std::array<int, 4>> stores;    // buf, slot, dim, flags
    auto mop = [&](int opc, int d, int a, int b, int c) { mops.push_back({opc | d << 8 | a << 16 | b << 24, c}); };
    max_dim = 0;
    for (size_t r = 0; r < ops.size(); ++r) {
        const OpH& o = ops[r];
        max_dim = std::max(max_dim, o.dim);
        const int R = res0 + (int)r;
        bool have = false;
        // adds (or, for a maximum node, merges) the product of the slots in `a` into R
        auto accumulate = [&](const std::vector<int>& a) {
            if (o.agg_max) {
                int v = a[0];
                if (a.size() > 1) {
                    for (size_t j = 1; j < a.size(); ++j) { mop(MOP_MUL, have ? tmp : R, v, a[j], 0); v = have ? tmp : R; }
                    if (have) mop(MOP_MAX, R, R, tmp, 0);
                } else if (!have) mop(MOP_MOV, R, v, 0, 0);
                else mop(MOP_MAX, R, R, v, 0);
            } else if (a.size() == 1) {
                if (!have) mop(MOP_MOV, R, a[0], 0, 0); else mop(MOP_ADD, R, R, a[0], 0);
            } else {
                int p = a[0];
                for (size_t j = 1; j + 1 < a.size(); ++j) { mop(MOP_MUL, tmp, p, a[j], 0); p = tmp; }
                if (!have) mop(MOP_MUL, R, p, a.back(), 0); else mop(MOP_FMA, R, p, a.back(), R);
            }
            have = true;
        };
        if (o.pre_buf >= 0) accumulate({L.gather_slot(o.pre_buf, 0, o.dim, GA_KIND_FRAMES)});
        if (o.bias_off >= 0) accumulate({ng + L.inv_index(o.bias_off, o.dim)});
        if (o.acc_buf >= 0) accumulate({L.gather_slot(o.acc_buf, o.acc_task, o.dim, GA_KIND_ACC)});
        if (o.polled_buf >= 0) accumulate({L.gather_slot(o.polled_buf, 0, o.dim, GA_KIND_POLLED)});
        for (const TermH& t : o.terms) {
            std::vector<int> atoms;
            // value of a factor: its slot, or (times its weight) in `scratch`
            auto value_of = [&](const FactorH& f, int scratch) {
                const int sl = f.slot >= 0 ? res0 + f.slot : L.gather_slot(f.buf, f.frame_off, buf_dim[f.buf], GA_KIND_FRAMES);
                if (!(f.w_off >= 0 || f.w_off <= -1000)) return sl;
                mop(MOP_MUL, scratch, sl, ng + L.inv_index(f.w_off, buf_dim[f.buf]), 0);
                return scratch;
            };
            bool mask = false;
            for (size_t i = 0; i < t.f.size(); ++i) {
                const FactorH& f = t.f[i];
                if (f.cmp != 0 && i + 1 < t.f.size()) {
                    const int va = value_of(f, tmp_a), vb = value_of(t.f[i + 1], tmp_b);
                    ++i;
                    if (!mask) mop(f.cmp == 1 ? MOP_GE : MOP_GT, tmp_mask, va, vb, 0);
                    else { mop(f.cmp == 1 ? MOP_GE : MOP_GT, tmp_a, va, vb, 0); mop(MOP_MUL, tmp_mask, tmp_mask, tmp_a, 0); }
                    mask = true;
                    continue;
                }
                atoms.push_back(f.slot >= 0 ? res0 + f.slot : L.gather_slot(f.buf, f.frame_off, buf_dim[f.buf], GA_KIND_FRAMES));
                if (f.w_off >= 0 || f.w_off <= -1000) atoms.push_back(ng + L.inv_index(f.w_off, buf_dim[f.buf]));
            }
            if (mask) atoms.push_back(tmp_mask);
            accumulate(atoms);
        }
        if (!have) mop(MOP_ZERO, R, 0, 0, 0);
        if (o.post == POST_SIGMOID) mop(MOP_SIG, R, R, 0, 0);
        else if (o.post == POST_TANH) mop(MOP_TANH, R, R, 0, 0);
        else if (o.post == POST_DSIGMOID) mop(MOP_DSIG, R, R, L.gather_slot(o.deriv_buf, 0, o.dim, GA_KIND_FRAMES), 0);
        else if (o.post == POST_DTANH) mop(MOP_DTANH, R, R, L.gather_slot(o.deriv_buf, 0, o.dim, GA_KIND_FRAMES), 0);
        else if (o.post == POST_RELU) mop(MOP_RELU, R, R, 0, 0);
        else if (o.post == POST_DRELU) mop(MOP_DRELU, R, R, L.gather_slot(o.deriv_buf, 0, o.dim, GA_KIND_FRAMES), 0);
        stores.push_back({o.out_buf, R, o.dim, 0});
    }
    const int off = (int)w.size();
    int32_t h[PG_HEADER_WORDS] = {0};
    h[PG_NGATHER] = ng; h[PG_NINV] = ni; h[PG_NOPS] = (int)mops.size(); h[PG_NSTORES] = (int)stores.size();
    h[PG_MAXDIM] = max_dim; h[PG_NSLOTS] = n_slots;
    w.insert(w.end(), h, h + PG_HEADER_WORDS);
    for (auto& g : L.gathers) {
        int kind = g[3], aux = 0;
        if (kind == GA_KIND_FRAMES && ctx && ctx->step_dir != 0) {
            const int buf = g[0], off = g[1];
            if (!(*ctx->written)[buf]) kind = GA_KIND_STATIC;
            else {
                for (size_t r = 0; r < ops.size(); ++r) {
                    if (off == 0 && ops[r].pre_buf == buf && ops[r].pre_static) { kind = GA_KIND_STATIC; break; }
                    if (off == ctx->step_dir && ops[r].out_buf == buf && !ops[r].partial_out) { kind = GA_KIND_CARRY; aux = res0 + (int)r; break; }
                }
            }
        }
        w.push_back(g[0]); w.push_back(g[1]); w.push_back(g[2]); w.push_back(kind); w.push_back(aux);
    }
    for (auto& v : L.invs) w.insert(w.end(), v.begin(), v.end());
    for (auto& m : mops) w.insert(w.end(), m.begin(), m.end());
    for (auto& st : stores) {
        if (ctx && ctx->shared && (*ctx->shared)[st[0]]) st[3] |= 1;
        w.insert(w.end(), st.begin(), st.end());
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

namespace {

bool op_fits(const OpH& o, const std::vector<int>& buf_dim, int slot_margin) {
    std::vector<OpH> one(1, o);
    for (TermH& t : one[0].terms) for (FactorH& f : t.f) f.slot = -1;
    // the margin is honoured by adding dummy invariant loads
    for (int i = 0; i < slot_margin; ++i) one[0].terms.push_back(TermH{{FactorH{o.out_buf, 0, -1000 - i, -1}}});
    std::vector<int32_t> sink; int md = 0;
    return emit_program(sink, one, 0, 1, buf_dim, md, true) == 0;
}

// A layer whose own sum has too many element-wise terms for one program is cut into parts that
// accumulate through a scratch tensor (part_buf): part 1 stores its partial sum, the next part
// starts from it, the last part applies the activation / derivative and stores the result.
bool split_wide_ops(std::vector<OpH>& ops, const std::vector<int>& part_bufs, const std::vector<int>& buf_dim,
                    std::vector<char>& buf_alloc, std::string& err) {
    std::vector<OpH> out;
    std::vector<int> new_index(ops.size(), 0);
    for (size_t r = 0; r < ops.size(); ++r) {
        const OpH& o = ops[r];
        if (op_fits(o, buf_dim, 0)) { new_index[r] = (int)out.size(); out.push_back(o); continue; }
        const int pb = part_bufs[r];
        buf_alloc[pb] = 1;
        OpH cur = o; cur.terms.clear(); cur.post = POST_NONE; cur.deriv_buf = -1; cur.out_buf = pb; cur.partial_out = true;
        for (const TermH& t : o.terms) {
            OpH trial = cur; trial.terms.push_back(t);
            if (op_fits(trial, buf_dim, 2)) { cur = trial; continue; }
            if (cur.terms.empty() && cur.pre_buf < 0 && cur.acc_buf < 0 && cur.bias_off < 0) {
                err = "a connection into a multiplicative layer has too many sibling connections for one step program";
                return false;
            }
            out.push_back(cur);
            cur = OpH(); cur.dim = o.dim; cur.pre_buf = pb; cur.out_buf = pb; cur.new_program = true; cur.partial_out = true; cur.agg_max = o.agg_max; cur.terms.push_back(t);
            if (!op_fits(cur, buf_dim, 2)) {
                err = "a connection into a multiplicative layer has too many sibling connections for one step program";
                return false;
            }
        }
        cur.post = o.post; cur.deriv_buf = o.deriv_buf; cur.out_buf = o.out_buf; cur.partial_out = false;
        new_index[r] = (int)out.size();
        out.push_back(cur);
    }
    for (size_t r = 0; r < out.size(); ++r) out[r].out_slot = (int)r;
    for (OpH& o : out)
        for (TermH& t : o.terms)
            for (FactorH& f : t.f) if (f.slot >= 0) f.slot = new_index[f.slot];
    ops.swap(out);
    return true;
}

// Emits the node operations of one phase as one or more programs; a phase is split when its
// operations together need more slots than a thread holds.  The matrix-vector tasks go with
// the first part (their sources never depend on this phase's own results).
bool emit_phase(Plan& P, std::vector<PhasePlan>& out, const std::vector<MvTaskH>& tasks, std::vector<OpH> ops,
                const std::vector<int>& part_bufs, std::vector<char> written, const std::vector<char>& shared, int step_dir,
                std::string& err) {
    if (!split_wide_ops(ops, part_bufs, P.buf_dim, P.buf_alloc, err)) return false;
    for (const OpH& o : ops) written[o.out_buf] = 1;
    EmitCtx ctx; ctx.written = &written; ctx.shared = &shared; ctx.step_dir = step_dir;
    int first = 0;
    bool first_part = true;
    const int n = (int)ops.size();
    while (first < n) {
        int last = first + 1, md = 0;
        if (emit_program(P.words, ops, first, last, P.buf_dim, md, true) < 0) {
            err = "a layer has too many element-wise connections for one step program";
            return false;
        }
        while (last < n && !ops[last].new_program && emit_program(P.words, ops, first, last + 1, P.buf_dim, md, true) == 0) ++last;
        PhasePlan ph;
        if (first_part && !tasks.empty()) { ph.mv_off = emit_matvecs(P.words, tasks, ph.mv_max_out); ph.n_mv_tasks = (int)tasks.size(); }
        ph.prog_off = emit_program(P.words, ops, first, last, P.buf_dim, ph.max_dim, false, &ctx);
        out.push_back(ph);
        first = last; first_part = false;
    }
    return true;
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
        if (e.wkind == W_FULL && (nodes[e.dst].kind == NODE_MUL || nodes[e.dst].kind == NODE_MAX)) {
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
    P.n_bufs = 7 * K;
    P.buf_dim.assign(P.n_bufs, 0);
    P.buf_alloc.assign(P.n_bufs, 0);
    P.hist = 0;
    P.input_staged.assign(K, 0);
    P.input_delayed.assign(K, 0);
    for (int m = 0; m < M; ++m) {
        P.hist = std::max(P.hist, xe[m].delay);
        if (xn[xe[m].src].kind == NODE_INPUT && xe[m].delay > 0) P.input_delayed[xe[m].src] = 1;
        if (xn[xe[m].src].kind == NODE_INPUT && (xe[m].delay > 0 || xe[m].wkind != W_FULL)) P.input_staged[xe[m].src] = 1;
    }
    for (int k = 0; k < K; ++k) {
        for (int b : {P.ybuf(k), P.dbuf(k), P.abuf(k), P.pbuf(k), P.qbuf(k), P.hbuf(k), P.fbuf(k)}) P.buf_dim[b] = xn[k].dim;
        if (xn[k].kind != NODE_INPUT) P.buf_alloc[P.ybuf(k)] = P.buf_alloc[P.dbuf(k)] = 1;
        else if (P.input_staged[k]) P.buf_alloc[P.ybuf(k)] = 1;
    }
    // y_src of a full connection inside a recurrent node is read by all workgroups during the
    // forward step loop, ds_dst during the backward one
    std::vector<char> shared_y(K, 0), shared_d(K, 0);
    for (int m = 0; m < M; ++m)
        if (xe[m].wkind == W_FULL && S.edge_class[m] != EDGE_BATCHED) { shared_y[xe[m].src] = 1; shared_d[xe[m].dst] = 1; }

    std::vector<std::vector<int>> in_e(K), out_e(K);
    for (int m = 0; m < M; ++m) { in_e[xe[m].dst].push_back(m); out_e[xe[m].src].push_back(m); }
    auto w_off_of = [&](int m) -> int { return xe[m].wkind == W_DIAG ? (int)P.edge_off[P.xedge_param[m]] : -1; };
    auto full_off = [&](int m) -> int64_t { return P.edge_off[P.xedge_param[m]]; };

    // Lowers component c into cp.  fused[m] marks full connections between different recurrent
    // components that the step kernel evaluates itself (as if they were delayed connections of
    // the component) instead of taking them from a GEMM over all frames.
    // fhelper / helper (optional): the forward / backward products of the fused connections go to
    // helper members instead (ChainPlan::fwd_split / bwd_split), which *fhelper / *helper receive;
    // one stays without a program if the component has no such connection in that direction.
    auto lower_component = [&](int c, const std::vector<char>& fused, CompPlan& cp, CompPlan* helper = nullptr, CompPlan* fhelper = nullptr) -> bool {
        auto batched = [&](int m) { return S.edge_class[m] == EDGE_BATCHED && !fused[m]; };
        cp.recurrent = S.comp_recurrent[c] != 0;
        std::vector<int> members;
        for (int k : S.comp_nodes[c]) if (xn[k].kind != NODE_INPUT) members.push_back(k);
        if (members.empty()) return true;
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
            GemmProblemPlan gp; gp.c_buf = shared_y[k] ? P.pbuf(k) : P.ybuf(k); gp.n = xn[k].dim;
            for (int m : in_e[k])
                if (xe[m].wkind == W_FULL && batched(m))
                    gp.pairs.push_back(GemmPairPlan{P.ybuf(xe[m].src), -1, full_off(m), xn[xe[m].src].dim, xe[m].delay});
            if (!gp.pairs.empty()) { cp.fwd_gemms.push_back(gp); P.buf_alloc[gp.c_buf] = 1; }
            if (shared_y[k]) cp.fwd_shared_bufs.push_back(P.ybuf(k));
            if (shared_d[k]) cp.bwd_shared_bufs.push_back(P.dbuf(k));
            if (xn[k].act == ACT_SOFTMAX) cp.softmax_node = k;
            else if (xn[k].is_output == OUT_SQUARED_ERROR) cp.sqerr_node = k;
        }
        for (int p = 0; p < n_phases; ++p) {
            std::vector<int> np;
            for (int k : members) if (phase[k] == p) np.push_back(k);
            std::map<int, int> slot;
            for (size_t i = 0; i < np.size(); ++i) slot[np[i]] = (int)i;
            std::vector<MvTaskH> tasks; std::vector<OpH> ops;
            std::vector<MvTaskH> htasks; std::vector<OpH> hops; std::vector<int> hparts;
            for (int k : np) {
                OpH o; o.dim = xn[k].dim; o.out_buf = P.ybuf(k); o.out_slot = slot[k];
                MvTaskH htask; htask.n_out = xn[k].dim; htask.acc_buf = P.abuf(k);
                o.post = xn[k].act == ACT_SIGMOID ? POST_SIGMOID : xn[k].act == ACT_TANH ? POST_TANH : xn[k].act == ACT_RELU ? POST_RELU : POST_NONE;
                if (xn[k].has_bias) o.bias_off = (int)P.bias_off[k];
                o.agg_max = xn[k].kind == NODE_MAX;
                MvTaskH task; task.n_out = xn[k].dim; task.acc_buf = P.abuf(k);
                TermH product;
                for (int m : in_e[k]) {
                    const GEdge& e = xe[m];
                    if (e.wkind == W_FULL) {
                        if (batched(m)) { o.pre_buf = shared_y[k] ? P.pbuf(k) : P.ybuf(k); o.pre_static = true; }
                        else if (fhelper && fused[m]) {
                            htask.edges.push_back(MvEdgeH{(int)full_off(m), xn[e.src].dim, 0, P.ybuf(e.src), -e.delay});
                            fhelper->step_weight_floats += (int64_t)xn[k].dim * xn[e.src].dim;
                        } else {
                            task.edges.push_back(MvEdgeH{(int)full_off(m), xn[e.src].dim, 0, P.ybuf(e.src), -e.delay});
                            cp.step_weight_floats += (int64_t)xn[k].dim * xn[e.src].dim;
                        }
                        continue;
                    }
                    FactorH f{P.ybuf(e.src), -e.delay, w_off_of(m), -1};
                    if (e.delay == 0 && slot.count(e.src) && slot[e.src] < slot[k]) f.slot = slot[e.src];
                    if (xn[k].kind == NODE_MUL) product.f.push_back(f);
                    else { TermH t; t.f.push_back(f); o.terms.push_back(t); }
                }
                if (xn[k].kind == NODE_MUL) o.terms.push_back(product);
                if (!task.edges.empty()) { o.acc_buf = task.acc_buf; o.acc_task = (int)tasks.size(); tasks.push_back(task); P.buf_alloc[task.acc_buf] = 2; }
                if (!htask.edges.empty()) {
                    // the helper's program: sum of its products, stored where this program polls it
                    o.polled_buf = P.fbuf(k);
                    OpH ho; ho.dim = xn[k].dim; ho.out_buf = P.fbuf(k); ho.out_slot = (int)hops.size();
                    ho.acc_buf = htask.acc_buf; ho.acc_task = (int)htasks.size();
                    htasks.push_back(htask); hops.push_back(ho); hparts.push_back(P.pbuf(k));
                    P.buf_alloc[htask.acc_buf] = 2; P.buf_alloc[P.fbuf(k)] = 1;
                    fhelper->fwd_shared_bufs.push_back(P.fbuf(k));
                }
                ops.push_back(o);
            }
            if (fhelper && !hops.empty()) {
                std::vector<char> hwritten(P.n_bufs, 0), hshared(P.n_bufs, 0);
                for (const OpH& ho : hops) hwritten[ho.out_buf] = hshared[ho.out_buf] = 1;
                if (!emit_phase(P, fhelper->fwd_phases, htasks, hops, hparts, hwritten, hshared, -1, err)) return false;
                fhelper->recurrent = true; fhelper->helper = true; fhelper->has_fwd_program = true;
            }
            std::vector<int> part_bufs;
            for (int k : np) part_bufs.push_back(P.pbuf(k));
            std::vector<char> written(P.n_bufs, 0);
            for (int k : members) written[P.ybuf(k)] = 1;
            std::vector<char> shared(P.n_bufs, 0);
            for (int k : members) if (shared_y[k]) shared[P.ybuf(k)] = 1;
            if (!emit_phase(P, cp.fwd_phases, tasks, ops, part_bufs, written, shared, cp.recurrent ? -1 : 0, err)) return false;
        }
        cp.has_fwd_program = true;
        auto emit_desc = [&](const std::vector<PhasePlan>& phs) {
            const int off = (int)P.words.size();
            P.words.push_back((int)phs.size());
            for (const PhasePlan& ph : phs) { P.words.push_back(ph.mv_off); P.words.push_back(ph.prog_off); }
            return off;
        };
        cp.fwd_desc_off = emit_desc(cp.fwd_phases);
        if (fhelper && fhelper->has_fwd_program) fhelper->fwd_desc_off = emit_desc(fhelper->fwd_phases);

        // ---- backward ----
        if (cp.softmax_node >= 0 || cp.sqerr_node >= 0) return true;   // the output delta comes from the error-criterion kernel
        for (int j : members) {
            GemmProblemPlan gp; gp.c_buf = shared_d[j] ? P.qbuf(j) : P.dbuf(j); gp.n = xn[j].dim;
            for (int m : out_e[j])
                if (xe[m].wkind == W_FULL && batched(m))
                    gp.pairs.push_back(GemmPairPlan{P.dbuf(xe[m].dst), -1, full_off(m), xn[xe[m].dst].dim, xe[m].delay});
            if (!gp.pairs.empty()) { cp.bwd_gemms.push_back(gp); P.buf_alloc[gp.c_buf] = 1; }
        }
        for (int p = n_phases - 1; p >= 0; --p) {
            std::vector<int> np;
            for (int k : members) if (phase[k] == p) np.push_back(k);
            std::reverse(np.begin(), np.end());
            std::map<int, int> slot;
            for (size_t i = 0; i < np.size(); ++i) slot[np[i]] = (int)i;
            std::vector<MvTaskH> tasks; std::vector<OpH> ops;
            std::vector<MvTaskH> htasks; std::vector<OpH> hops; std::vector<int> hparts;
            for (int j : np) {
                OpH o; o.dim = xn[j].dim; o.out_buf = P.dbuf(j); o.out_slot = slot[j];
                MvTaskH htask; htask.n_out = xn[j].dim; htask.acc_buf = P.abuf(j);
                if (xn[j].act == ACT_SIGMOID) { o.post = POST_DSIGMOID; o.deriv_buf = P.ybuf(j); }
                else if (xn[j].act == ACT_TANH) { o.post = POST_DTANH; o.deriv_buf = P.ybuf(j); }
                else if (xn[j].act == ACT_RELU) { o.post = POST_DRELU; o.deriv_buf = P.ybuf(j); }
                MvTaskH task; task.n_out = xn[j].dim; task.acc_buf = P.abuf(j);
                for (int m : out_e[j]) {
                    const GEdge& e = xe[m];
                    const int k = e.dst;
                    if (e.wkind == W_FULL) {
                        if (batched(m)) { o.pre_buf = shared_d[j] ? P.qbuf(j) : P.dbuf(j); o.pre_static = true; }
                        else if (helper && fused[m]) {
                            htask.edges.push_back(MvEdgeH{(int)full_off(m), xn[k].dim, 1, P.dbuf(k), e.delay});
                            helper->step_weight_floats += (int64_t)xn[j].dim * xn[k].dim;
                        }
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
                    if (xn[k].kind == NODE_MAX)      // the error goes to the connection that holds the maximum (the first one of several)
                        for (int m2 : in_e[k])
                            if (m2 != m) {
                                t.f.push_back(FactorH{P.ybuf(j), 0, w_off_of(m), -1, m2 < m ? 2 : 1});
                                t.f.push_back(FactorH{P.ybuf(xe[m2].src), e.delay - xe[m2].delay, w_off_of(m2), -1});
                            }
                    o.terms.push_back(t);
                }
                if (!task.edges.empty()) { o.acc_buf = task.acc_buf; o.acc_task = (int)tasks.size(); tasks.push_back(task); P.buf_alloc[task.acc_buf] = 2; }
                if (!htask.edges.empty()) {
                    // the helper's program: sum of its products, stored where this program polls it
                    o.polled_buf = P.hbuf(j);
                    OpH ho; ho.dim = xn[j].dim; ho.out_buf = P.hbuf(j); ho.out_slot = (int)hops.size();
                    ho.acc_buf = htask.acc_buf; ho.acc_task = (int)htasks.size();
                    htasks.push_back(htask); hops.push_back(ho); hparts.push_back(P.qbuf(j));
                    P.buf_alloc[htask.acc_buf] = 2; P.buf_alloc[P.hbuf(j)] = 1;
                    helper->bwd_shared_bufs.push_back(P.hbuf(j));
                }
                ops.push_back(o);
            }
            if (helper && !hops.empty()) {
                std::vector<char> hwritten(P.n_bufs, 0), hshared(P.n_bufs, 0);
                for (const OpH& ho : hops) hwritten[ho.out_buf] = hshared[ho.out_buf] = 1;
                if (!emit_phase(P, helper->bwd_phases, htasks, hops, hparts, hwritten, hshared, 1, err)) return false;
                helper->recurrent = true; helper->helper = true; helper->has_bwd_program = true;
            }
            std::vector<int> part_bufs;
            for (int j : np) part_bufs.push_back(P.qbuf(j));
            std::vector<char> written(P.n_bufs, 0);
            for (int k : members) written[P.dbuf(k)] = 1;
            std::vector<char> shared(P.n_bufs, 0);
            for (int k : members) if (shared_d[k]) shared[P.dbuf(k)] = 1;
            if (!emit_phase(P, cp.bwd_phases, tasks, ops, part_bufs, written, shared, cp.recurrent ? 1 : 0, err)) return false;
        }
        cp.has_bwd_program = true;
        cp.bwd_desc_off = emit_desc(cp.bwd_phases);
        if (helper && helper->has_bwd_program) helper->bwd_desc_off = emit_desc(helper->bwd_phases);
        return true;
    };
    P.comps.assign(S.n_comps, CompPlan());
    const std::vector<char> none(M, 0);
    for (int c = 0; c < S.n_comps; ++c)
        if (!lower_component(c, none, P.comps[c])) return false;

    // ---- chains of recurrent components that one step kernel can run side by side ----
    // Consecutive single-phase recurrent components c, c + 1, ... form a chain if every connection
    // between two of them is a full one whose source is already exchanged between workgroups in
    // the forward loop and whose destination is in the backward loop, and every other connection
    // of a member comes from a component before the chain or leads to one after it.
    {
        auto single_phase = [&](const CompPlan& cp) {
            return cp.recurrent && cp.fwd_phases.size() == 1 && cp.bwd_phases.size() == 1 && cp.softmax_node < 0 && cp.sqerr_node < 0;
        };
        int c = 0;
        while (c < S.n_comps) {
            if (!single_phase(P.comps[c])) { ++c; continue; }
            int last = c;
            while (last + 1 < S.n_comps && last + 1 - c + 1 <= STEP_MAX_GROUPS && single_phase(P.comps[last + 1])) {
                // try to extend the chain [c, last] by last + 1
                const int cand = last + 1;
                bool ok = true, linked = false;
                for (int m = 0; m < M && ok; ++m) {
                    const int cs = S.node_comp[xe[m].src], cd = S.node_comp[xe[m].dst];
                    if (cs == cd) continue;
                    const bool s_in = cs >= c && cs <= cand, d_in = cd >= c && cd <= cand;
                    if (s_in && d_in) {
                        if (xe[m].wkind != W_FULL || !shared_y[xe[m].src] || !shared_d[xe[m].dst] || cs > cd) ok = false;
                        else if (cd == cand) linked = true;
                    } else if (s_in && cd < cand) ok = false;       // leaves the chain into an earlier component
                    else if (d_in && cs > c) ok = false;            // enters the chain from a later component
                }
                if (!ok || !linked) break;
                last = cand;
            }
            if (last > c) {
                std::vector<char> fused(M, 0);
                for (int m = 0; m < M; ++m) {
                    const int cs = S.node_comp[xe[m].src], cd = S.node_comp[xe[m].dst];
                    if (cs != cd && cs >= c && cs <= last && cd >= c && cd <= last) fused[m] = 1;
                }
                ChainPlan ch; ch.first = c; ch.last = last;
                for (int k = c; k <= last; ++k) {
                    CompPlan fc;
                    if (!lower_component(k, fused, fc)) return false;
                    if (fc.fwd_phases.size() != 1 || fc.bwd_phases.size() != 1) { ch.members.clear(); break; }
                    ch.members.push_back(fc);
                }
                if (!ch.members.empty()) {
                    // the launches with helper members
                    std::vector<CompPlan> split(last - c + 1), bh(last - c + 1), fh(last - c + 1);
                    bool fok = true, bok = true;
                    for (int k = c; k <= last; ++k) {
                        const int i = k - c;
                        if (!lower_component(k, fused, split[i], &bh[i], &fh[i])) return false;
                        if (split[i].fwd_phases.size() != 1 || split[i].bwd_phases.size() != 1) fok = bok = false;
                        if (k > c && (!fh[i].has_fwd_program || fh[i].fwd_phases.size() != 1)) fok = false;
                        if (k < last && (!bh[i].has_bwd_program || bh[i].bwd_phases.size() != 1)) bok = false;
                    }
                    if (fok && 2 * (last - c) + 1 <= STEP_MAX_GROUPS) {
                        ch.fwd_split.push_back(ch.members.front());
                        for (int k = c + 1; k <= last; ++k) { ch.fwd_split.push_back(fh[k - c]); ch.fwd_split.push_back(split[k - c]); }
                    }
                    if (bok && 2 * (last - c) + 1 <= STEP_MAX_GROUPS) {
                        ch.bwd_split.push_back(ch.members.back());
                        for (int k = last - 1; k >= c; --k) { ch.bwd_split.push_back(bh[k - c]); ch.bwd_split.push_back(split[k - c]); }
                    }
                    for (int k = c; k <= last; ++k) P.comps[k].chain = (int)P.chains.size();
                    P.chains.push_back(ch);
                }
            }
            c = last + 1;
        }
    }

    // ---- exchange bundles: equally wide shared tensors of one single-phase recurrent component ----
    {
        auto make_bundles = [&](const std::vector<int>& shared_bufs) {
            size_t i = 0;
            while (i < shared_bufs.size()) {
                size_t j = i + 1;
                while (j < shared_bufs.size() && j - i < 4 && P.buf_dim[shared_bufs[j]] == P.buf_dim[shared_bufs[i]]) ++j;
                if (j - i >= 2) {
                    BundlePlan b;
                    b.B = j - i == 2 ? 2 : 4; b.dim = P.buf_dim[shared_bufs[i]];
                    for (size_t m = i; m < j; ++m) b.members[m - i] = shared_bufs[m];
                    b.ebuf = (int)P.buf_dim.size();
                    P.buf_dim.push_back(b.B * b.dim); P.buf_alloc.push_back(1);
                    P.bundles.push_back(b);
                }
                i = j;
            }
        };
        for (const CompPlan& cp : P.comps) {
            if (!cp.recurrent || cp.fwd_phases.size() != 1 || cp.bwd_phases.size() != 1) continue;
            make_bundles(cp.fwd_shared_bufs);
            make_bundles(cp.bwd_shared_bufs);
        }
        // ---- tile-blocked twins of the exchanged tensors ----
        P.twin_base = (int)P.buf_dim.size();
        for (int b = 0; b < P.twin_base; ++b) { P.buf_dim.push_back(P.buf_dim[b]); P.buf_alloc.push_back(0); }
        auto make_twins = [&](const CompPlan& cp) {
            if (!cp.recurrent || cp.fwd_phases.size() != 1 || cp.bwd_phases.size() != 1) return;
            for (const std::vector<int>* list : {&cp.fwd_shared_bufs, &cp.bwd_shared_bufs})
                for (int b : *list)
                    if (b < P.twin_base && P.buf_alloc[b] == 1 && P.buf_dim[b] % 16 == 0) P.buf_alloc[P.twin_base + b] = 3;
        };
        for (const CompPlan& cp : P.comps) make_twins(cp);
        for (const ChainPlan& ch : P.chains) for (const CompPlan& cp : ch.members) make_twins(cp);
        P.n_bufs = (int)P.buf_dim.size();
        P.bundle_of.assign(P.n_bufs, -1);
        for (size_t i = 0; i < P.bundles.size(); ++i)
            for (int m : P.bundles[i].members) if (m >= 0) P.bundle_of[m] = (int)i;
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
        for (const FactorH& f : fs) { P.words.push_back(f.buf); P.words.push_back(f.frame_off); P.words.push_back(f.w_off); P.words.push_back(f.cmp); }
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
        if (xn[e.dst].kind == NODE_MAX)
            for (int m2 : in_e[e.dst])
                if (m2 != m) {
                    fs.push_back(FactorH{P.ybuf(e.src), -e.delay, w_off_of(m), -1, m2 < m ? 2 : 1});
                    fs.push_back(FactorH{P.ybuf(xe[m2].src), -xe[m2].delay, w_off_of(m2), -1});
                }
        emit_colsum(xn[e.dst].dim, (int)full_off(m), fs);
    }
    for (int k = 0; k < K0; ++k)
        if (nodes[k].has_bias) emit_colsum(nodes[k].dim, (int)P.bias_off[k], {FactorH{P.dbuf(k), 0, -1, -1}});
    return true;
}

}  // namespace rnng
