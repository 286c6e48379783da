"""Seeded synthetic workloads: graph descriptions and input data.

This module is shared by the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds *no arithmetic of the method*: only (a) node / edge / delay
lists describing networks in the paper's graph notation (Section 2.1: a node is a
layer, an edge is a connection with a weight matrix and a delay) and (b) seeded
random weights, inputs and targets.

Enumerations are the interface's integer codes (they appear in the C header too):
  node kind : 0 input, 1 additive, 2 multiplicative, 3 element-wise maximum
  activation: 0 linear, 1 logistic sigmoid, 2 tanh, 3 softmax (output nodes only), 4 rectifier max(0, s)
  weight kind: 0 full matrix [n_dst x n_src], 1 diagonal (vector), 2 identity
  is_output : 0 no, 1 softmax output with class targets (cross-entropy), 2 output with dense
              targets under the squared error (linear, sigmoid, tanh or rectifier activation)
"""
from __future__ import annotations

import numpy as np

INPUT, ADD, MUL, MAX = 0, 1, 2, 3
LINEAR, SIGMOID, TANH, SOFTMAX, RELU = 0, 1, 2, 3, 4
FULL, DIAG, IDENTITY = 0, 1, 2
CROSS_ENTROPY, SQUARED_ERROR = 1, 2


class GraphSpec:
    """A network as a plain node list and edge list."""

    def __init__(self):
        self.nodes = []   # dicts: kind, act, dim, has_bias, is_output, name
        self.edges = []   # dicts: src, dst, delay, wkind

    def add_node(self, kind, act, dim, has_bias=False, is_output=False, name=""):
        self.nodes.append(dict(kind=int(kind), act=int(act), dim=int(dim),
                               has_bias=int(bool(has_bias)), is_output=int(is_output),
                               name=name or f"n{len(self.nodes)}"))
        return len(self.nodes) - 1

    def add_edge(self, src, dst, wkind, delay=0):
        self.edges.append(dict(src=int(src), dst=int(dst), delay=int(delay), wkind=int(wkind)))
        return len(self.edges) - 1

    # ---- flat int32 views in the C-ABI's descriptor layout -------------------------
    def node_array(self):
        return np.array([[n["kind"], n["act"], n["dim"], n["has_bias"], n["is_output"]]
                         for n in self.nodes], dtype=np.int32).reshape(-1, 5)

    def edge_array(self):
        return np.array([[e["src"], e["dst"], e["delay"], e["wkind"]]
                         for e in self.edges], dtype=np.int32).reshape(-1, 4)

    def input_nodes(self):
        return [k for k, n in enumerate(self.nodes) if n["kind"] == INPUT]

    def output_nodes(self):
        return [k for k, n in enumerate(self.nodes) if n["is_output"]]

    def node_by_name(self, name):
        for k, n in enumerate(self.nodes):
            if n["name"] == name:
                return k
        raise KeyError(name)

    def permuted(self, node_perm, edge_perm):
        """A relabelled copy: old node k becomes node_perm[k]; old edge m becomes edge_perm[m]."""
        g = GraphSpec()
        inv_n = np.argsort(np.asarray(node_perm))
        inv_e = np.argsort(np.asarray(edge_perm))
        for new in range(len(self.nodes)):
            g.nodes.append(dict(self.nodes[int(inv_n[new])]))
        for new in range(len(self.edges)):
            e = dict(self.edges[int(inv_e[new])])
            e["src"] = int(node_perm[e["src"]])
            e["dst"] = int(node_perm[e["dst"]])
            g.edges.append(e)
        return g


# ------------------------------------------------------------------------------------
# Network builders
# ------------------------------------------------------------------------------------
def add_lstm_layer(g, x, n_cells, tag, output_recurrence=True, extra_delay2_to_input_gate=False):
    """LSTM memory-block layer with forget gates and peepholes as add / multiply nodes
    (the construction of the paper's Fig. 1): 9 nodes, 20 edges (16 without the
    block-output -> gate recurrence, which is the variant used in the paper's
    language-model experiment, Section 4).  Returns a dict of node ids."""
    H = n_cells
    i = g.add_node(ADD, SIGMOID, H, has_bias=True, name=f"{tag}.i")
    f = g.add_node(ADD, SIGMOID, H, has_bias=True, name=f"{tag}.f")
    gg = g.add_node(ADD, TANH, H, has_bias=True, name=f"{tag}.g")
    mig = g.add_node(MUL, LINEAR, H, name=f"{tag}.m_ig")
    mfc = g.add_node(MUL, LINEAR, H, name=f"{tag}.m_fc")
    c = g.add_node(ADD, LINEAR, H, name=f"{tag}.c")
    o = g.add_node(ADD, SIGMOID, H, has_bias=True, name=f"{tag}.o")
    tc = g.add_node(ADD, TANH, H, name=f"{tag}.tc")
    h = g.add_node(MUL, LINEAR, H, name=f"{tag}.h")
    # input gate, forget gate, cell input, in this order of edges per node
    for gate in (i, f):
        g.add_edge(x, gate, FULL, 0)
        if output_recurrence:
            g.add_edge(h, gate, FULL, 1)
        g.add_edge(c, gate, DIAG, 1)          # peephole from c(t-1)
    g.add_edge(x, gg, FULL, 0)
    if output_recurrence:
        g.add_edge(h, gg, FULL, 1)
    g.add_edge(i, mig, IDENTITY, 0)
    g.add_edge(gg, mig, IDENTITY, 0)
    g.add_edge(f, mfc, IDENTITY, 0)
    g.add_edge(c, mfc, IDENTITY, 1)
    g.add_edge(mig, c, IDENTITY, 0)
    g.add_edge(mfc, c, IDENTITY, 0)
    g.add_edge(x, o, FULL, 0)
    if output_recurrence:
        g.add_edge(h, o, FULL, 1)
    g.add_edge(c, o, DIAG, 0)                 # peephole from c(t)
    g.add_edge(c, tc, IDENTITY, 0)
    g.add_edge(o, h, IDENTITY, 0)
    g.add_edge(tc, h, IDENTITY, 0)
    if extra_delay2_to_input_gate:
        g.add_edge(h, i, FULL, 2)
    return dict(i=i, f=f, g=gg, m_ig=mig, m_fc=mfc, c=c, o=o, tc=tc, h=h)


def lstm_net(n_in, hidden, n_out, output_recurrence=True, squared_error_act=None):
    """Stacked peephole-LSTM layers with an output layer on the top block output: softmax with
    class targets, or (squared_error_act = LINEAR / SIGMOID / TANH) a layer with dense targets
    under the squared error."""
    g = GraphSpec()
    x = g.add_node(INPUT, LINEAR, n_in, name="x")
    top = x
    for l, H in enumerate(hidden):
        top = add_lstm_layer(g, top, H, f"L{l + 1}", output_recurrence)["h"]
    if squared_error_act is None:
        out = g.add_node(ADD, SOFTMAX, n_out, has_bias=True, is_output=CROSS_ENTROPY, name="out")
    else:
        out = g.add_node(ADD, squared_error_act, n_out, has_bias=True, is_output=SQUARED_ERROR, name="out")
    g.add_edge(top, out, FULL, 0)
    return g


def elman_net(n_in, n_hidden, n_out, act=TANH):
    """Elman network: one hidden layer with a delay-1 full self-loop (Section 4's other net)."""
    g = GraphSpec()
    x = g.add_node(INPUT, LINEAR, n_in, name="x")
    h = g.add_node(ADD, act, n_hidden, has_bias=True, name="h")
    out = g.add_node(ADD, SOFTMAX, n_out, has_bias=True, is_output=True, name="out")
    g.add_edge(x, h, FULL, 0)
    g.add_edge(h, h, FULL, 1)
    g.add_edge(h, out, FULL, 0)
    return g


def generalized_net(n_in=128, n_cells=1024, n_layers=3, n_out=256):
    """Three peephole-LSTM layers, each with an extra delay-2 full edge from its block
    output to its own input gate; between consecutive layers a sigmoid node q (full
    edge from the lower block output, bias) gates the lower block output through a
    multiplicative node p, which is the next layer's input."""
    g = GraphSpec()
    x = g.add_node(INPUT, LINEAR, n_in, name="x")
    top = x
    for l in range(n_layers):
        h = add_lstm_layer(g, top, n_cells, f"L{l + 1}", True, extra_delay2_to_input_gate=True)["h"]
        if l + 1 < n_layers:
            q = g.add_node(ADD, SIGMOID, n_cells, has_bias=True, name=f"q{l + 1}")
            p = g.add_node(MUL, LINEAR, n_cells, name=f"p{l + 1}")
            g.add_edge(h, q, FULL, 0)
            g.add_edge(h, p, IDENTITY, 0)
            g.add_edge(q, p, IDENTITY, 0)
            top = p
        else:
            top = h
    out = g.add_node(ADD, SOFTMAX, n_out, has_bias=True, is_output=True, name="out")
    g.add_edge(top, out, FULL, 0)
    return g


def random_graph(rng, n_inner=6, max_dim=5, p_edge=0.35, max_delay=3, n_inputs=1, force_mul=True, squared_error_outputs=0,
                 acts=(LINEAR, SIGMOID, TANH), max_fraction=0.0):
    """A small random valid graph for brute-force / finite-difference tests: additive and
    multiplicative nodes, full / diagonal / identity edges, delays 0..max_delay, multiple
    edges between a node pair, self-loops; delay-0 edges only run from lower to higher node
    id, so the delay-0 subgraph is acyclic.  acts: the activations the inner nodes draw from;
    max_fraction: share of the inner nodes that take the element-wise maximum of their inputs."""
    g = GraphSpec()
    dims = [int(rng.integers(2, max_dim + 1)) for _ in range(2)]   # two dim classes
    ins = [g.add_node(INPUT, LINEAR, dims[int(rng.integers(0, 2))], name=f"x{j}") for j in range(n_inputs)]
    inner = []
    for j in range(n_inner):
        kind = MUL if (rng.random() < 0.35 or (force_mul and j == n_inner // 2)) else ADD
        if max_fraction > 0 and not (force_mul and j == n_inner // 2) and rng.random() < max_fraction:
            kind = MAX
        act = int(acts[int(rng.integers(0, len(acts)))])
        dim = dims[int(rng.integers(0, 2))]
        inner.append(g.add_node(kind, act, dim, has_bias=(kind == ADD and rng.random() < 0.5), name=f"v{j}"))
    out = g.add_node(ADD, SOFTMAX, int(rng.integers(2, 5)), has_bias=True, is_output=True, name="out")

    def wkind_for(s, d):
        if g.nodes[s]["dim"] == g.nodes[d]["dim"]:
            return int(rng.integers(0, 3))
        return FULL

    for d in inner:
        cands = [s for s in ins + inner]
        n_in_edges = 0
        for s in cands:
            if rng.random() < p_edge:
                delay = int(rng.integers(0, max_delay + 1))
                if s >= d and delay == 0:
                    delay = 1 + int(rng.integers(0, max_delay))
                g.add_edge(s, d, wkind_for(s, d), delay)
                n_in_edges += 1
                if rng.random() < 0.15:            # a second edge on the same node pair
                    g.add_edge(s, d, wkind_for(s, d), 1 + int(rng.integers(0, max_delay)))
        if n_in_edges == 0:                         # every non-input node needs an in-edge
            s = ins[0] if d == inner[0] else int(rng.choice([v for v in ins + inner if v < d]))
            g.add_edge(s, d, wkind_for(s, d), 0)
    # output reads a random non-empty subset of inner nodes (not all: some stay unreachable)
    k = int(rng.integers(1, max(2, n_inner // 2)))
    for s in rng.choice(inner, size=k, replace=False):
        g.add_edge(int(s), out, FULL, int(rng.integers(0, 2)))
    # further output nodes with dense targets under the squared error (drawn after everything
    # else, so that graphs without them are what they were)
    for j in range(squared_error_outputs):
        o2 = g.add_node(ADD, int(rng.integers(0, 3)), int(rng.integers(2, 5)), has_bias=True, is_output=SQUARED_ERROR, name=f"sq{j}")
        for s in rng.choice(inner, size=int(rng.integers(1, 3)), replace=False):
            g.add_edge(int(s), o2, FULL, int(rng.integers(0, 2)))
    return g


# ------------------------------------------------------------------------------------
# Seeded data
# ------------------------------------------------------------------------------------
def draw_params(spec, rng, scale, bias_scale=0.0):
    """Weights per edge (index order): FULL -> [n_dst, n_src], DIAG -> [dim], IDENTITY -> None,
    uniform in (-scale, scale), float32.  Biases per node (index order): zeros unless
    bias_scale > 0."""
    weights, biases = [], []
    for e in spec.edges:
        ns, nd = spec.nodes[e["src"]]["dim"], spec.nodes[e["dst"]]["dim"]
        if e["wkind"] == FULL:
            weights.append(rng.uniform(-scale, scale, size=(nd, ns)).astype(np.float32))
        elif e["wkind"] == DIAG:
            weights.append(rng.uniform(-scale, scale, size=(nd,)).astype(np.float32))
        else:
            weights.append(None)
    for n in spec.nodes:
        if n["has_bias"]:
            if bias_scale > 0:
                biases.append(rng.uniform(-bias_scale, bias_scale, size=(n["dim"],)).astype(np.float32))
            else:
                biases.append(np.zeros((n["dim"],), dtype=np.float32))
        else:
            biases.append(None)
    return weights, biases


def draw_gaussian_inputs(spec, rng, T, N):
    return {k: rng.standard_normal(size=(T, N, spec.nodes[k]["dim"])).astype(np.float32)
            for k in spec.input_nodes()}


def draw_class_targets(spec, rng, T, N, masked_fraction=0.0):
    """Targets per output node: class indices [T, N] (int32, -1 = masked frame) for softmax
    outputs, dense N(0, 1) vectors [T, N, dim] (float32, NaN = masked frame) for squared-error outputs."""
    tg = {}
    for k in spec.output_nodes():
        if spec.nodes[k]["is_output"] == SQUARED_ERROR:
            t = rng.standard_normal(size=(T, N, spec.nodes[k]["dim"])).astype(np.float32)
            if masked_fraction > 0:
                t[rng.random(size=(T, N)) < masked_fraction] = np.nan
            tg[k] = t
            continue
        t = rng.integers(0, spec.nodes[k]["dim"], size=(T, N)).astype(np.int32)
        if masked_fraction > 0:
            t[rng.random(size=(T, N)) < masked_fraction] = -1
        tg[k] = t
    return tg


def draw_symbol_streams(spec, rng, T, N):
    """Character-LM-shaped data: each stream is its own uniform symbol sequence u(0..T);
    input frame t is one-hot of u(t), target is u(t+1).  Streams are drawn in order."""
    (x,) = spec.input_nodes()
    (o,) = spec.output_nodes()
    V = spec.nodes[x]["dim"]
    assert spec.nodes[o]["dim"] == V
    inp = np.zeros((T, N, V), dtype=np.float32)
    tgt = np.zeros((T, N), dtype=np.int32)
    for n in range(N):
        u = rng.integers(0, V, size=T + 1)
        inp[np.arange(T), n, u[:T]] = 1.0
        tgt[:, n] = u[1:]
    return {x: inp}, {o: tgt}


def draw_word_streams(spec, rng, T, N):
    """Word-LM-shaped data (the shape of the paper's Section 4 experiment): input frame t is the
    one-hot of a uniform word over the input vocabulary, the target a uniform word over the
    (smaller) output vocabulary.  Streams are drawn in order."""
    (x,) = spec.input_nodes()
    (o,) = spec.output_nodes()
    V, Vo = spec.nodes[x]["dim"], spec.nodes[o]["dim"]
    inp = np.zeros((T, N, V), dtype=np.float32)
    tgt = np.zeros((T, N), dtype=np.int32)
    for n in range(N):
        inp[np.arange(T), n, rng.integers(0, V, size=T)] = 1.0
        tgt[:, n] = rng.integers(0, Vo, size=T)
    return {x: inp}, {o: tgt}


class Workload:
    def __init__(self, name, spec, T, N, weights, biases, inputs, targets):
        self.name, self.spec, self.T, self.N = name, spec, T, N
        self.weights, self.biases, self.inputs, self.targets = weights, biases, inputs, targets

    def n_params(self):
        return sum(w.size for w in self.weights if w is not None) + \
            sum(b.size for b in self.biases if b is not None)


CONFIG_NAMES = ["tiny", "speech_n1", "charlm_n1", "charlm_n32", "generalized_n64"]
EXPERIMENT_SHAPES = ["lm_elman_n1", "lm_lstm_n1"]      # the paper's own Section 4 network shapes, synthetic words
# Section 4, second experiment (Fig. 4): peephole LSTM whose input, LSTM and output layers are all
# H wide, mini-batch N * h' = 1,024 frames with BPTT(2h'; h'), i.e. a window of T = 2,048 / N frames
FIG4_SHAPES = [f"fig4_h{H}_n{N}" for H in (1024, 2048, 4096) for N in (1, 16, 64)]


def make_config(name, seed=0, T=None, N=None, bias_scale=0.0):
    """The five benchmark / parity configurations.  Draw order: weights (edge index order),
    biases, inputs, targets -- all from one numpy PCG64 generator seeded with `seed`."""
    rng = np.random.default_rng(seed)
    if name == "tiny":
        spec, T0, N0, a, kind = lstm_net(8, [16], 4), 20, 1, 0.1, "gauss"
    elif name == "speech_n1":
        spec, T0, N0, a, kind = lstm_net(40, [256, 256], 61), 1024, 1, 0.1, "gauss"
    elif name == "charlm_n1":
        spec, T0, N0, a, kind = lstm_net(30, [512, 512], 30), 512, 1, 0.08, "symbols"
    elif name == "charlm_n32":
        spec, T0, N0, a, kind = lstm_net(30, [512, 512], 30), 256, 32, 0.08, "symbols"
    elif name == "generalized_n64":
        spec, T0, N0, a, kind = generalized_net(128, 1024, 3, 256), 128, 64, 0.05, "gauss"
    elif name == "lm_elman_n1":      # Section 4: Elman network 38,000-512-20,000, mini-batch 1,024, BPTT(2h'; h')
        spec, T0, N0, a, kind = elman_net(38000, 512, 20000), 2048, 1, 0.05, "words"
    elif name == "lm_lstm_n1":       # Section 4: LSTM without the block-output -> gate recurrence, same sizes
        spec, T0, N0, a, kind = lstm_net(38000, [512], 20000, output_recurrence=False), 2048, 1, 0.05, "words"
    elif name.startswith("fig4_h"):
        H, N0 = (int(v) for v in name[len("fig4_h"):].split("_n"))
        spec, T0, a, kind = lstm_net(H, [H], H), 2048 // N0, 0.02, "gauss"
    else:
        raise ValueError(name)
    T = T0 if T is None else T
    N = N0 if N is None else N
    weights, biases = draw_params(spec, rng, a, bias_scale)
    if kind == "gauss":
        inputs = draw_gaussian_inputs(spec, rng, T, N)
        targets = draw_class_targets(spec, rng, T, N)
    elif kind == "words":
        inputs, targets = draw_word_streams(spec, rng, T, N)
    else:
        inputs, targets = draw_symbol_streams(spec, rng, T, N)
    return Workload(name, spec, T, N, weights, biases, inputs, targets)


def make_workload(name, spec, T, N, seed=0, scale=0.3, bias_scale=0.2, masked_fraction=0.0):
    rng = np.random.default_rng(seed)
    weights, biases = draw_params(spec, rng, scale, bias_scale)
    inputs = draw_gaussian_inputs(spec, rng, T, N)
    targets = draw_class_targets(spec, rng, T, N, masked_fraction)
    return Workload(name, spec, T, N, weights, biases, inputs, targets)
