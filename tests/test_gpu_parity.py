"""GPU parity: the HIP path (through the C ABI) against the float64 oracle, element by element,
on the same seeded inputs.  Bars: outputs / activations within 1e-4, gradients (state gradients
and weight gradients) within 1e-3, per tensor both normwise, max|gpu - oracle| / max|oracle|, and
element by element, |gpu - oracle| / (|oracle| + max|oracle| / 10); the loss within 1e-5 relative.  Schedule parity (bit-exact) is a CPU test in test_abi_host.py."""
import numpy as np
import pytest

import workloads as wl
from oracle import graph_oracle as go

pytestmark = pytest.mark.gpu

OUT_TOL, GRAD_TOL = 1e-4, 1e-3
WORST = {}      # label -> worst normwise errors seen (printed)


def nerr(a, b):
    """Normwise error max|a - b| / max|b|, and on top of it an element-wise bound: every element
    must lie within the same relative tolerance of its own oracle value once that value is above a
    tenth of the tensor's maximum (so an element far below the maximum cannot be wholly wrong
    unseen).  Returned: the larger of the normwise error and the worst such element-wise error
    (scaled so that the callers' bars apply to both)."""
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    if not den > 0:
        return np.abs(a).max()
    normwise = np.abs(a - b).max() / den
    elementwise = (np.abs(a - b) / (np.abs(b) + 0.1 * den)).max()
    return max(normwise, elementwise)


def run_both(w, check_all_nodes=True, label=""):
    from paper_1503_02852_amd.runner import window_for
    print(f"[parity] {label or w.name}: T={w.T} N={w.N} nodes={len(w.spec.nodes)} params={w.n_params()}", flush=True)
    win = window_for(w)
    win.forward()
    win.bptt()
    loss = win.compute_grads(want_loss=True)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    worst_y = worst_d = worst_g = 0.0
    nodes = range(len(w.spec.nodes)) if check_all_nodes else w.spec.output_nodes()
    for k in nodes:
        if w.spec.nodes[k]["kind"] == wl.INPUT:
            continue
        e = nerr(win.node_output(k), ref["y"][k])
        worst_y = max(worst_y, e)
        assert e < OUT_TOL, (label, "y", w.spec.nodes[k]["name"], e)
        # library returns dE/ds = -delta
        e = nerr(win.node_state_grad(k), -ref["delta"][k])
        worst_d = max(worst_d, e)
        assert e < GRAD_TOL, (label, "ds", w.spec.nodes[k]["name"], e)
    gw, gb = win.grads_unpacked()
    for m, g in enumerate(ref["grad_w"]):
        if g is None:
            continue
        e = nerr(gw[m], g)
        worst_g = max(worst_g, e)
        assert e < GRAD_TOL, (label, "grad_w", m, w.spec.edges[m], e)
    for k, g in enumerate(ref["grad_b"]):
        if g is None:
            continue
        e = nerr(gb[k], g)
        worst_g = max(worst_g, e)
        assert e < GRAD_TOL, (label, "grad_b", w.spec.nodes[k]["name"], e)
    assert abs(loss - ref["loss"]) <= 1e-5 * max(1.0, abs(ref["loss"])), (label, loss, ref["loss"])
    win.check()
    builds = sorted({win.g.step_build(k, b) for k in range(len(w.spec.nodes)) for b in (False, True)} - {("none", False)})
    print(f"[parity] {label or w.name}: worst y {worst_y:.2e}  ds {worst_d:.2e}  grad {worst_g:.2e}  loss {loss:.6f}  "
          f"step builds {builds}", flush=True)
    WORST[label or w.name] = dict(y=worst_y, ds=worst_d, grad=worst_g)
    return win, ref


def test_tiny_config():
    run_both(wl.make_config("tiny"))


def test_tiny_config_with_biases_and_masked_targets():
    spec = wl.lstm_net(8, [16], 4)
    run_both(wl.make_workload("tiny_masked", spec, 20, 3, seed=1, scale=0.5, bias_scale=0.3, masked_fraction=0.3))


@pytest.mark.parametrize("seed", range(10))
def test_random_graphs(seed):
    rng = np.random.default_rng(100 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, n_inputs=1 + seed % 2)
    run_both(wl.make_workload(f"rand{seed}", spec, T=7 + seed, N=1 + seed % 4, seed=seed, scale=0.8, bias_scale=0.5,
                              masked_fraction=0.2 if seed % 2 else 0.0))


def test_elman():
    run_both(wl.make_workload("elman", wl.elman_net(20, 150, 11), T=33, N=5, seed=2, scale=0.15))


RELU_ACTS = (wl.LINEAR, wl.SIGMOID, wl.TANH, wl.RELU, wl.RELU)


@pytest.mark.parametrize("N", [1, 5, 33])
def test_rectifier_elman(N):
    """A rectified Elman layer (Section 2.1 leaves the activation function open): weights in
    registers at few streams, matrix cores at many."""
    w = wl.make_workload("elman_relu", wl.elman_net(20, 150, 11, act=wl.RELU), T=21, N=N, seed=5, scale=0.1, bias_scale=0.2)
    win, ref = run_both(w, label=f"rectifier Elman, N={N}")
    h = ref["y"][1]
    assert (h == 0).any() and (h > 0).any()


@pytest.mark.parametrize("seed", range(6))
def test_random_graphs_with_rectifiers(seed):
    """Random recurrent graphs whose additive and multiplicative nodes draw the rectifier too."""
    rng = np.random.default_rng(900 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, n_inputs=1 + seed % 2, acts=RELU_ACTS)
    run_both(wl.make_workload(f"rand_relu{seed}", spec, T=8 + seed, N=1 + 4 * (seed % 3), seed=seed, scale=0.8, bias_scale=0.5,
                              masked_fraction=0.2 if seed % 2 else 0.0))


def maxout_net(n_in, H, n_out, pieces=3):
    """An Elman-like layer of maximum units (Section 2.1: another aggregation function): `pieces`
    tanh layers fed by the input and the delayed output, whose element-wise maximum (taken through
    diagonal and identity connections, one of them delayed) is the layer's output."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, n_in, name="x")
    ps = [g.add_node(wl.ADD, wl.TANH, H, has_bias=True, name=f"p{j}") for j in range(pieces)]
    m = g.add_node(wl.MAX, wl.LINEAR, H, name="m")
    out = g.add_node(wl.ADD, wl.SOFTMAX, n_out, has_bias=True, is_output=True, name="out")
    for j, p in enumerate(ps):
        g.add_edge(x, p, wl.FULL, 0)
        g.add_edge(m, p, wl.FULL, 1)
        g.add_edge(p, m, wl.DIAG if j % 2 == 0 else wl.IDENTITY, 0)
    g.add_edge(m, m, wl.DIAG, 2)
    g.add_edge(m, out, wl.FULL, 0)
    return g


@pytest.mark.parametrize("H,N", [(24, 1), (150, 3), (64, 20), (256, 32)])
def test_maximum_units(H, N):
    """Layers of maximum units inside a recurrent node, at few streams and many."""
    w = wl.make_workload("maxout", maxout_net(10, H, 6), T=14, N=N, seed=9, scale=0.5 if H < 100 else 0.12, bias_scale=0.3, masked_fraction=0.2)
    run_both(w, label=f"maximum units, H={H}, N={N}")


def test_full_connection_into_a_maximum_node():
    """Full connections into a maximum node go through a linear node of their own, as into a
    multiplicative node; here outside any recurrent node (batched)."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 7, name="x")
    h = g.add_node(wl.ADD, wl.TANH, 9, has_bias=True, name="h")
    m = g.add_node(wl.MAX, wl.SIGMOID, 9, name="m")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 4, has_bias=True, is_output=True, name="out")
    g.add_edge(x, h, wl.FULL, 0); g.add_edge(h, h, wl.FULL, 1)
    g.add_edge(x, m, wl.FULL, 0); g.add_edge(h, m, wl.IDENTITY, 0); g.add_edge(h, m, wl.DIAG, 1); g.add_edge(x, m, wl.FULL, 2)
    g.add_edge(m, out, wl.FULL, 0)
    run_both(wl.make_workload("max_full", g, T=11, N=3, seed=10, scale=0.6, bias_scale=0.3), label="full connections into a maximum node")


@pytest.mark.parametrize("seed", [0, 1, 2, 4, 5, 7, 9, 10])
def test_random_graphs_with_maximum_nodes(seed):
    rng = np.random.default_rng(950 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, n_inputs=1 + seed % 2, max_fraction=0.5, acts=RELU_ACTS)
    run_both(wl.make_workload(f"rand_max{seed}", spec, T=8 + seed, N=1 + 4 * (seed % 3), seed=seed, scale=0.8, bias_scale=0.5,
                              masked_fraction=0.2 if seed % 2 else 0.0))


def test_maximum_units_with_the_interpreting_step_kernel(monkeypatch):
    monkeypatch.setenv("RNNG_JIT", "0")
    run_both(wl.make_workload("maxout", maxout_net(10, 24, 6), T=14, N=2, seed=11, scale=0.5, bias_scale=0.3), label="maximum units, RNNG_JIT=0")


def test_rectifier_with_the_interpreting_step_kernel(monkeypatch):
    monkeypatch.setenv("RNNG_JIT", "0")
    run_both(wl.make_workload("elman_relu", wl.elman_net(9, 40, 5, act=wl.RELU), T=13, N=3, seed=6, scale=0.2, bias_scale=0.2), label="rectifier Elman, RNNG_JIT=0")


def test_lstm_without_output_recurrence():
    run_both(wl.make_workload("lm_lstm", wl.lstm_net(12, [70], 9, output_recurrence=False), T=40, N=3, seed=3, scale=0.3))


def test_delay0_full_edge_inside_recurrent_node():
    """A recurrent node whose per-step DAG contains a full (not element-wise) edge: h -> p (full,
    delay 0), p -> h (full, delay 1) -- needs a second phase inside every step."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 6, name="x")
    h = g.add_node(wl.ADD, wl.TANH, 40, has_bias=True, name="h")
    p = g.add_node(wl.ADD, wl.SIGMOID, 17, has_bias=True, name="p")
    m = g.add_node(wl.MUL, wl.LINEAR, 17, name="m")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 5, has_bias=True, is_output=True, name="out")
    g.add_edge(x, h, wl.FULL, 0); g.add_edge(h, p, wl.FULL, 0); g.add_edge(p, h, wl.FULL, 1)
    g.add_edge(p, m, wl.IDENTITY, 0); g.add_edge(h, m, wl.FULL, 2); g.add_edge(m, out, wl.FULL, 0)
    g.add_edge(m, h, wl.FULL, 1)
    run_both(wl.make_workload("two_phase", g, T=19, N=3, seed=4, scale=0.4, bias_scale=0.2))


def test_widths_spanning_tiles_with_ragged_tails():
    """2-layer LSTM with widths that are not multiples of the GEMM tile, the wavefront or 4."""
    run_both(wl.make_workload("ragged", wl.lstm_net(37, [130, 67], 13), T=50, N=7, seed=5, scale=0.2, bias_scale=0.1))


def test_generalized_small():
    run_both(wl.make_workload("gen_small", wl.generalized_net(24, 96, 3, 10), T=24, N=5, seed=6, scale=0.15, bias_scale=0.1))


def test_single_frame_window():
    run_both(wl.make_workload("T1", wl.lstm_net(5, [8], 3), T=1, N=2, seed=7))
    run_both(wl.make_workload("T2_gen", wl.generalized_net(5, 8, 2, 3), T=2, N=1, seed=8))


def test_all_targets_masked_gives_zero_gradients():
    from paper_1503_02852_amd.runner import window_for
    w = wl.make_workload("masked", wl.lstm_net(5, [8], 3), T=6, N=2, seed=9, masked_fraction=1.1)
    win = window_for(w)
    win.forward(); win.bptt()
    loss = win.compute_grads(want_loss=True)
    assert loss == 0.0
    assert float(win.grads.abs().max().item()) == 0.0


def test_repeated_windows_reuse_the_workspace():
    """Two different windows through one handle; the second (smaller inputs) must not see the first."""
    from paper_1503_02852_amd.runner import window_for
    w1 = wl.make_workload("a", wl.lstm_net(6, [20], 4), T=15, N=2, seed=10)
    win, ref1 = run_both(w1)
    w2 = wl.make_workload("b", w1.spec, T=15, N=2, seed=11)
    win.set_params(w2.weights, w2.biases); win.set_inputs(w2.inputs); win.set_targets(w2.targets)
    win.forward(); win.bptt(); loss = win.compute_grads(want_loss=True)
    ref2 = go.forward_bptt(w2.spec.nodes, w2.spec.edges, w2.weights, w2.biases, w2.inputs, w2.targets, w2.T, w2.N)
    gw, gb = win.grads_unpacked()
    for m, g in enumerate(ref2["grad_w"]):
        if g is not None:
            assert nerr(gw[m], g) < GRAD_TOL
    assert abs(loss - ref2["loss"]) <= 1e-5 * abs(ref2["loss"])


@pytest.mark.parametrize("name", ["speech_n1", "charlm_n1", "charlm_n32"])
def test_full_size_configs(name):
    run_both(wl.make_config(name), label=name)


def test_generalized_full_width_reduced_window():
    """The generalized configuration at its full widths and stream count (3 x 1024, N = 64) over a
    24-frame window, which the oracle finishes in seconds."""
    run_both(wl.make_config("generalized_n64", T=24), check_all_nodes=True, label="generalized_n64_T24")


def test_generalized_full_size():
    """The generalized configuration as benchmarked: 3 x 1024, N = 64, T = 128 (the oracle needs
    about half a minute)."""
    win, _ = run_both(wl.make_config("generalized_n64"), check_all_nodes=True, label="generalized_n64")
    spec = wl.make_config("generalized_n64", T=1).spec
    assert win.g.step_build(spec.node_by_name("L1.h"))[0] in ("matrix", "matrix_2d")


@pytest.mark.parametrize("seed", [8, 17])
def test_dense_random_graph_splits_step_programs(seed):
    """Dense random graphs whose recurrent node needs more element-wise values per step than one
    program holds: the planner splits the step into several programs (and wide sums into parts)."""
    rng = np.random.default_rng(1000 + seed)
    spec = wl.random_graph(rng, n_inner=3 + seed % 9, p_edge=0.15 + 0.05 * (seed % 6), max_delay=3, n_inputs=1 + seed % 2)
    run_both(wl.make_workload(f"dense{seed}", spec, T=9, N=2, seed=seed, scale=0.5, bias_scale=0.3))


def test_many_streams_ragged_widths():
    """More than 8 streams (matrix-core step kernel) with widths and a stream count that are not
    multiples of the MFMA tile or of 4."""
    run_both(wl.make_workload("ragged_n19", wl.lstm_net(37, [130, 67], 13), T=12, N=19, seed=12, scale=0.2, bias_scale=0.1))
    run_both(wl.make_workload("elman_n33", wl.elman_net(20, 150, 11), T=9, N=33, seed=13, scale=0.15))


def test_many_streams_generalized_small():
    run_both(wl.make_workload("gen_n24", wl.generalized_net(24, 96, 3, 10), T=10, N=24, seed=14, scale=0.15, bias_scale=0.1))


# ---- recurrent components that run side by side in one launch (stacked layers linked by full edges) ----

def test_three_layer_lstm_stack():
    spec = wl.lstm_net(12, [20, 24, 16], 5)
    run_both(wl.make_workload("lstm3", spec, T=19, N=2, seed=21, scale=0.4, bias_scale=0.3, masked_fraction=0.2))


@pytest.mark.parametrize("layers,N", [([24, 20], 16), ([16, 24, 12], 20), ([40, 36], 33)])
def test_lstm_stack_with_many_streams_runs_side_by_side(layers, N):
    """Stacked layers at N >= 9 (matrix-core build): the members of a stack share one launch."""
    spec = wl.lstm_net(12, layers, 5)
    run_both(wl.make_workload("lstm_stack_streams", spec, T=15, N=N, seed=31, scale=0.4, bias_scale=0.3, masked_fraction=0.2))


@pytest.mark.parametrize("helpers", ["1", "0"])
@pytest.mark.parametrize("layers,N", [([64, 32], 32), ([128, 128], 16), ([32, 64], 48)])
def test_two_layer_stack_backward_with_and_without_helper_members(monkeypatch, layers, N, helpers):
    """A two-layer stack at a multiple of 16 streams: in the backward launch the products of the
    connections between the layers are computed by a helper member on otherwise idle compute units
    and polled element by element by the lower layer's program (RNNG_CHAIN_HELPERS = 0: contracted
    by the lower layer itself)."""
    monkeypatch.setenv("RNNG_CHAIN_HELPERS", helpers)
    spec = wl.lstm_net(12, layers, 5)
    win, _ = run_both(wl.make_workload("lstm_stack_helpers", spec, T=17, N=N, seed=35, scale=0.3, bias_scale=0.3, masked_fraction=0.2),
                      label=f"stack {layers}, N={N}, RNNG_CHAIN_HELPERS={helpers}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, True) == ("matrix", True) for k in rec)
    assert all(win.g.step_build_has_helpers(k, True) == (helpers == "1") for k in rec)
    assert not any(win.g.step_build_has_helpers(k, False) for k in rec)


@pytest.mark.parametrize("N,fwd,bwd", [(1, False, True), (2, False, True)])
def test_helper_groups_chosen_by_the_work_they_take_over(N, fwd, bwd):
    """Two 256-wide layers, default switches: the helper group takes 32 multiply-adds per lane,
    step and stream from the layer it serves; backward launches get it from 24 on, forward launches
    from 100 on (the full-size charlm_n1 configuration, 128 per lane, has it in both)."""
    spec = wl.lstm_net(12, [256, 256], 5)
    win, _ = run_both(wl.make_workload("lstm_stack_256", spec, T=15, N=N, seed=38, scale=0.08, bias_scale=0.3, masked_fraction=0.2), label=f"stack [256, 256], N={N}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b) == ("wave", True) for k in rec for b in (False, True))
    assert all(win.g.step_build_has_helpers(k, False) == fwd and win.g.step_build_has_helpers(k, True) == bwd for k in rec)


def test_small_stack_at_eight_streams_in_one_launch():
    """Two 40-wide layers at 8 streams: the source areas of the backward launch's two groups (eight
    and four short source vectors, a quad per lane each: 128 + 64 KiB) fit the 160 KiB of LDS only
    because the groups' areas lie on top of each other."""
    spec = wl.lstm_net(12, [40, 40], 5)
    win, _ = run_both(wl.make_workload("lstm_stack_n8", spec, T=19, N=8, seed=37, scale=0.3, bias_scale=0.3, masked_fraction=0.2), label="stack [40, 40], N=8")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b) == ("wave", True) for k in rec for b in (False, True))


@pytest.mark.parametrize("helpers", ["1", "0"])
@pytest.mark.parametrize("layers,N", [([24, 20], 1), ([64, 48], 2), ([40, 40], 4), ([512, 512], 1)])
def test_two_layer_stack_at_few_streams_with_and_without_helper_groups(monkeypatch, layers, N, helpers):
    """A two-layer stack in the weights-in-registers build: with RNNG_CHAIN_HELPERS = 1 a third
    group of workgroups (on an XCD of its own) computes the products of the connections between the
    layers in both directions, and the layers' programs poll its sums element by element."""
    monkeypatch.setenv("RNNG_CHAIN_HELPERS", helpers)
    spec = wl.lstm_net(12, layers, 5)
    win, _ = run_both(wl.make_workload("lstm_stack_wave_helpers", spec, T=19, N=N, seed=36, scale=0.3 if layers[0] < 100 else 0.06, bias_scale=0.3, masked_fraction=0.2),
                      label=f"stack {layers}, N={N}, RNNG_CHAIN_HELPERS={helpers}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b) == ("wave", True) for k in rec for b in (False, True))
    assert all(win.g.step_build_has_helpers(k, b) == (helpers == "1") for k in rec for b in (False, True))


@pytest.mark.parametrize("chain", ["1", "0"])
@pytest.mark.parametrize("N", [2, 24])
def test_stack_in_one_launch_and_layers_one_after_another(monkeypatch, chain, N):
    """Stacked layers in one step launch (the connections between them stepped) and one launch per
    layer (those connections batched over frames, the paper's schedule), each against the oracle."""
    monkeypatch.setenv("RNNG_CHAIN", chain)
    spec = wl.lstm_net(10, [32, 28], 6)
    w = wl.make_workload("stack", spec, T=13, N=N, seed=32, scale=0.4, bias_scale=0.3)
    win, _ = run_both(w, label=f"stack N={N} RNNG_CHAIN={chain}")
    for name in ("L1.h", "L2.h"):
        for backward in (False, True):
            build, chained = win.g.step_build(spec.node_by_name(name), backward)
            assert build == ("wave" if N <= 8 else "matrix") and chained == (chain == "1")


def test_interpreting_build_of_the_step_kernel(monkeypatch):
    """RNNG_JIT=0: the ahead-of-time build that interprets the step programs (it serves N <= 8;
    more streams step with per-frame launches), single- and multi-phase components."""
    monkeypatch.setenv("RNNG_JIT", "0")
    spec = wl.lstm_net(12, [40, 24], 5)
    win, _ = run_both(wl.make_workload("lstm2_interp", spec, T=17, N=3, seed=61, scale=0.4, bias_scale=0.3, masked_fraction=0.2), label="RNNG_JIT=0 stack")
    assert win.g.step_build(spec.node_by_name("L1.h")) == ("interpreted", False)
    assert win.g.step_build(spec.node_by_name("L2.c"), True) == ("interpreted", False)
    spec = wl.generalized_net(8, 16, 2, 4)
    run_both(wl.make_workload("gen_interp", spec, T=9, N=1, seed=62, scale=0.4, bias_scale=0.3), label="RNNG_JIT=0 generalized")
    spec = wl.lstm_net(6, [20], 4)
    win, _ = run_both(wl.make_workload("lstm_frames", spec, T=7, N=12, seed=63, scale=0.4, bias_scale=0.3), label="RNNG_JIT=0 N=12")
    assert win.g.step_build(spec.node_by_name("L1.h")) == ("per_frame", False)


def test_without_exchange_bundles(monkeypatch):
    """RNNG_BUNDLE=0: every exchanged tensor polled on its own (no interleaved bundle tensors)."""
    monkeypatch.setenv("RNNG_BUNDLE", "0")
    spec = wl.lstm_net(12, [40, 24], 5)
    win, _ = run_both(wl.make_workload("lstm2_nobundle", spec, T=17, N=2, seed=64, scale=0.4, bias_scale=0.3, masked_fraction=0.2), label="RNNG_BUNDLE=0")
    assert win.g.step_build(spec.node_by_name("L1.h"), True) == ("wave", True)


def test_target_index_out_of_range_is_reported():
    from paper_1503_02852_amd.binding import RnnError
    from paper_1503_02852_amd.runner import window_for
    w = wl.make_workload("badtarget", wl.lstm_net(5, [8], 3), T=6, N=2, seed=65)
    (out,) = w.spec.output_nodes()
    w.targets[out][2, 1] = 3          # classes are 0..2
    win = window_for(w)
    win.forward(); win.bptt()
    with pytest.raises(RnnError) as ei:
        win.compute_grads(want_loss=True)
    assert ei.value.code == -1
    with pytest.raises(RnnError):
        win.check()
    # the flag belongs to that window: the next one starts clean
    w.targets[out][2, 1] = -1
    win.set_targets(w.targets)
    win.forward(); win.bptt(); win.compute_grads(want_loss=True); win.check()
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    gw, _ = win.grads_unpacked()
    for m, g in enumerate(ref["grad_w"]):
        if g is not None:
            assert nerr(gw[m], g) < GRAD_TOL


@pytest.mark.parametrize("helpers,N", [(None, 1), ("1", 1), ("1", 32)])
def test_a_wait_that_runs_into_its_limit_is_reported_on_every_path(monkeypatch, helpers, N):
    """RNNG_SPIN_LIMIT=1 makes every bounded wait of the step kernels give up after one repeat: the
    kernels then stop waiting, run to their end and raise the error word.  rnn_check must report
    it after a forward pass alone and after rnn_grads without a loss pointer; a window in which no
    wait happened to expire must be correct.  Also with helper members in the launches (their sums
    are waited for like every exchanged value), weights in registers and matrix cores."""
    from paper_1503_02852_amd.binding import RnnError
    from paper_1503_02852_amd.runner import window_for
    monkeypatch.setenv("RNNG_SPIN_LIMIT", "1")
    if helpers is not None:
        monkeypatch.setenv("RNNG_CHAIN_HELPERS", helpers)
    w = wl.make_workload("spin", wl.lstm_net(8, [64, 64], 4), T=200 if N == 1 else 60, N=N, seed=66, scale=0.3)
    win = window_for(w)
    win.forward()
    flagged = False
    try:
        win.check()
    except RnnError as e:
        assert e.code == -5
        flagged = True
    win.bptt(); win.compute_grads(False)
    try:
        win.check()
        assert not flagged      # a flag raised by the forward pass stays up for the whole window
    except RnnError as e:
        assert e.code == -5
        flagged = True
    print(f"[parity] spin limit 1: flagged = {flagged}", flush=True)
    if not flagged:
        ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
        gw, _ = win.grads_unpacked()
        for m, g in enumerate(ref["grad_w"]):
            if g is not None:
                assert nerr(gw[m], g) < GRAD_TOL


@pytest.mark.parametrize("kind,N", [("elman", 16), ("lstm", 24), ("lstm", 40), ("elman", 64)])
def test_wide_layers_with_the_two_dimensional_split(monkeypatch, kind, N):
    """1024-wide recurrent layers at many streams with the matrix-core kernel's two-dimensional
    split forced for both directions: 4 and 16 rows per workgroup, 1 to 4 stream tiles (3 tiles take
    the other assignment of tiles to wavefronts), a window computed in two pieces."""
    from paper_1503_02852_amd.runner import window_for
    monkeypatch.setenv("RNNG_MSTEP_2D", "1")
    spec = wl.elman_net(12, 1024, 6) if kind == "elman" else wl.lstm_net(12, [1024], 6)
    w = wl.make_workload(f"wide_{kind}", spec, T=5, N=N, seed=41, scale=0.05, bias_scale=0.1, masked_fraction=0.2)
    win, ref = run_both(w, label=f"2-D split, {kind}, N={N}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b) == ("matrix_2d", False) for k in rec for b in (False, True))
    win2 = window_for(w)
    win2.forward_range(0, 2); win2.forward_range(2, 5)
    win2.bptt(); win2.compute_grads()
    for k in w.spec.output_nodes():
        assert nerr(win2.node_output(k), ref["y"][k]) < OUT_TOL


@pytest.mark.parametrize("kind,N", [("elman", 16), ("lstm", 16), ("lstm", 24), ("lstm", 64), ("elman", 48)])
def test_wide_layers_with_weight_rows_in_registers(kind, N):
    """1024-wide recurrent layers at many streams with the one-dimensional split: the weight rows
    of a workgroup exceed LDS, so whole sources stay in vector registers.  Stream counts that are
    multiples of 16 exchange through the tile-blocked twins (one and several stream groups), the
    others through the row-major tensors; a window computed in two pieces."""
    from paper_1503_02852_amd.runner import window_for
    spec = wl.elman_net(12, 1024, 6) if kind == "elman" else wl.lstm_net(12, [1024], 6)
    w = wl.make_workload(f"wide_{kind}", spec, T=5, N=N, seed=43, scale=0.05, bias_scale=0.1, masked_fraction=0.2)
    win, ref = run_both(w, label=f"weights in registers, {kind}, N={N}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    # (a backward loop that cannot fill a 16-row tile per workgroup may take the two-dimensional split)
    assert rec and all(win.g.step_build(k, False) == ("matrix", False) for k in rec)
    assert N % 16 or all(win.g.step_build(k, True) == ("matrix", False) for k in rec)
    win2 = window_for(w)
    win2.forward_range(0, 2); win2.forward_range(2, 5)
    win2.bptt(); win2.compute_grads()
    for k in w.spec.output_nodes():
        assert nerr(win2.node_output(k), ref["y"][k]) < OUT_TOL


MANY_STREAM_NETS = {
    "elman_1024_n16": lambda: (wl.elman_net(12, 1024, 6), 16, 0.05),
    "lstm_1024_n64": lambda: (wl.lstm_net(12, [1024], 6), 64, 0.05),
    "lstm_stack_n32": lambda: (wl.lstm_net(12, [256, 128, 256], 6), 32, 0.15),
    "generalized_n48": lambda: (wl.generalized_net(8, 128, 3, 4), 48, 0.2),
    "elman_2048_n16": lambda: (wl.elman_net(12, 2048, 6), 16, 0.03),
}


@pytest.mark.parametrize("name", sorted(MANY_STREAM_NETS))
def test_many_stream_layers_of_several_widths(name):
    """Matrix-core step kernels at stream counts that are multiples of 16 (exchange through the
    tile-blocked twins): single wide layers with weight rows in registers, a stack of three layers
    of different widths in one launch, delay-2 connections, three to four stream groups."""
    spec, N, scale = MANY_STREAM_NETS[name]()
    w = wl.make_workload(name, spec, T=13, N=N, seed=61, scale=scale, bias_scale=0.1, masked_fraction=0.2)
    win, ref = run_both(w, label=f"many streams, {name}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b)[0] in ("matrix", "matrix_2d") for k in rec for b in (False, True))


@pytest.mark.parametrize("env", [{"RNNG_MSTEP_BLOCKED": "0"}, {"RNNG_MSTEP_WAVES": "4"}, {"RNNG_MSTEP_WAVES": "4", "RNNG_MSTEP_BLOCKED": "0"},
                                 {"RNNG_MSTEP_REGS": "0"}, {"RNNG_MSTEP_FLAT_MAX": "1"}, {"RNNG_MSTEP_FLAT_MAX": "1", "RNNG_MSTEP_WAVES": "4"}])
def test_matrix_core_kernel_switches(monkeypatch, env):
    """The matrix-core step kernel with four wavefronts, with the exchange through the row-major
    tensors at a stream count that would allow the tile-blocked twins, without weight rows in
    registers, and with the chunk sequence run source by source in groups (as for very long
    sequences) instead of unrolled: a stack (one launch for both layers) and a single layer with a
    delay-2 connection."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    run_both(wl.make_workload("stack", wl.lstm_net(12, [64, 48], 5), T=9, N=32, seed=51, scale=0.3, bias_scale=0.2, masked_fraction=0.2),
             label=f"stack, {env}")
    run_both(wl.make_workload("gen", wl.generalized_net(8, 64, 2, 4), T=7, N=16, seed=52, scale=0.3, bias_scale=0.2), label=f"generalized, {env}")


@pytest.mark.parametrize("local", ["0", "1"])
def test_exchange_written_through_and_through_the_xcd_cache(monkeypatch, local):
    """Both forms of the exchange inside a group of workgroups (plain stores served by the XCD's
    L2, or every exchanged tensor written through) on a stack (values that another group polls are
    written through one step late) and on a single recurrent layer."""
    monkeypatch.setenv("RNNG_XCD_LOCAL", local)
    run_both(wl.make_workload("lstm3", wl.lstm_net(12, [20, 24, 16], 5), T=23, N=2, seed=22, scale=0.4, bias_scale=0.3, masked_fraction=0.2),
             label=f"stack, RNNG_XCD_LOCAL={local}")
    run_both(wl.make_workload("lstm1", wl.lstm_net(9, [40], 6), T=17, N=1, seed=23, scale=0.4, bias_scale=0.3), label=f"layer, RNNG_XCD_LOCAL={local}")
    run_both(wl.make_workload("elman", wl.elman_net(7, 33, 4), T=12, N=3, seed=24, scale=0.4, bias_scale=0.3), label=f"elman, RNNG_XCD_LOCAL={local}")


@pytest.mark.parametrize("window", ["0", "1"])
@pytest.mark.parametrize("early", ["0", "1"])
def test_store_descriptors_and_poll_placement(monkeypatch, window, early):
    """The wave-autonomous kernels with one buffer descriptor over the workspace or one per stored
    tensor, with a step's first polling attempt issued at its start or behind the stores of the
    step before, and with the stores nobody polls early or one step late, in all four pairings
    (also with wavefronts that own no units: 33 units on 32 workgroups)."""
    monkeypatch.setenv("RNNG_STORE_WINDOW", window)
    monkeypatch.setenv("RNNG_WAVE_POLL_EARLY", early)
    monkeypatch.setenv("RNNG_WAVE_EARLY_STORES", early if window == "1" else str(1 - int(early)))
    tag = f"RNNG_STORE_WINDOW={window} RNNG_WAVE_POLL_EARLY={early}"
    run_both(wl.make_workload("lstm2", wl.lstm_net(12, [64, 48], 5), T=19, N=2, seed=31, scale=0.4, bias_scale=0.3, masked_fraction=0.2), label="stack, " + tag)
    run_both(wl.make_workload("lstm1", wl.lstm_net(9, [512], 6), T=9, N=1, seed=32, scale=0.2, bias_scale=0.3), label="wide layer, " + tag)
    run_both(wl.make_workload("elman", wl.elman_net(7, 33, 4), T=12, N=3, seed=33, scale=0.4, bias_scale=0.3), label="elman, " + tag)


def test_stacked_elman_layers_with_delayed_link():
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 9, name="x")
    h1 = g.add_node(wl.ADD, wl.TANH, 37, has_bias=True, name="h1")
    h2 = g.add_node(wl.ADD, wl.SIGMOID, 22, has_bias=True, name="h2")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 6, has_bias=True, is_output=True, name="out")
    g.add_edge(x, h1, wl.FULL, 0); g.add_edge(h1, h1, wl.FULL, 1)
    g.add_edge(h1, h2, wl.FULL, 0); g.add_edge(h1, h2, wl.FULL, 2)      # the link between the layers, also delayed
    g.add_edge(h2, h2, wl.FULL, 1); g.add_edge(h2, h2, wl.FULL, 3)
    g.add_edge(h2, out, wl.FULL, 0); g.add_edge(h1, out, wl.FULL, 1)    # the lower layer also feeds the output
    run_both(wl.make_workload("elman2", g, T=23, N=3, seed=22, scale=0.3, bias_scale=0.2))


def test_lstm_stack_with_skip_connection_from_the_input():
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 10, name="x")
    l1 = wl.add_lstm_layer(g, x, 18, "L1")
    l2 = wl.add_lstm_layer(g, l1["h"], 18, "L2")
    g.add_edge(x, l2["g"], wl.FULL, 1)               # a batched edge into the upper layer from outside the stack
    g.add_edge(l1["h"], l2["i"], wl.FULL, 2)         # a second, delayed link between the layers
    out = g.add_node(wl.ADD, wl.SOFTMAX, 4, has_bias=True, is_output=True, name="out")
    g.add_edge(l2["h"], out, wl.FULL, 0)
    run_both(wl.make_workload("lstm_skip", g, T=17, N=1, seed=23, scale=0.4, bias_scale=0.3))


def test_lstm_stack_single_frame_and_two_frames():
    spec = wl.lstm_net(6, [10, 12], 3)
    run_both(wl.make_workload("lstm2_T1", spec, T=1, N=2, seed=24, scale=0.5))
    run_both(wl.make_workload("lstm2_T2", spec, T=2, N=1, seed=25, scale=0.5))


# ---- the paper's own Section 4 network shapes (38,000-word one-hot input, 20,000-way softmax) ----

@pytest.mark.parametrize("name", ["lm_elman_n1", "lm_lstm_n1"])
def test_language_model_shapes_short_window(name):
    run_both(wl.make_config(name, T=24, N=2), check_all_nodes=True, label=name)


# ---- output layers with dense targets under the squared error (Section 2.2: the output delta follows the error criterion) ----

@pytest.mark.parametrize("act", [wl.LINEAR, wl.SIGMOID, wl.TANH, wl.RELU])
def test_squared_error_output_layer(act):
    spec = wl.lstm_net(12, [40, 24], 7, squared_error_act=act)
    run_both(wl.make_workload("lstm_sq", spec, T=21, N=3, seed=80 + act, scale=0.4, bias_scale=0.3, masked_fraction=0.25), label=f"squared error, act {act}")


@pytest.mark.parametrize("seed", range(4))
def test_random_graphs_with_mixed_output_criteria(seed):
    rng = np.random.default_rng(800 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, n_inputs=1 + seed % 2, squared_error_outputs=1 + seed % 2)
    run_both(wl.make_workload(f"rand_sq{seed}", spec, T=9 + seed, N=1 + 5 * (seed % 3), seed=seed, scale=0.8, bias_scale=0.5, masked_fraction=0.2))


def test_squared_error_many_streams_full_width_frame():
    """A regression-shaped net at many streams: 256-wide LSTM, 130-wide linear output, N = 40."""
    spec = wl.lstm_net(20, [256], 130, squared_error_act=wl.LINEAR)
    run_both(wl.make_workload("lstm_sq_n40", spec, T=12, N=40, seed=84, scale=0.1, bias_scale=0.1), label="squared error, N = 40")


# ---- Section 4, second experiment (Fig. 4): LSTM nets whose input, LSTM and output layers are equally wide ----

@pytest.mark.parametrize("H,N,T", [(1024, 1, 6), (1024, 16, 5), (1024, 64, 4), (2048, 1, 6), (2048, 16, 4), (2048, 64, 3),
                                   (4096, 1, 5), (4096, 16, 3), (4096, 64, 3)])
def test_fig4_shapes_short_window(H, N, T):
    """Full widths and stream counts over a short window (the full windows have 2,048 / N frames).
    At 2,048 units and one stream (or 16) a layer's recurrent weights still fit on chip, 256 KiB
    per workgroup; at 64 streams, and from 4,096 units on, the step kernel streams them from memory
    every step."""
    w = wl.make_config(f"fig4_h{H}_n{N}", T=T)
    win, _ = run_both(w, check_all_nodes=True, label=f"fig4_h{H}_n{N}_T{T}")
    print(f"[parity] fig4_h{H}_n{N}: forward build {win.g.step_build(w.spec.node_by_name('L1.h'))}, "
          f"backward build {win.g.step_build(w.spec.node_by_name('L1.h'), True)}", flush=True)


LONG_ROW_NETS = {
    "lstm_1280_n1": (lambda: wl.lstm_net(20, [1280], 8), 7, 1),       # 20 elements per lane, bundled gate deltas of 5,120 words
    "lstm_2048_n2": (lambda: wl.lstm_net(12, [2048], 8), 5, 2),       # forward in registers at 2 streams, backward streamed
    "elman_1800_n3": (lambda: wl.elman_net(9, 1800, 6), 8, 3),        # 29 elements per lane (ragged: 1,800 = 62 * 29 + 2)
    "elman_1999_n1": (lambda: wl.elman_net(9, 1999, 6), 8, 1),        # odd width: polled word by word
}


@pytest.mark.parametrize("name", sorted(LONG_ROW_NETS))
def test_register_build_with_long_weight_rows(name):
    """The weights-in-registers build with rows of 1,025 to 2,048 elements (17 to 32 per lane),
    at widths that are no multiple of 64, odd, and at more than one stream."""
    make, T, N = LONG_ROW_NETS[name]
    w = wl.make_workload(name, make(), T=T, N=N, seed=77, scale=0.04, bias_scale=0.3, masked_fraction=0.1)
    win, ref = run_both(w, label=f"long rows, {name}")
    rec = [k for k in range(len(w.spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, False)[0] == "wave" for k in rec)


def test_a_2048_wide_layer_at_four_streams_streams_its_weights():
    """At four streams the weights, source values and partial sums of a 2,048-wide LSTM layer no
    longer fit a lane's registers: both directions take the streaming build."""
    w = wl.make_workload("lstm_2048_n4", wl.lstm_net(12, [2048], 8), T=5, N=4, seed=78, scale=0.04, bias_scale=0.3)
    win, ref = run_both(w, label="2,048-wide layer, N=4")
    rec = [k for k in range(len(w.spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b)[0] == "streaming" for k in rec for b in (False, True))


# ---- the streaming step kernel (weights read from memory every step) on small and ragged shapes ----

@pytest.mark.parametrize("case", ["lstm_n1", "lstm_n3_ragged", "elman_n8", "generalized_n2", "stack_n1", "gates_n5",
                                  "lstm_n12", "lstm_n40_ragged", "elman_n33", "generalized_n20", "stack_n16", "wide_units_n70"])
def test_streaming_step_kernel_on_small_shapes(monkeypatch, case):
    """RNNG_STEP_BUILD=stream makes the streaming variant take shapes the register / LDS variants
    would serve: widths that are no multiples of 256 or 64 (ragged last chunk), of the 4 wavefronts'
    share or of the workgroup count, several sources per task, 1 to 8 streams (vector arithmetic)
    and more (matrix cores), both directions (the backward one reads transposed copies), a window
    computed in two pieces."""
    from paper_1503_02852_amd.runner import window_for
    monkeypatch.setenv("RNNG_STEP_BUILD", "stream")
    spec, T, N = {
        "lstm_n1": (wl.lstm_net(12, [512], 6), 9, 1),
        "lstm_n3_ragged": (wl.lstm_net(9, [300], 5), 7, 3),
        "elman_n8": (wl.elman_net(7, 1100, 4), 6, 8),
        "generalized_n2": (wl.generalized_net(8, 260, 2, 4), 8, 2),
        "stack_n1": (wl.lstm_net(10, [768, 520], 6), 7, 1),
        "gates_n5": (wl.lstm_net(6, [64], 4), 11, 5),
        # more than 8 streams: the matrix-core form of the streaming variant
        "lstm_n12": (wl.lstm_net(12, [512], 6), 6, 12),
        "lstm_n40_ragged": (wl.lstm_net(9, [300], 5), 5, 40),
        "elman_n33": (wl.elman_net(7, 1100, 4), 5, 33),
        "generalized_n20": (wl.generalized_net(8, 260, 2, 4), 6, 20),
        "stack_n16": (wl.lstm_net(10, [768, 520], 6), 5, 16),
        "wide_units_n70": (wl.lstm_net(6, [1536], 4), 4, 70),      # 6 units per workgroup x 70 streams: two element-wise passes
    }[case]
    w = wl.make_workload(case, spec, T=T, N=N, seed=90, scale=0.05 if max(n["dim"] for n in spec.nodes) > 400 else 0.2, bias_scale=0.2, masked_fraction=0.2)
    win, ref = run_both(w, label=f"streaming {case}")
    rec = [k for k in range(len(spec.nodes)) if win.g.step_build(k)[0] != "none"]
    assert rec and all(win.g.step_build(k, b) == ("streaming", False) for k in rec for b in (False, True))
    win2 = window_for(w)
    win2.forward_range(0, 3); win2.forward_range(3, T)
    win2.bptt(); win2.compute_grads(); win2.check()
    for k in spec.output_nodes():
        assert nerr(win2.node_output(k), ref["y"][k]) < OUT_TOL


def test_deterministic_gradient_sums():
    """rnn_set_deterministic: the gradients of two runs agree to the last bit (one writer per element,
    no atomic splits of the sums over frames) and still match the oracle; with class-index inputs
    the scatter-add runs in frame order."""
    from paper_1503_02852_amd.runner import window_for
    w = wl.make_workload("det", wl.lstm_net(30, [96, 64], 30), T=300, N=3, seed=95, scale=0.3, bias_scale=0.2)
    runs = []
    for _ in range(2):
        win = window_for(w)
        win.g.set_deterministic(True)
        win.forward(); win.bptt(); win.compute_grads(); win.check()
        runs.append(win.grads.cpu().numpy().copy())
    assert np.array_equal(runs[0], runs[1])
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    gw, gb = win.grads_unpacked()
    for m, g in enumerate(ref["grad_w"]):
        if g is not None:
            assert nerr(gw[m], g) < GRAD_TOL
    # one-hot input given as indices: ordered scatter-add
    c = wl.make_config("charlm_n1", T=200)
    idx = {k: x.argmax(axis=2) for k, x in c.inputs.items()}
    runs = []
    for _ in range(2):
        win = window_for(c)
        win.set_onehot_inputs(idx)
        win.g.set_deterministic(True)
        win.forward(); win.bptt(); win.compute_grads(); win.check()
        runs.append(win.grads.cpu().numpy().copy())
    assert np.array_equal(runs[0], runs[1])
    ref = go.forward_bptt(c.spec.nodes, c.spec.edges, c.weights, c.biases, c.inputs, c.targets, c.T, c.N)
    gw, gb = win.grads_unpacked()
    for m, g in enumerate(ref["grad_w"]):
        if g is not None:
            assert nerr(gw[m], g) < GRAD_TOL
