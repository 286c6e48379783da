"""CPU-only tests of the C-ABI library's host side: exported symbols, the analyser's schedule
(bit-exact against the brute-force oracle), parameter layout, and error handling.  No GPU
compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import schedule_oracle as so
from paper_1503_02852_amd import AUX_EXPORTS, EXPORTS, LIB_PATH, Graph, RnnError, load_library

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = load_library()
    for header_name, names in (("rnngraph.h", EXPORTS), ("rnngraph_aux.h", AUX_EXPORTS)):
        header = open(os.path.join(ROOT, "include", header_name)).read()
        declared = set(re.findall(r"^(?:int|int64_t|void|const char\*)\s+(rnn_[a-z_]+)\s*\(", header, flags=re.M))
        assert declared == set(names), header_name
        for name in declared:
            assert hasattr(lib, name), name
    assert os.path.exists(LIB_PATH)


def schedules_equal(spec):
    g = Graph(spec.node_array(), spec.edge_array())
    return g.schedule(), so.schedule(spec.nodes, spec.edges)


@pytest.mark.parametrize("builder", [
    lambda: wl.lstm_net(8, [16], 4), lambda: wl.lstm_net(8, [16], 4, output_recurrence=False),
    lambda: wl.lstm_net(40, [256, 256], 61), lambda: wl.generalized_net(), lambda: wl.elman_net(5, 7, 3)])
def test_schedule_matches_oracle_on_named_nets(builder):
    got, exp = schedules_equal(builder())
    assert got == exp


@pytest.mark.parametrize("seed", range(40))
def test_schedule_matches_oracle_on_random_graphs(seed):
    rng = np.random.default_rng(1000 + seed)
    spec = wl.random_graph(rng, n_inner=3 + seed % 9, p_edge=0.15 + 0.05 * (seed % 6), max_delay=3, n_inputs=1 + seed % 2)
    got, exp = schedules_equal(spec)
    assert got == exp
    # relabelled copy too
    spec2 = spec.permuted(rng.permutation(len(spec.nodes)), rng.permutation(len(spec.edges)))
    got2, exp2 = schedules_equal(spec2)
    assert got2 == exp2


def test_param_layout_is_disjoint_and_complete():
    spec = wl.generalized_net(6, 8, 2, 5)
    g = Graph(spec.node_array(), spec.edge_array())
    total = g.param_count()
    used = np.zeros(total, dtype=np.int32)
    for m, e in enumerate(spec.edges):
        off, ln = g.edge_param(m)
        exp = {wl.FULL: spec.nodes[e["dst"]]["dim"] * spec.nodes[e["src"]]["dim"], wl.DIAG: spec.nodes[e["dst"]]["dim"], wl.IDENTITY: 0}[e["wkind"]]
        assert ln == exp
        used[off:off + ln] += 1
    for k, n in enumerate(spec.nodes):
        off, ln = g.bias_param(k)
        assert ln == (n["dim"] if n["has_bias"] else 0)
        used[off:off + ln] += 1
    assert used.max() == 1
    w = wl.make_workload("g", spec, 2, 1, seed=0)
    assert used.sum() == w.n_params()
    flat = g.pack_params(w.weights, w.biases)
    ws, bs = g.unpack_params(flat)
    for a, b in zip(ws + bs, w.weights + w.biases):
        assert (a is None) == (b is None)
        if a is not None:
            assert np.array_equal(a, b)


def bad(nodes, edges):
    with pytest.raises(RnnError) as ei:
        Graph(np.array(nodes, np.int32), np.array(edges, np.int32).reshape(-1, 4))
    assert ei.value.code == -2
    return str(ei.value)


def test_invalid_graphs_are_rejected():
    X = [wl.INPUT, wl.LINEAR, 3, 0, 0]
    H = [wl.ADD, wl.TANH, 3, 1, 0]
    O = [wl.ADD, wl.SOFTMAX, 2, 1, 1]
    ok_edges = [[0, 1, 0, wl.FULL], [1, 2, 0, wl.FULL]]
    Graph(np.array([X, H, O], np.int32), np.array(ok_edges, np.int32))
    assert "cycle" in bad([X, H, H, O], [[0, 1, 0, 0], [1, 2, 0, 0], [2, 1, 0, 0], [2, 3, 0, 0]])
    assert "cycle" in bad([X, H, O], ok_edges + [[1, 1, 0, wl.FULL]])          # delay-0 self-loop
    bad([X, H, O], [[0, 1, 0, 0], [1, 5, 0, 0]])                                # node id out of range
    bad([X, [wl.ADD, wl.TANH, 0, 0, 0], O], ok_edges)                           # dim 0
    bad([X, [wl.ADD, wl.TANH, 4, 0, 0], O], [[0, 1, 0, wl.IDENTITY], [1, 2, 0, 0]])   # identity across widths
    bad([X, H, O], [[0, 1, -1, 0], [1, 2, 0, 0]])                               # negative delay
    bad([X, H, O], ok_edges + [[1, 0, 1, 0]])                                   # edge into an input
    bad([X, H, H, O], ok_edges[:1] + [[1, 3, 0, 0]])                            # node 2 without in-edge
    bad([X, [wl.ADD, wl.SOFTMAX, 3, 0, 0], O], ok_edges)                        # softmax on a hidden node
    bad([X, H, [wl.ADD, wl.TANH, 2, 1, 1]], ok_edges)                           # output that is not softmax
    bad([X, H, O, H], ok_edges + [[2, 3, 0, 0]])                                # edge leaving an output
    bad([X, [wl.MUL, wl.LINEAR, 3, 1, 0], O], [[0, 1, 0, 2], [1, 2, 0, 0]])     # bias on a multiplicative node
    bad([X, H], [[0, 1, 0, 0]])                                                 # no output node
    bad([X, [7, 0, 3, 0, 0], O], ok_edges)                                      # unknown kind
    bad([X, H, [wl.ADD, wl.SOFTMAX, 2, 1, 2]], ok_edges)                        # squared-error output with softmax
    bad([X, H, [wl.MUL, wl.LINEAR, 3, 0, 2]], [[0, 1, 0, 0], [1, 2, 0, 2]])     # squared-error output that is multiplicative
    bad([X, H, [wl.ADD, wl.TANH, 2, 1, 3]], ok_edges)                           # unknown output kind
    Graph(np.array([X, H, [wl.ADD, wl.TANH, 2, 1, 2]], np.int32), np.array(ok_edges, np.int32))      # a valid squared-error output
    assert "activation" in bad([X, [wl.ADD, 5, 3, 1, 0], O], ok_edges)          # unknown activation
    bad([X, [wl.MAX, wl.LINEAR, 3, 1, 0], O], [[0, 1, 0, 2], [1, 2, 0, 0]])     # bias on a maximum node
    Graph(np.array([X, [wl.MAX, wl.TANH, 3, 0, 0], O], np.int32), np.array([[0, 1, 0, 2], [0, 1, 1, 1], [1, 2, 0, 0]], np.int32))   # a maximum node
    bad([X, H, [wl.ADD, wl.RELU, 2, 1, 1]], ok_edges)                           # cross-entropy output with a rectifier
    Graph(np.array([X, [wl.ADD, wl.RELU, 3, 1, 0], [wl.ADD, wl.RELU, 2, 1, 2]], np.int32), np.array(ok_edges, np.int32))   # rectified hidden and squared-error layers


def test_runtime_argument_errors_without_gpu_work():
    spec = wl.lstm_net(4, [5], 3)
    g = Graph(spec.node_array(), spec.edge_array())
    with pytest.raises(RnnError) as ei:
        g.workspace_bytes(0, 1)
    assert ei.value.code == -1
    with pytest.raises(RnnError) as ei:
        g.bptt(1, [1])
    assert ei.value.code == -4          # bptt before forward
    with pytest.raises(RnnError) as ei:
        g.grads(1)
    assert ei.value.code == -4
    with pytest.raises(RnnError) as ei:
        g.forward(1, [1], 4, 1, None, 1 << 30)
    assert ei.value.code == -3          # NULL workspace
    with pytest.raises(RnnError) as ei:
        g.forward(1, [1], 4, 1, 256, 16)
    assert ei.value.code == -3          # too small
    with pytest.raises(RnnError) as ei:
        g.forward(1, [1], 4, 1, 257, 1 << 30)
    assert ei.value.code == -3          # misaligned
    with pytest.raises(RnnError) as ei:
        g.forward(None, [1], 4, 1, 256, 1 << 30)
    assert ei.value.code == -1
    assert g.workspace_bytes(4, 1) > 0


def test_stacked_layers_get_a_side_by_side_step_kernel(monkeypatch):
    """Two stacked LSTM layers form a chain: besides one step kernel per layer and direction the
    run-time compiler builds one kernel per direction that runs both layers in one launch."""
    import workloads as wl
    from paper_1503_02852_amd import binding
    spec = wl.lstm_net(8, [16, 16], 4)
    monkeypatch.setenv("RNNG_CHAIN", "0")
    g0 = binding.Graph(spec.node_array(), spec.edge_array())
    n_plain = g0.specialise(1)
    monkeypatch.setenv("RNNG_CHAIN", "1")
    g1 = binding.Graph(spec.node_array(), spec.edge_array())
    n_all = g1.specialise(1)
    if n_plain == 0:
        pytest.skip("run-time compiler not available")
    assert n_plain == 4 and n_all == 6
    # a layer pair linked through a non-recurrent node is not a chain
    spec5 = wl.generalized_net(8, 16, 2, 4)
    g2 = binding.Graph(spec5.node_array(), spec5.edge_array())
    assert g2.specialise(1) == 4


@pytest.mark.parametrize("early,window", [("1", "1"), ("0", "0")])
def test_step_kernel_variants_compile(monkeypatch, early, window):
    """The generated step kernels compile for gfx950 in both placements of the stores nobody polls
    and of a step's first polling attempt, with one store window and with one descriptor per
    stored tensor (a stack, and an Elman layer whose 33 units leave wavefronts without units)."""
    import workloads as wl
    from paper_1503_02852_amd import binding
    monkeypatch.setenv("RNNG_WAVE_POLL_EARLY", early)
    monkeypatch.setenv("RNNG_WAVE_EARLY_STORES", early)
    monkeypatch.setenv("RNNG_JIT_DEFINES", f"-DRNNG_STORE_WINDOW={window}")
    spec = wl.lstm_net(8, [16, 16], 4)
    g = binding.Graph(spec.node_array(), spec.edge_array())
    n = g.specialise(1)
    if n == 0:
        pytest.skip("run-time compiler not available")
    assert n == 6
    spec2 = wl.elman_net(7, 33, 4)
    g2 = binding.Graph(spec2.node_array(), spec2.edge_array())
    assert g2.specialise(3) == 2


@pytest.mark.parametrize("H,N", [(4096, 1), (2048, 64), (4096, 16), (4096, 64)])
def test_wide_layers_get_a_streaming_step_kernel(H, N):
    """Section 4's second experiment (all layers 4,096 wide, or 2,048 wide at many streams): the
    recurrent weights fit neither registers nor LDS, so both directions must be served by the streaming build (one
    kernel per direction compiles for gfx950) and the backward one needs the transposed copy of
    the parameter buffer in the workspace."""
    import workloads as wl
    from paper_1503_02852_amd import binding
    spec = wl.lstm_net(H, [H], H)
    g = binding.Graph(spec.node_array(), spec.edge_array())
    n = g.specialise(N)
    if n == 0:
        pytest.skip("run-time compiler not available")
    assert n == 2
    # room for the transposed copy of the parameter buffer
    assert g.workspace_bytes(8, N) > 4 * g.param_count()


@pytest.mark.parametrize("N", [1, 16])
def test_a_2048_wide_layer_keeps_its_weights_on_chip(N):
    """All layers 2,048 wide: 256 workgroups hold the 64 MiB of recurrent weights on chip, 256 KiB
    each (at one stream in registers alone, at 16 streams in registers and LDS), so no transposed
    copy of the parameters is needed."""
    import workloads as wl
    from paper_1503_02852_amd import binding
    spec = wl.lstm_net(2048, [2048], 2048)
    g = binding.Graph(spec.node_array(), spec.edge_array())
    if g.specialise(N) == 0:
        pytest.skip("run-time compiler not available")
    assert g.workspace_bytes(8, N) < 4 * g.param_count()


def test_headers_are_plain_c(tmp_path):
    """The boundary is a C ABI: both headers must compile as C (no C++ in the signatures)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "t.c"
    src.write_text('#include "rnngraph.h"\n#include "rnngraph_aux.h"\nint main(void) { return rnn_last_error() == 0; }\n')
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-I", os.path.join(ROOT, "include"), str(src)], check=True)
