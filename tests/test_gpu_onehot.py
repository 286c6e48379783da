"""GPU parity for one-hot input layers given as class indices (the word input of Section 4): the
full connections leaving such a layer run as column gathers and scatter-adds.  The float64 oracle
gets the same frames as dense one-hot vectors.  Bars as in test_gpu_parity.py."""
import numpy as np
import pytest

import workloads as wl
from oracle import graph_oracle as go
from tests.test_gpu_parity import GRAD_TOL, OUT_TOL, nerr
from tests.test_gpu_window import check_against

pytestmark = pytest.mark.gpu


def two_input_net(V=37, n_dense=6, D=14, n_out=5):
    """A one-hot layer x that reaches the hidden layer now and one frame late, and a second hidden
    layer that sums a dense input and the one-hot layer (gather on top of a GEMM's result)."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, V, name="x")
    u = g.add_node(wl.INPUT, wl.LINEAR, n_dense, name="u")
    h = g.add_node(wl.ADD, wl.TANH, D, has_bias=True, name="h")
    k = g.add_node(wl.ADD, wl.SIGMOID, D, has_bias=True, name="k")
    g.add_edge(x, h, wl.FULL, 0); g.add_edge(x, h, wl.FULL, 1); g.add_edge(h, h, wl.FULL, 1)
    g.add_edge(u, k, wl.FULL, 0); g.add_edge(x, k, wl.FULL, 2); g.add_edge(h, k, wl.FULL, 0)
    out = g.add_node(wl.ADD, wl.SOFTMAX, n_out, has_bias=True, is_output=True, name="out")
    g.add_edge(k, out, wl.FULL, 0); g.add_edge(x, out, wl.FULL, 0)
    return g, x


def elman(V, D, Vo):
    g = wl.elman_net(V, D, Vo)
    return g, g.input_nodes()[0]


def lstm(V, D, Vo):
    g = wl.lstm_net(V, [D], Vo, output_recurrence=False)
    return g, g.input_nodes()[0]


NETS = {
    "elman_n3": lambda: elman(50, 24, 9) + (3,),
    "elman_wide_n1": lambda: elman(700, 40, 300) + (1,),
    "lstm_n2": lambda: lstm(40, 16, 7) + (2,),
    "two_inputs_n4": lambda: two_input_net() + (4,),
    "elman_n20": lambda: elman(33, 32, 6) + (20,),
}


def with_word_input(name, T, seed, empty_fraction=0.15):
    spec, x, N = NETS[name]()
    w = wl.make_workload(name, spec, T=T, N=N, seed=seed, scale=0.4, bias_scale=0.3, masked_fraction=0.2)
    rng = np.random.default_rng(seed + 1000)
    V = spec.nodes[x]["dim"]
    idx = rng.integers(0, V, size=(T, N)).astype(np.int32)
    idx[rng.random((T, N)) < empty_fraction] = -1
    dense = np.zeros((T, N, V), dtype=np.float32)
    tt, nn = np.nonzero(idx >= 0)
    dense[tt, nn, idx[tt, nn]] = 1.0
    w.inputs[x] = dense
    return w, x, idx


@pytest.mark.parametrize("name", sorted(NETS))
def test_index_input_matches_the_oracle_on_dense_one_hot_frames(name):
    from paper_1503_02852_amd.runner import window_for
    w, x, idx = with_word_input(name, T=21, seed=7)
    print(f"[onehot] {name}: T={w.T} N={w.N}", flush=True)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    win = window_for(w)
    win.set_onehot_inputs({x: idx})
    win.forward(); win.bptt()
    loss = win.compute_grads(want_loss=True)
    assert abs(loss - ref["loss"]) <= 1e-4 * max(1.0, abs(ref["loss"]))
    check_against(win, w, ref, name)


def test_index_input_with_a_window_computed_in_pieces_and_the_frame_by_frame_schedule(monkeypatch):
    from paper_1503_02852_amd.runner import window_for
    w, x, idx = with_word_input("two_inputs_n4", T=17, seed=3)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    win = window_for(w)
    win.set_onehot_inputs({x: idx})
    for t0, t1 in ((0, 1), (1, 9), (9, 17)):
        win.forward_range(t0, t1)
    win.bptt(); win.compute_grads()
    check_against(win, w, ref, "pieces")
    monkeypatch.setenv("RNNG_SCHEDULE", "framewise")
    win = window_for(w)
    win.set_onehot_inputs({x: idx})
    win.forward(); win.bptt(); win.compute_grads()
    check_against(win, w, ref, "framewise")


def test_dense_input_can_be_restored_and_non_full_connections_are_refused():
    import torch
    from paper_1503_02852_amd.binding import RnnError
    from paper_1503_02852_amd.runner import window_for
    w, x, idx = with_word_input("elman_n3", T=9, seed=5)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    win = window_for(w)
    dense = win.inputs[x]
    win.set_onehot_inputs({x: idx})
    win.forward()
    y_idx = [win.node_output(k).copy() for k in range(len(w.spec.nodes)) if w.spec.nodes[k]["kind"] != wl.INPUT]
    win.g.set_onehot_input(0, 0)
    win.inputs[x] = dense
    win.forward(); win.bptt(); win.compute_grads()
    check_against(win, w, ref, "dense again")
    y_dense = [win.node_output(k) for k in range(len(w.spec.nodes)) if w.spec.nodes[k]["kind"] != wl.INPUT]
    for a, b in zip(y_idx, y_dense):
        assert nerr(a, b) < OUT_TOL
    with pytest.raises(RnnError):
        win.g.set_onehot_input(5, win.onehot[x].data_ptr())
    # an input that feeds a node through a per-unit (diagonal) connection cannot be given as indices
    g = wl.GraphSpec()
    a = g.add_node(wl.INPUT, wl.LINEAR, 6, name="a")
    h = g.add_node(wl.ADD, wl.TANH, 6, name="h")
    g.add_edge(a, h, wl.DIAG, 0); g.add_edge(h, h, wl.FULL, 1)
    o = g.add_node(wl.ADD, wl.SOFTMAX, 3, is_output=True, name="o")
    g.add_edge(h, o, wl.FULL, 0)
    w2 = wl.make_workload("diag", g, T=4, N=1, seed=1)
    win2 = window_for(w2)
    with pytest.raises(RnnError):
        win2.g.set_onehot_input(0, torch.zeros(4, dtype=torch.int32, device="cuda:0").data_ptr())


def test_index_input_with_delayed_connections_in_a_carried_window():
    """A one-hot layer with delayed connections (delays 1 and 2), given as class indices, in a
    window that is moved ahead twice: the library keeps the indices of the history frames, so the
    forward pass and the truncated gradient see the real word of frame t - d before the window start."""
    import torch
    from paper_1503_02852_amd.runner import window_for
    from tests.test_gpu_window import mask_older_frames
    T, hp = 12, 6
    L = T + 2 * hp
    long, x, idx = with_word_input("two_inputs_n4", T=L, seed=11, empty_fraction=0.1)
    spec, N = long.spec, long.N
    y_long, z_long = go.forward(spec.nodes, spec.edges, long.weights, long.biases, long.inputs, L, N)
    first = wl.Workload(name="carry", spec=spec, T=T, N=N, weights=long.weights, biases=long.biases,
                        inputs={k: v[:T].copy() for k, v in long.inputs.items()}, targets={k: v[:T].copy() for k, v in long.targets.items()})
    win = window_for(first)
    win.set_onehot_inputs({x: idx[:T]})
    win.forward()
    for step in (1, 2):
        a, b = step * hp, step * hp + T
        win.g.shift_window(hp, win._stream())
        # the caller shifts its own tensors: the dense input, the class indices, the targets
        for k, ten in list(win.inputs.items()):
            ten[:T - hp] = ten[hp:].clone()
            ten[T - hp:] = torch.from_numpy(long.inputs[k][b - hp:b]).to(win.dev)
        win.onehot[x][:T - hp] = win.onehot[x][hp:].clone()
        win.onehot[x][T - hp:] = torch.from_numpy(idx[b - hp:b]).to(win.dev)
        for k, ten in win.targets.items():
            ten[:T - hp] = ten[hp:].clone()
            ten[T - hp:] = torch.from_numpy(long.targets[k][b - hp:b]).to(win.dev)
        win.forward_range(T - hp, T)
        masked = mask_older_frames({k: v[a:b].copy() for k, v in long.targets.items()}, T - hp)
        mask_older_frames(win.targets, T - hp)
        win.bptt()
        loss = win.compute_grads(want_loss=True)
        tl = {k: np.concatenate([v[:a], masked[k], v[b:]]) for k, v in long.targets.items()}
        ref = go.bptt_window(spec.nodes, spec.edges, long.weights, long.biases, y_long, z_long, tl, a, T, N)
        check_against(win, first, ref, f"index input, advance {step}")
        assert abs(loss - ref["loss"]) <= 1e-4 * max(1.0, abs(ref["loss"]))
