"""GPU parity for BPTT(h; h') of Section 3.2: a window computed in pieces, a window moved ahead
with the state carried over, and the frame-by-frame schedule (no batching over frames), against
the float64 oracle.  Bars as in test_gpu_parity.py."""
import numpy as np
import pytest

import workloads as wl
from oracle import graph_oracle as go
from tests.test_gpu_parity import GRAD_TOL, OUT_TOL, nerr

pytestmark = pytest.mark.gpu


def check_against(win, w, ref, label):
    for k in range(len(w.spec.nodes)):
        if w.spec.nodes[k]["kind"] == wl.INPUT:
            continue
        e = nerr(win.node_output(k), ref["y"][k])
        assert e < OUT_TOL, (label, "y", w.spec.nodes[k]["name"], e)
        e = nerr(win.node_state_grad(k), -ref["delta"][k])
        assert e < GRAD_TOL, (label, "ds", w.spec.nodes[k]["name"], e)
    gw, gb = win.grads_unpacked()
    for m, g in enumerate(ref["grad_w"]):
        if g is not None:
            e = nerr(gw[m], g)
            assert e < GRAD_TOL, (label, "grad_w", m, e)
    for k, g in enumerate(ref["grad_b"]):
        if g is not None:
            e = nerr(gb[k], g)
            assert e < GRAD_TOL, (label, "grad_b", k, e)


def gated_net(n_gates, D=12, n_in=7, n_out=4, feed_from_m=True):
    """A recurrent layer with n_gates equally wide gate nodes that all read h(t-1) (and m(t-2))
    through full edges: the gates' state gradients are exchanged together in the backward loop and
    h, m together in the forward loop (2, 3, 4 or 5 tensors of one width)."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, n_in, name="x")
    gates = [g.add_node(wl.ADD, wl.SIGMOID if j % 2 else wl.TANH, D, has_bias=True, name=f"g{j}") for j in range(n_gates)]
    m = g.add_node(wl.MUL, wl.LINEAR, D, name="m")
    h = g.add_node(wl.ADD, wl.TANH, D, name="h")
    for gate in gates:
        g.add_edge(x, gate, wl.FULL, 0)
        g.add_edge(h, gate, wl.FULL, 1)
    if feed_from_m:
        g.add_edge(m, gates[0], wl.FULL, 2)
    g.add_edge(gates[0], m, wl.IDENTITY, 0); g.add_edge(gates[1], m, wl.IDENTITY, 0)
    g.add_edge(m, h, wl.IDENTITY, 0)
    for gate in gates[2:]:
        g.add_edge(gate, h, wl.DIAG, 0)
    g.add_edge(h, h, wl.DIAG, 1)
    out = g.add_node(wl.ADD, wl.SOFTMAX, n_out, has_bias=True, is_output=True, name="out")
    g.add_edge(h, out, wl.FULL, 0)
    return g


WINDOW_NETS = {
    "gates2": lambda: (gated_net(2), 1),
    "gates3": lambda: (gated_net(3), 2),
    "gates5": lambda: (gated_net(5, D=20), 1),
    "lstm2": lambda: (wl.lstm_net(10, [24, 20], 5), 1),
    "lstm2_streams": lambda: (wl.lstm_net(10, [24, 20], 5), 3),
    "generalized": lambda: (wl.generalized_net(8, 16, 2, 4), 2),
    "lstm_many_streams": lambda: (wl.lstm_net(8, [32], 4), 20),
    "lstm2_many_streams": lambda: (wl.lstm_net(8, [32, 24], 4), 18),
    # 128-wide layers at a multiple of 16 streams: tile-blocked exchange forward, products sent backward
    # (a stack in one launch; delay-2 connections and gated layer inputs)
    "lstm2_16_streams": lambda: (wl.lstm_net(8, [128, 128], 4), 16),
    "generalized_32_streams": lambda: (wl.generalized_net(8, 128, 2, 4), 32),
    # random graphs: delays up to 3, multiplicative nodes fed through delayed connections, inputs
    # with delayed and element-wise out-connections (the library keeps its own history of those)
    "random_a": lambda: (wl.random_graph(np.random.default_rng(501), n_inner=7, max_delay=3, n_inputs=2), 2),
    "random_b": lambda: (wl.random_graph(np.random.default_rng(502), n_inner=8, max_delay=3, n_inputs=1), 3),
    "random_many_streams": lambda: (wl.random_graph(np.random.default_rng(503), n_inner=6, max_delay=2, n_inputs=2), 11),
    # dense targets under the squared error (masked by NaN)
    "lstm_squared_error": lambda: (wl.lstm_net(10, [24], 5, squared_error_act=wl.TANH), 2),
    # maximum units (another aggregation function)
    "random_maximum": lambda: (wl.random_graph(np.random.default_rng(955), n_inner=7, max_delay=3, max_fraction=0.5), 2),
    # rectified units
    "elman_rectifier": lambda: (wl.elman_net(8, 30, 5, act=wl.RELU), 2),
    "random_rectifier": lambda: (wl.random_graph(np.random.default_rng(505), n_inner=7, max_delay=3, acts=(wl.LINEAR, wl.SIGMOID, wl.TANH, wl.RELU, wl.RELU)), 3),
    "random_squared_error": lambda: (wl.random_graph(np.random.default_rng(504), n_inner=7, max_delay=3, squared_error_outputs=2), 2),
}


def mask_older_frames(targets, n_frames):
    """No error at the first n_frames frames: class index -1, or NaN for dense target vectors."""
    for k in targets:
        if isinstance(targets[k], np.ndarray):
            targets[k][:n_frames] = np.nan if targets[k].dtype.kind == "f" else -1
        else:
            targets[k][:n_frames] = float("nan") if targets[k].is_floating_point() else -1
    return targets


@pytest.mark.parametrize("name", sorted(WINDOW_NETS))
def test_window_computed_in_pieces_equals_the_window_at_once(name):
    from paper_1503_02852_amd.runner import window_for
    spec, N = WINDOW_NETS[name]()
    w = wl.make_workload(name, spec, T=24, N=N, seed=41, scale=0.4, bias_scale=0.3, masked_fraction=0.3)
    print(f"[window] pieces {name}: T={w.T} N={w.N}", flush=True)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    win = window_for(w)
    for t0, t1 in ((0, 7), (7, 8), (8, 19), (19, 24)):
        win.forward_range(t0, t1)
    win.bptt()
    loss = win.compute_grads(want_loss=True)
    check_against(win, w, ref, name)
    assert abs(loss - ref["loss"]) <= 1e-5 * max(1.0, abs(ref["loss"]))


def test_forward_range_needs_the_earlier_frames():
    from paper_1503_02852_amd.binding import RnnError
    from paper_1503_02852_amd.runner import window_for
    w = wl.make_workload("seq", wl.lstm_net(6, [8], 3), T=10, N=1, seed=42)
    win = window_for(w)
    with pytest.raises(RnnError):
        win.forward_range(4, 10)          # nothing computed yet
    win.forward_range(0, 4)
    with pytest.raises(RnnError):
        win.forward_range(6, 10)          # gap
    with pytest.raises(RnnError):
        win.bptt()                        # window incomplete
    win.forward_range(4, 10)
    win.bptt()


@pytest.mark.parametrize("name", sorted(WINDOW_NETS))
def test_window_moved_ahead_with_carried_state(name):
    """Forward over T frames, then the window advances twice by h' = T / 2 new frames.  Activations
    must equal the oracle's forward pass over the whole sequence; the gradients (targets of the
    older half masked) must equal the oracle's backward pass over the window's frames."""
    from paper_1503_02852_amd.runner import window_for
    spec, N = WINDOW_NETS[name]()
    T, hp = 16, 8
    L = T + 2 * hp
    long = wl.make_workload(name, spec, T=L, N=N, seed=43, scale=0.4, bias_scale=0.3)
    print(f"[window] carry {name}: T={T} h'={hp} N={N}", flush=True)
    y_long, z_long = go.forward(long.spec.nodes, long.spec.edges, long.weights, long.biases, long.inputs, L, N)
    first = wl.Workload(name=name, spec=spec, T=T, N=N, weights=long.weights, biases=long.biases,
                        inputs={k: v[:T].copy() for k, v in long.inputs.items()},
                        targets={k: v[:T].copy() for k, v in long.targets.items()})
    win = window_for(first)
    win.forward()
    differs = 0.0
    for step in (1, 2):
        a, b = step * hp, step * hp + T
        new_targets = {k: v[b - hp:b] for k, v in long.targets.items()}
        win.advance({k: v[b - hp:b] for k, v in long.inputs.items()}, new_targets)
        # the older part of the window has been trained on already: mask it
        masked = mask_older_frames({k: v[a:b].copy() for k, v in long.targets.items()}, T - hp)
        mask_older_frames(win.targets, T - hp)
        win.bptt()
        loss = win.compute_grads(want_loss=True)
        tl = {k: np.concatenate([v[:a], masked[k], v[b:]]) for k, v in long.targets.items()}      # (only the window's frames count)
        ref = go.bptt_window(long.spec.nodes, long.spec.edges, long.weights, long.biases, y_long, z_long, tl, a, T, N)
        check_against(win, first, ref, f"{name} advance {step}")
        assert abs(loss - ref["loss"]) <= 1e-5 * max(1.0, abs(ref["loss"]))
        # what the same frames give as a fresh window (zero state in front): the carried history matters
        fresh = go.forward_bptt(long.spec.nodes, long.spec.edges, long.weights, long.biases,
                                {k: v[a:b] for k, v in long.inputs.items()}, masked, T, N)
        for g1, g2 in zip(ref["grad_w"], fresh["grad_w"]):
            if g1 is not None:
                differs = max(differs, nerr(g2, g1))
    if not name.startswith("random"):      # (in a random graph the state may hardly reach the unmasked frames)
        assert differs > 1e-3, "the carried state made no difference: the test does not tell the two apart"


@pytest.mark.parametrize("name", ["lstm2", "lstm2_streams", "lstm2_16_streams"])
def test_windows_with_helper_members_in_every_launch(monkeypatch, name):
    """The same two checks with helper members forced into both launches of the stacks (forward
    pieces: the helper's sums cover exactly the frames of a piece; moved windows: nothing of a
    helper's tensors is carried)."""
    monkeypatch.setenv("RNNG_CHAIN_HELPERS", "1")
    test_window_computed_in_pieces_equals_the_window_at_once(name)
    test_window_moved_ahead_with_carried_state(name)


def test_frame_by_frame_schedule_gives_the_same_results(monkeypatch):
    """The baseline schedule of Section 4 (every frame on its own) must reach the oracle as well."""
    from paper_1503_02852_amd.runner import window_for
    monkeypatch.setenv("RNNG_SCHEDULE", "framewise")
    w = wl.make_workload("framewise", wl.generalized_net(8, 16, 2, 4), T=11, N=2, seed=44, scale=0.4, bias_scale=0.3)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    win = window_for(w)
    win.forward(); win.bptt()
    loss = win.compute_grads(want_loss=True)
    check_against(win, w, ref, "framewise")
    assert abs(loss - ref["loss"]) <= 1e-5 * max(1.0, abs(ref["loss"]))


@pytest.mark.parametrize("n_gates,N", [(2, 1), (3, 1), (3, 4), (4, 2), (5, 1)])
def test_equally_wide_exchanged_tensors(n_gates, N):
    """2 to 5 equally wide tensors exchanged between workgroups in one step (bundled stores)."""
    from paper_1503_02852_amd.runner import window_for
    spec = gated_net(n_gates, D=40 if n_gates == 4 else 12)
    w = wl.make_workload(f"gates{n_gates}", spec, T=15, N=N, seed=50 + n_gates, scale=0.4, bias_scale=0.3, masked_fraction=0.2)
    ref = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    win = window_for(w)
    win.forward(); win.bptt()
    loss = win.compute_grads(want_loss=True)
    check_against(win, w, ref, f"gates{n_gates}")
    assert abs(loss - ref["loss"]) <= 1e-5 * max(1.0, abs(ref["loss"]))
