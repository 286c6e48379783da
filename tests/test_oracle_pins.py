"""Pins for the float64 graph oracle (CPU only).

The paper prints no worked numerical example, so the oracle is pinned to what the paper and
the mathematics fix: exact equivalence to textbook LSTM / Elman BPTT (Sections 1, 2, 4),
delta / epsilon / nabla W being derivatives of E_total (Section 2.2) checked by central finite
differences, and structural invariants (stream independence of Section 3.2, delay indexing
of the first equation of Section 2.1, unreachable nodes, relabelling)."""
import numpy as np
import pytest

import workloads as wl
from oracle import graph_oracle as go
from tests import textbook_nets as tb


def run_oracle(w):
    return go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)


def find_edge(spec, src, dst, delay=None, wkind=None):
    s, d = spec.node_by_name(src), spec.node_by_name(dst)
    hits = [m for m, e in enumerate(spec.edges) if e["src"] == s and e["dst"] == d
            and (delay is None or e["delay"] == delay) and (wkind is None or e["wkind"] == wkind)]
    assert len(hits) == 1, (src, dst, hits)
    return hits[0]


def lstm_layer_params(w, tag, below, use_h=True):
    """Pick the textbook parameter set of one LSTM layer out of the per-edge weight list."""
    sp = w.spec
    p = {}
    for name, node in (("i", "i"), ("f", "f"), ("g", "g"), ("o", "o")):
        p["Wx" + name] = w.weights[find_edge(sp, below, f"{tag}.{node}", 0)]
        H = p["Wx" + name].shape[0]
        p["Wh" + name] = w.weights[find_edge(sp, f"{tag}.h", f"{tag}.{node}", 1)] if use_h else np.zeros((H, H))
        p["b" + name] = w.biases[sp.node_by_name(f"{tag}.{node}")]
    p["wci"] = w.weights[find_edge(sp, f"{tag}.c", f"{tag}.i", 1)]
    p["wcf"] = w.weights[find_edge(sp, f"{tag}.c", f"{tag}.f", 1)]
    p["wco"] = w.weights[find_edge(sp, f"{tag}.c", f"{tag}.o", 0)]
    return p


def lstm_layer_edges(sp, tag, below, use_h=True):
    """(textbook name -> edge index / node index) for the gradient comparison."""
    em, bm = {}, {}
    for name in "ifgo":
        em["Wx" + name] = find_edge(sp, below, f"{tag}.{name}", 0)
        if use_h:
            em["Wh" + name] = find_edge(sp, f"{tag}.h", f"{tag}.{name}", 1)
        bm["b" + name] = sp.node_by_name(f"{tag}.{name}")
    em["wci"] = find_edge(sp, f"{tag}.c", f"{tag}.i", 1)
    em["wcf"] = find_edge(sp, f"{tag}.c", f"{tag}.f", 1)
    em["wco"] = find_edge(sp, f"{tag}.c", f"{tag}.o", 0)
    return em, bm


def relerr(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    return np.abs(a - b).max() / (den if den > 0 else 1.0)


@pytest.mark.parametrize("hidden,use_h", [([6], True), ([5, 7], True), ([6], False), ([4, 3], False)])
def test_textbook_peephole_lstm_equivalence(hidden, use_h):
    """P1: the graph oracle on the Fig. 1 construction == textbook peephole LSTM with full BPTT."""
    T, N = 9, 3
    spec = wl.lstm_net(4, hidden, 5, output_recurrence=use_h)
    w = wl.make_workload("lstm", spec, T, N, seed=11, scale=0.7, bias_scale=0.5, masked_fraction=0.2)
    r = run_oracle(w)
    (x,) = spec.input_nodes(); (out,) = spec.output_nodes()
    tags = [f"L{l + 1}" for l in range(len(hidden))]
    below = ["x"] + [f"{t}.h" for t in tags[:-1]]
    params = [lstm_layer_params(w, t, b, use_h) for t, b in zip(tags, below)]
    e_out = find_edge(spec, f"{tags[-1]}.h", "out")
    tot_loss = 0.0
    G_layers = [None] * len(hidden); GWy = 0.0; Gby = 0.0
    for n in range(N):
        loss, probs, grads, dWy, dby, hs = tb.lstm_stack_loss_and_grads(
            params, w.weights[e_out], w.biases[out], w.inputs[x][:, n], w.targets[out][:, n], use_h)
        tot_loss += loss
        assert relerr(r["y"][out][:, n], probs) < 1e-12
        for l, t in enumerate(tags):
            assert relerr(r["y"][spec.node_by_name(f"{t}.h")][:, n], hs[l]) < 1e-12
        for l in range(len(hidden)):
            G_layers[l] = grads[l] if G_layers[l] is None else {k: G_layers[l][k] + grads[l][k] for k in grads[l]}
        GWy = GWy + dWy; Gby = Gby + dby
    assert abs(r["loss"] - tot_loss) < 1e-10 * max(1.0, abs(tot_loss))
    assert relerr(r["grad_w"][e_out], GWy) < 1e-11
    assert relerr(r["grad_b"][out], Gby) < 1e-11
    for l, (t, b) in enumerate(zip(tags, below)):
        em, bm = lstm_layer_edges(spec, t, b, use_h)
        for name, m in em.items():
            assert relerr(r["grad_w"][m], G_layers[l][name]) < 1e-10, (t, name)
        for name, k in bm.items():
            assert relerr(r["grad_b"][k], G_layers[l][name]) < 1e-10, (t, name)


def test_textbook_elman_equivalence():
    """P2: a singleton with a delay-1 full self-loop == textbook Elman net."""
    T, N = 12, 2
    spec = wl.elman_net(5, 7, 4)
    w = wl.make_workload("elman", spec, T, N, seed=5, scale=0.6, bias_scale=0.4, masked_fraction=0.15)
    r = run_oracle(w)
    x, h, out = 0, 1, 2
    tot = 0.0; G = None
    for n in range(N):
        loss, probs, g, hh = tb.elman_loss_and_grads(w.weights[0], w.weights[1], w.biases[h], w.weights[2],
                                                     w.biases[out], w.inputs[x][:, n], w.targets[out][:, n])
        tot += loss
        assert relerr(r["y"][out][:, n], probs) < 1e-12
        assert relerr(r["y"][h][:, n], hh) < 1e-12
        G = g if G is None else {k: G[k] + g[k] for k in g}
    assert abs(r["loss"] - tot) < 1e-11 * max(1.0, abs(tot))
    for m, name in ((0, "Wx"), (1, "Wh"), (2, "Wy")):
        assert relerr(r["grad_w"][m], G[name]) < 1e-11
    assert relerr(r["grad_b"][h], G["bh"]) < 1e-11
    assert relerr(r["grad_b"][out], G["by"]) < 1e-11


def total_loss(w, weights, biases):
    y, _ = go.forward(w.spec.nodes, w.spec.edges, weights, biases, w.inputs, w.T, w.N)
    return go.loss(w.spec.nodes, y, w.targets)


def check_finite_differences(w, n_probe=6, h=1e-5, tol=2e-6, seed=0):
    r = run_oracle(w)
    rng = np.random.default_rng(seed)
    W64 = [None if a is None else a.astype(np.float64) for a in w.weights]
    B64 = [None if a is None else a.astype(np.float64) for a in w.biases]
    worst = 0.0
    for group, grads, store in (("w", r["grad_w"], W64), ("b", r["grad_b"], B64)):
        for idx, g in enumerate(grads):
            if g is None:
                continue
            flat = store[idx].reshape(-1)
            for j in rng.choice(flat.size, size=min(n_probe, flat.size), replace=False):
                old = flat[j]
                flat[j] = old + h; ep = total_loss(w, W64, B64)
                flat[j] = old - h; em = total_loss(w, W64, B64)
                flat[j] = old
                fd = (ep - em) / (2 * h)
                an = g.reshape(-1)[j]
                err = abs(fd - an) / max(1e-3, abs(fd), abs(an))
                worst = max(worst, err)
                assert err < tol, (group, idx, j, fd, an)
    return worst


@pytest.mark.parametrize("seed", range(8))
def test_finite_differences_random_graphs(seed):
    """P3: every gradient formula (incl. the multiplicative-layer epsilon and window edges)."""
    rng = np.random.default_rng(100 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3)
    w = wl.make_workload("rand", spec, T=6, N=2, seed=seed, scale=0.8, bias_scale=0.5,
                         masked_fraction=0.2 if seed % 2 else 0.0)
    check_finite_differences(w, n_probe=4, seed=seed)


def test_finite_differences_generalized_lstm():
    """P3 on the generalized net (delay-2 edge, sigmoid-gated multiplicative inter-layer node)."""
    spec = wl.generalized_net(3, 4, 2, 3)
    w = wl.make_workload("gen", spec, T=6, N=2, seed=3, scale=0.8, bias_scale=0.5)
    check_finite_differences(w, n_probe=3)


def test_unreachable_node_has_zero_gradient():
    """P4: a node with no path to any output receives no error; its in-edges get exactly 0."""
    spec = wl.lstm_net(3, [4], 3)
    dead = spec.add_node(wl.ADD, wl.TANH, 4, has_bias=True, name="dead")
    e1 = spec.add_edge(spec.node_by_name("L1.h"), dead, wl.FULL, 0)
    e2 = spec.add_edge(dead, dead, wl.FULL, 1)
    e3 = spec.add_edge(spec.node_by_name("L1.c"), dead, wl.DIAG, 2)
    w = wl.make_workload("dead", spec, T=7, N=2, seed=1)
    r = run_oracle(w)
    for m in (e1, e2, e3):
        assert np.all(r["grad_w"][m] == 0.0)
    assert np.all(r["grad_b"][dead] == 0.0)
    assert np.abs(r["y"][dead]).max() > 0          # it does compute something forward
    assert np.abs(r["grad_w"][0]).max() > 0         # the live part has gradients


def test_stream_independence():
    """P5: N streams == N independent single-stream runs, gradients summed (Section 3.2)."""
    spec = wl.generalized_net(3, 4, 2, 3)
    w = wl.make_workload("gen", spec, T=5, N=3, seed=9)
    r = run_oracle(w)
    gsum = None; lsum = 0.0
    for n in range(w.N):
        one = wl.Workload("one", spec, w.T, 1, w.weights, w.biases,
                          {k: v[:, n:n + 1] for k, v in w.inputs.items()},
                          {k: v[:, n:n + 1] for k, v in w.targets.items()})
        r1 = run_oracle(one)
        lsum += r1["loss"]
        for k in range(len(spec.nodes)):
            assert np.array_equal(r1["y"][k][:, 0], r["y"][k][:, n]) or relerr(r1["y"][k][:, 0], r["y"][k][:, n]) < 1e-14
        g = [None if a is None else a.copy() for a in r1["grad_w"]]
        gsum = g if gsum is None else [None if a is None else a + b for a, b in zip(gsum, g)]
    assert abs(lsum - r["loss"]) < 1e-11 * abs(lsum)
    for a, b in zip(gsum, r["grad_w"]):
        if a is not None:
            assert relerr(b, a) < 1e-11


@pytest.mark.parametrize("d", [0, 1, 3])
def test_pure_delay_line(d):
    """P6: input -> identity edge with delay d -> linear node gives y(t) = x(t - d), zero before."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 3, name="x")
    v = g.add_node(wl.ADD, wl.LINEAR, 3, name="v")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 3, has_bias=True, is_output=True, name="out")
    g.add_edge(x, v, wl.IDENTITY, d)
    g.add_edge(v, out, wl.FULL, 0)
    w = wl.make_workload("dl", g, T=8, N=2, seed=2)
    r = run_oracle(w)
    exp = np.zeros((8, 2, 3))
    exp[d:] = w.inputs[x][:8 - d]
    assert np.array_equal(r["y"][v], exp)


def test_feed_forward_graph_is_per_frame_mlp():
    """P7: with no delayed edges every frame is an independent MLP evaluation."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 4, name="x")
    a = g.add_node(wl.ADD, wl.TANH, 6, has_bias=True, name="a")
    b = g.add_node(wl.ADD, wl.SIGMOID, 6, has_bias=True, name="b")
    m = g.add_node(wl.MUL, wl.LINEAR, 6, name="m")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 3, has_bias=True, is_output=True, name="out")
    ea = g.add_edge(x, a, wl.FULL); eb = g.add_edge(x, b, wl.FULL)
    g.add_edge(a, m, wl.IDENTITY); ed = g.add_edge(b, m, wl.DIAG)
    eo = g.add_edge(m, out, wl.FULL)
    w = wl.make_workload("ff", g, T=5, N=2, seed=4)
    r = run_oracle(w)
    W = [None if q is None else q.astype(np.float64) for q in w.weights]
    X = w.inputs[x].astype(np.float64)
    A = np.tanh(X @ W[ea].T + w.biases[a]); Bv = 1 / (1 + np.exp(-(X @ W[eb].T + w.biases[b])))
    M = A * (Bv * W[ed])
    L = M @ W[eo].T + w.biases[out]
    P = np.exp(L - L.max(-1, keepdims=True)); P /= P.sum(-1, keepdims=True)
    assert relerr(r["y"][out], P) < 1e-13
    # gradient of the output layer in closed form
    D = P.copy()
    tg = w.targets[out]
    for t in range(5):
        for n in range(2):
            D[t, n, tg[t, n]] -= 1
    assert relerr(r["grad_w"][eo], np.einsum("tni,tnj->ij", D, M)) < 1e-12
    assert relerr(r["grad_b"][out], D.sum((0, 1))) < 1e-12


def test_relabelling_invariance():
    """P8: permuting node and edge ids permutes outputs and gradients accordingly."""
    rng = np.random.default_rng(77)
    spec = wl.generalized_net(3, 4, 2, 3)
    w = wl.make_workload("gen", spec, T=5, N=2, seed=8)
    r = run_oracle(w)
    K, M = len(spec.nodes), len(spec.edges)
    np_, ep = rng.permutation(K), rng.permutation(M)
    spec2 = spec.permuted(np_, ep)
    w2 = wl.Workload("perm", spec2, w.T, w.N,
                     [w.weights[int(np.argsort(ep)[m])] for m in range(M)],
                     [w.biases[int(np.argsort(np_)[k])] for k in range(K)],
                     {int(np_[k]): v for k, v in w.inputs.items()},
                     {int(np_[k]): v for k, v in w.targets.items()})
    r2 = run_oracle(w2)
    assert abs(r2["loss"] - r["loss"]) < 1e-12 * abs(r["loss"])
    for k in range(K):
        assert relerr(r2["y"][int(np_[k])], r["y"][k]) < 1e-13
    for m in range(M):
        if r["grad_w"][m] is not None:
            assert relerr(r2["grad_w"][int(ep[m])], r["grad_w"][m]) < 1e-11


def test_delta_is_negative_state_gradient():
    """Section 2.2 defines delta_k(t) = -dE_total/ds_k(t): perturbing the bias of an additive
    node shifts s_k at every frame, so -sum_t delta_k(t) must equal the bias gradient, and the
    softmax output delta must be d - y."""
    spec = wl.lstm_net(3, [4], 3)
    w = wl.make_workload("l", spec, T=6, N=2, seed=6)
    r = run_oracle(w)
    (out,) = spec.output_nodes()
    onehot = np.zeros_like(r["y"][out])
    for t in range(w.T):
        for n in range(w.N):
            onehot[t, n, w.targets[out][t, n]] = 1
    assert np.allclose(r["delta"][out], onehot - r["y"][out], atol=1e-15)
    for k, nd in enumerate(spec.nodes):
        if nd["has_bias"]:
            assert relerr(r["grad_b"][k], -r["delta"][k].sum((0, 1))) < 1e-13


def test_delay0_cycle_is_rejected():
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 2); a = g.add_node(wl.ADD, wl.TANH, 2); b = g.add_node(wl.ADD, wl.TANH, 2)
    g.add_edge(x, a, wl.FULL); g.add_edge(a, b, wl.FULL); g.add_edge(b, a, wl.FULL, 0)
    with pytest.raises(ValueError):
        go.delay0_topological_order(g.nodes, g.edges)


# ---- BPTT(h; h') of Section 3.2: backward pass over the last frames of a longer forward pass ----

def max_delay(spec):
    return max([e["delay"] for e in spec.edges] + [1])


def history_before(y_long, t_first, depth):
    """The `depth` frames in front of frame t_first of every node (zeros where the sequence has none)."""
    hist = []
    for a in y_long:
        h = np.zeros((depth,) + a.shape[1:])
        n = min(depth, t_first)
        if n:
            h[depth - n:] = a[t_first - n:t_first]
        hist.append(h)
    return hist


@pytest.mark.parametrize("seed", range(4))
def test_forward_with_history_continues_the_sequence(seed):
    """Section 3.2: the forward pass of a later window starts from the state the earlier frames
    left.  A sequence cut at any frame and continued from the d_max frames in front of the cut
    must give the activations of the uncut forward pass."""
    rng = np.random.default_rng(300 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, n_inputs=1 + seed % 2)
    L, N = 11, 2
    w = wl.make_workload("cut", spec, T=L, N=N, seed=seed, scale=0.8, bias_scale=0.5)
    y_long, z_long = go.forward(spec.nodes, spec.edges, w.weights, w.biases, w.inputs, L, N)
    for cut in (1, 4, 9):
        hist = history_before(y_long, cut, max_delay(spec))
        y2, z2 = go.forward(spec.nodes, spec.edges, w.weights, w.biases, {k: v[cut:] for k, v in w.inputs.items()}, L - cut, N, history=hist)
        for k in range(len(spec.nodes)):
            np.testing.assert_allclose(y2[k], y_long[k][cut:], rtol=1e-13, atol=1e-15)
        for m in range(len(spec.edges)):
            np.testing.assert_allclose(z2[m], z_long[m][cut:], rtol=1e-13, atol=1e-15)


def test_windowed_bptt_over_the_whole_sequence_is_plain_bptt():
    w = wl.make_workload("gen", wl.generalized_net(5, 6, 2, 3), T=9, N=2, seed=31, scale=0.6, bias_scale=0.3)
    ref = run_oracle(w)
    win = go.bptt_window(w.spec.nodes, w.spec.edges, w.weights, w.biases, ref["y"], ref["z"], w.targets, 0, w.T, w.N)
    assert win["loss"] == pytest.approx(ref["loss"], rel=1e-14)
    for a, b in zip(win["grad_w"], ref["grad_w"]):
        if b is not None:
            np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)
    for k in range(len(w.spec.nodes)):
        np.testing.assert_allclose(win["delta"][k], ref["delta"][k], rtol=1e-13, atol=1e-15)


def check_truncated_gradient_by_finite_differences(w, t_first, n_probe=4, h=1e-5, tol=2e-6, seed=0):
    """The truncated gradient of Section 2.2 (errors stop at t0', the sums over t0' < t <= t1 keep
    the real y_k(t - d_m)) is the derivative of the window's error with every activation at or
    before t0' held constant: central differences of exactly that function."""
    spec, L, N = w.spec, w.T, w.N
    T = L - t_first
    y_long, z_long = go.forward(spec.nodes, spec.edges, w.weights, w.biases, w.inputs, L, N)
    win = go.bptt_window(spec.nodes, spec.edges, w.weights, w.biases, y_long, z_long, w.targets, t_first, T, N)
    hist = history_before(y_long, t_first, max_delay(spec))        # computed once, with the unperturbed weights
    win_inputs = {k: v[t_first:] for k, v in w.inputs.items()}
    win_targets = {k: v[t_first:] for k, v in w.targets.items()}

    def window_error(weights, biases):
        y, _ = go.forward(spec.nodes, spec.edges, weights, biases, win_inputs, T, N, history=hist)
        return go.loss(spec.nodes, y, win_targets)

    W64 = [None if a is None else a.astype(np.float64) for a in w.weights]
    B64 = [None if a is None else a.astype(np.float64) for a in w.biases]
    assert window_error(W64, B64) == pytest.approx(win["loss"], rel=1e-13)
    rng = np.random.default_rng(seed)
    n_nonzero = 0
    for group, grads, store in (("w", win["grad_w"], W64), ("b", win["grad_b"], B64)):
        for idx, g in enumerate(grads):
            if g is None:
                continue
            flat = store[idx].reshape(-1)
            for j in rng.choice(flat.size, size=min(n_probe, flat.size), replace=False):
                old = flat[j]
                flat[j] = old + h; ep = window_error(W64, B64)
                flat[j] = old - h; em = window_error(W64, B64)
                flat[j] = old
                fd = (ep - em) / (2 * h)
                an = g.reshape(-1)[j]
                assert abs(fd - an) / max(1e-3, abs(fd), abs(an)) < tol, (group, idx, j, fd, an)
                n_nonzero += abs(an) > 1e-9
    assert n_nonzero > 0
    return win


@pytest.mark.parametrize("seed", range(8))
def test_windowed_bptt_is_the_truncated_gradient_random_graphs(seed):
    rng = np.random.default_rng(100 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, n_inputs=1 + seed % 2)
    w = wl.make_workload("rand", spec, T=9, N=2, seed=seed, scale=0.8, bias_scale=0.5,
                         masked_fraction=0.2 if seed % 2 else 0.0)
    check_truncated_gradient_by_finite_differences(w, t_first=3 + seed % 3, seed=seed)


def test_windowed_bptt_is_the_truncated_gradient_generalized_lstm():
    spec = wl.generalized_net(3, 4, 2, 3)
    w = wl.make_workload("gen", spec, T=8, N=2, seed=3, scale=0.8, bias_scale=0.5)
    check_truncated_gradient_by_finite_differences(w, t_first=3, n_probe=3)


def test_truncated_gradient_differs_from_a_fresh_window_when_state_is_carried():
    """Guards the pins above against a vacuous pass: with a non-zero carried state the terms that
    pair the window's first frames with pre-window activations are not zero."""
    spec = wl.lstm_net(4, [5], 3)
    L, T, N = 10, 5, 2
    w = wl.make_workload("carry", spec, T=L, N=N, seed=34, scale=0.7, bias_scale=0.3)
    y, z = go.forward(spec.nodes, spec.edges, w.weights, w.biases, w.inputs, L, N)
    win = go.bptt_window(spec.nodes, spec.edges, w.weights, w.biases, y, z, w.targets, L - T, T, N)
    # the window's frames alone, with everything before them zero in the backward pass as well
    y0 = [a.copy() for a in y]; z0 = [a.copy() for a in z]
    for a in y0 + z0:
        a[:L - T] = 0.0
    for m, e in enumerate(spec.edges):          # connection outputs that came from pre-window frames
        if e["delay"] > 0:
            z0[m][L - T:L - T + e["delay"]] = 0.0
    cut = go.bptt_window(spec.nodes, spec.edges, w.weights, w.biases, y0, z0, w.targets, L - T, T, N)
    m_hf = find_edge(spec, "L1.h", "L1.f", 1)
    m_cf = find_edge(spec, "L1.c", "L1.f", 1)
    assert relerr(cut["grad_w"][m_hf], win["grad_w"][m_hf]) > 1e-3
    assert relerr(cut["grad_w"][m_cf], win["grad_w"][m_cf]) > 1e-3


@pytest.mark.parametrize("hidden", [[6], [5, 7]])
def test_windowed_bptt_equals_textbook_lstm_started_from_the_carried_state(hidden):
    """Truncated BPTT over consecutive windows as textbooks have it: the window starts from
    (h, c) of the frame before it, taken as constants.  The textbook net is written separately."""
    L, T, N = 13, 7, 2
    t_first = L - T
    spec = wl.lstm_net(4, hidden, 5)
    w = wl.make_workload("lstm", spec, L, N, seed=12, scale=0.7, bias_scale=0.5, masked_fraction=0.2)
    y, z = go.forward(spec.nodes, spec.edges, w.weights, w.biases, w.inputs, L, N)
    win = go.bptt_window(spec.nodes, spec.edges, w.weights, w.biases, y, z, w.targets, t_first, T, N)
    (x,) = spec.input_nodes(); (out,) = spec.output_nodes()
    tags = [f"L{l + 1}" for l in range(len(hidden))]
    below = ["x"] + [f"{t}.h" for t in tags[:-1]]
    params = [lstm_layer_params(w, t, b) for t, b in zip(tags, below)]
    e_out = find_edge(spec, f"{tags[-1]}.h", "out")
    tot = 0.0; G_layers = [None] * len(hidden); GWy = 0.0
    for n in range(N):
        state0 = [(y[spec.node_by_name(f"{t}.h")][t_first - 1, n], y[spec.node_by_name(f"{t}.c")][t_first - 1, n]) for t in tags]
        loss, probs, grads, dWy, dby, hs = tb.lstm_stack_loss_and_grads(
            params, w.weights[e_out], w.biases[out], w.inputs[x][t_first:, n], w.targets[out][t_first:, n], True, state0)
        tot += loss
        assert relerr(win["y"][out][:, n], probs) < 1e-12
        for l in range(len(hidden)):
            G_layers[l] = grads[l] if G_layers[l] is None else {k: G_layers[l][k] + grads[l][k] for k in grads[l]}
        GWy = GWy + dWy
    assert abs(win["loss"] - tot) < 1e-10 * max(1.0, abs(tot))
    assert relerr(win["grad_w"][e_out], GWy) < 1e-11
    for l, (t, b) in enumerate(zip(tags, below)):
        em, bm = lstm_layer_edges(spec, t, b)
        for name, m in em.items():
            assert relerr(win["grad_w"][m], G_layers[l][name]) < 1e-10, (t, name)
        for name, k in bm.items():
            assert relerr(win["grad_b"][k], G_layers[l][name]) < 1e-10, (t, name)


def test_windowed_bptt_equals_textbook_elman_started_from_the_carried_state():
    L, T, N = 14, 6, 2
    t_first = L - T
    spec = wl.elman_net(5, 7, 4)
    w = wl.make_workload("elman", spec, L, N, seed=5, scale=0.6, bias_scale=0.4, masked_fraction=0.15)
    y, z = go.forward(spec.nodes, spec.edges, w.weights, w.biases, w.inputs, L, N)
    win = go.bptt_window(spec.nodes, spec.edges, w.weights, w.biases, y, z, w.targets, t_first, T, N)
    x, h, out = 0, 1, 2
    tot = 0.0; G = None
    for n in range(N):
        loss, probs, g, hh = tb.elman_loss_and_grads(w.weights[0], w.weights[1], w.biases[h], w.weights[2], w.biases[out],
                                                     w.inputs[x][t_first:, n], w.targets[out][t_first:, n], h0=y[h][t_first - 1, n])
        tot += loss
        assert relerr(win["y"][h][:, n], hh) < 1e-12
        G = g if G is None else {k: G[k] + g[k] for k in g}
    assert abs(win["loss"] - tot) < 1e-11 * max(1.0, abs(tot))
    for m, name in ((0, "Wx"), (1, "Wh"), (2, "Wy")):
        assert relerr(win["grad_w"][m], G[name]) < 1e-11
    assert relerr(win["grad_b"][h], G["bh"]) < 1e-11


def test_windowed_bptt_with_zero_carried_state_is_a_fresh_window():
    """Zero inputs and zero biases keep every LSTM activation that feeds a delayed connection
    (c, h) at exactly zero, so the state carried into the window is the fresh state and the window
    must give what forward + BPTT on its frames alone gives."""
    spec = wl.lstm_net(4, [5, 6], 3)
    L, T, N = 13, 8, 2
    w = wl.make_workload("carry0", spec, T=L, N=N, seed=32, scale=0.7, bias_scale=0.0)
    t_first = L - T
    for k in w.inputs:
        w.inputs[k][:t_first] = 0.0
    # the output bias may be anything; the LSTM gate biases are zero (bias_scale = 0)
    y, z = go.forward(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, L, N)
    for name in ("L1.c", "L1.h", "L2.c", "L2.h"):
        assert np.all(y[spec.node_by_name(name)][:t_first] == 0.0)
    win = go.bptt_window(w.spec.nodes, w.spec.edges, w.weights, w.biases, y, z, w.targets, t_first, T, N)
    fresh = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases,
                            {k: v[t_first:] for k, v in w.inputs.items()}, {k: v[t_first:] for k, v in w.targets.items()}, T, N)
    assert win["loss"] == pytest.approx(fresh["loss"], rel=1e-13)
    for a, b in zip(win["grad_w"], fresh["grad_w"]):
        if b is not None:
            np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    for a, b in zip(win["grad_b"], fresh["grad_b"]):
        if b is not None:
            np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_windowed_bptt_on_a_delay_free_graph_is_the_window_alone():
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 4, name="x")
    a = g.add_node(wl.ADD, wl.TANH, 6, has_bias=True, name="a")
    b = g.add_node(wl.ADD, wl.SIGMOID, 6, has_bias=True, name="b")
    m = g.add_node(wl.MUL, wl.LINEAR, 6, name="m")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 3, has_bias=True, is_output=True, name="out")
    g.add_edge(x, a, wl.FULL, 0); g.add_edge(x, b, wl.FULL, 0)
    g.add_edge(a, m, wl.IDENTITY, 0); g.add_edge(b, m, wl.DIAG, 0); g.add_edge(m, out, wl.FULL, 0)
    L, T, N = 11, 5, 3
    w = wl.make_workload("ff", g, T=L, N=N, seed=33, scale=0.8, bias_scale=0.5)
    y, z = go.forward(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, L, N)
    win = go.bptt_window(w.spec.nodes, w.spec.edges, w.weights, w.biases, y, z, w.targets, L - T, T, N)
    alone = go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases,
                            {k: v[L - T:] for k, v in w.inputs.items()}, {k: v[L - T:] for k, v in w.targets.items()}, T, N)
    for p, q in zip(win["grad_w"], alone["grad_w"]):
        if q is not None:
            np.testing.assert_allclose(p, q, rtol=1e-12, atol=1e-14)


def test_windowed_bptt_keeps_pre_window_connection_outputs():
    """Hand-derived one-frame window.  p(t) = u(t) * x(t-1), u = w x, y = softmax(W2 p); the window
    is the sequence's second frame, t = 2, so x(t-1) lies before it.  Section 2.2's epsilon of the
    multiplicative layer carries the real z_n(t): eps on u -> p is delta_p * x(t-1), hence
    dE/dw = (W2^T (y - d)) x(t-1) x(t), and dE/dW2 = (y - d) p^T."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 1, name="x")
    u = g.add_node(wl.ADD, wl.LINEAR, 1, name="u")
    p = g.add_node(wl.MUL, wl.LINEAR, 1, name="p")
    out = g.add_node(wl.ADD, wl.SOFTMAX, 2, is_output=True, name="out")
    e_w = g.add_edge(x, u, wl.FULL, 0)
    g.add_edge(u, p, wl.IDENTITY, 0)
    g.add_edge(x, p, wl.IDENTITY, 1)
    e_w2 = g.add_edge(p, out, wl.FULL, 0)
    weights = [None] * len(g.edges)
    weights[e_w] = np.array([[0.7]]); weights[e_w2] = np.array([[0.4], [-0.9]])
    biases = [None] * len(g.nodes)
    xs = np.array([1.5, -2.0]).reshape(2, 1, 1)
    targets = {out: np.array([[1], [0]])}
    y, z = go.forward(g.nodes, g.edges, weights, biases, {x: xs}, 2, 1)
    p1 = 0.7 * (-2.0) * 1.5
    assert y[p][1, 0, 0] == pytest.approx(p1)
    win = go.bptt_window(g.nodes, g.edges, weights, biases, y, z, targets, 1, 1, 1)
    s = np.array([0.4 * p1, -0.9 * p1])
    sm = np.exp(s) / np.exp(s).sum()
    dEds = sm - np.array([1.0, 0.0])
    assert win["loss"] == pytest.approx(-np.log(sm[0]))
    np.testing.assert_allclose(win["grad_w"][e_w2][:, 0], dEds * p1, rtol=1e-12)
    dEdp = 0.4 * dEds[0] - 0.9 * dEds[1]
    assert win["grad_w"][e_w][0, 0] == pytest.approx(dEdp * 1.5 * (-2.0), rel=1e-12)
    assert abs(win["grad_w"][e_w][0, 0]) > 1e-3


# ---- the squared-error criterion (Section 2.2: delta of an output layer follows the error criterion; Section 4 names the MSE) ----

@pytest.mark.parametrize("act", [wl.LINEAR, wl.SIGMOID, wl.TANH, wl.RELU])
def test_squared_error_output_layer_closed_form(act):
    """One layer y = f(W x + b) under E = 1/2 sum (d - y)^2: dE/dW = sum_t ((y - d) f'(s)) x^T in
    closed form, NaN targets left out, and delta = (d - y) f'(s)."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 5, name="x")
    out = g.add_node(wl.ADD, act, 3, has_bias=True, is_output=wl.SQUARED_ERROR, name="out")
    e = g.add_edge(x, out, wl.FULL, 0)
    w = wl.make_workload("reg", g, T=7, N=2, seed=40 + act, scale=0.6, bias_scale=0.4, masked_fraction=0.3)
    assert np.isnan(w.targets[out]).any() and not np.isnan(w.targets[out]).all()
    r = run_oracle(w)
    X = w.inputs[x].astype(np.float64)
    S = X @ w.weights[e].astype(np.float64).T + w.biases[out]
    Y = S if act == wl.LINEAR else 1 / (1 + np.exp(-S)) if act == wl.SIGMOID else np.tanh(S) if act == wl.TANH else np.where(S > 0, S, 0.0)
    dY = np.ones_like(Y) if act == wl.LINEAR else Y * (1 - Y) if act == wl.SIGMOID else 1 - Y * Y if act == wl.TANH else np.where(S > 0, 1.0, 0.0)
    D = w.targets[out].astype(np.float64)
    err = np.where(np.isnan(D), 0.0, Y - D)
    assert r["loss"] == pytest.approx(0.5 * (err ** 2).sum(), rel=1e-13)
    assert relerr(r["y"][out], Y) < 1e-14
    np.testing.assert_allclose(r["delta"][out], -err * dY, rtol=1e-13, atol=1e-16)
    assert relerr(r["grad_w"][e], np.einsum("tni,tnj->ij", err * dY, X)) < 1e-13
    assert relerr(r["grad_b"][out], (err * dY).sum((0, 1))) < 1e-13


@pytest.mark.parametrize("seed", range(6))
def test_finite_differences_with_squared_error_outputs(seed):
    """Random recurrent graphs with a softmax output and one or two squared-error outputs
    (linear / sigmoid / tanh, masked elements): every gradient against central differences."""
    rng = np.random.default_rng(700 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, squared_error_outputs=1 + seed % 2)
    w = wl.make_workload("rand_sq", spec, T=6, N=2, seed=seed, scale=0.8, bias_scale=0.5, masked_fraction=0.25)
    assert sum(n["is_output"] == wl.SQUARED_ERROR for n in spec.nodes) == 1 + seed % 2
    check_finite_differences(w, n_probe=4, seed=seed)


def test_squared_error_lstm_finite_differences_and_truncated_window():
    spec = wl.lstm_net(3, [4], 3, squared_error_act=wl.TANH)
    w = wl.make_workload("lstm_sq", spec, T=8, N=2, seed=44, scale=0.8, bias_scale=0.5, masked_fraction=0.2)
    check_finite_differences(w, n_probe=3)
    check_truncated_gradient_by_finite_differences(w, t_first=3, n_probe=3)


# ---- the rectifier as an activation function f_k (Section 2.1 leaves f_k open; Section 2.2 needs f_k') ----

def test_rectifier_layer_closed_form():
    """One hidden layer y = max(0, W x + b) under a linear squared-error read-out with fixed
    numbers: values, the zero derivative of the units that are off (and of a unit exactly at 0),
    and the weight gradient, all written out by hand."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 2, name="x")
    h = g.add_node(wl.ADD, wl.RELU, 3, has_bias=True, name="h")
    out = g.add_node(wl.ADD, wl.LINEAR, 1, is_output=wl.SQUARED_ERROR, name="out")
    e_xh = g.add_edge(x, h, wl.FULL, 0)
    e_ho = g.add_edge(h, out, wl.FULL, 0)
    W = np.array([[1.0, -1.0], [0.5, 0.5], [2.0, 1.0]])
    b = np.array([0.0, -2.0, -5.0])
    V = np.array([[1.0, 2.0, 3.0]])
    weights = [None, None]; weights[e_xh] = W; weights[e_ho] = V
    biases = [None, b, None]
    X = np.array([[[3.0, 1.0]], [[1.0, 3.0]]])          # T = 2, N = 1
    D = np.array([[[1.0]], [[0.5]]])
    # frame 0: s = (2, 0, 2): unit 1 sits exactly at 0; frame 1: s = (-2, 0, 0)
    r = go.forward_bptt(g.nodes, g.edges, weights, biases, {x: X}, {out: D}, 2, 1)
    np.testing.assert_array_equal(r["y"][h], np.array([[[2.0, 0.0, 2.0]], [[0.0, 0.0, 0.0]]]))
    np.testing.assert_array_equal(r["y"][out], np.array([[[8.0]], [[0.0]]]))
    assert r["loss"] == pytest.approx(0.5 * (7.0 ** 2 + 0.5 ** 2))
    # dE/ds_h = (y - d) V f'(s): frame 0 -> 7 * (1, 0, 3), frame 1 -> all units off
    np.testing.assert_allclose(r["grad_b"][h], np.array([7.0, 0.0, 21.0]))
    np.testing.assert_allclose(r["grad_w"][e_xh], np.outer([7.0, 0.0, 21.0], [3.0, 1.0]))
    np.testing.assert_allclose(r["grad_w"][e_ho], np.array([[7.0 * 2.0, 0.0, 7.0 * 2.0]]))


def test_textbook_rectifier_elman_equivalence():
    """A singleton with a delay-1 full self-loop and the rectifier == a textbook Elman net with
    rectified hidden units, values and full BPTT gradients."""
    T, N = 12, 2
    spec = wl.elman_net(5, 7, 4, act=wl.RELU)
    w = wl.make_workload("elman_relu", spec, T, N, seed=6, scale=0.5, bias_scale=0.4, masked_fraction=0.15)
    r = run_oracle(w)
    x, h, out = 0, 1, 2
    assert (r["y"][h] == 0).any() and (r["y"][h] > 0).any()
    tot = 0.0; G = None
    for n in range(N):
        loss, probs, g, hh = tb.elman_loss_and_grads(w.weights[0], w.weights[1], w.biases[h], w.weights[2],
                                                     w.biases[out], w.inputs[x][:, n], w.targets[out][:, n], rectifier=True)
        tot += loss
        assert relerr(r["y"][out][:, n], probs) < 1e-12
        assert relerr(r["y"][h][:, n], hh) < 1e-12
        G = g if G is None else {k: G[k] + g[k] for k in g}
    assert abs(r["loss"] - tot) < 1e-11 * max(1.0, abs(tot))
    for m, name in ((0, "Wx"), (1, "Wh"), (2, "Wy")):
        assert relerr(r["grad_w"][m], G[name]) < 1e-11
    assert relerr(r["grad_b"][h], G["bh"]) < 1e-11


@pytest.mark.parametrize("seed", range(6))
def test_finite_differences_random_graphs_with_rectifiers(seed):
    """Random recurrent graphs whose inner nodes (additive and multiplicative) draw from linear /
    sigmoid / tanh / rectifier: every gradient against central differences (the probes' steps of
    1e-5 stay clear of the kinks for these seeds), forward + BPTT and a carried window."""
    rng = np.random.default_rng(900 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, acts=(wl.LINEAR, wl.SIGMOID, wl.TANH, wl.RELU, wl.RELU))
    assert any(n["act"] == wl.RELU for n in spec.nodes)
    w = wl.make_workload("rand_relu", spec, T=6, N=2, seed=seed, scale=0.8, bias_scale=0.5, masked_fraction=0.2 if seed % 2 else 0.0)
    check_finite_differences(w, n_probe=4, seed=seed)
    check_truncated_gradient_by_finite_differences(w, t_first=2, n_probe=3)


# ---- a third aggregation function: the element-wise maximum (Section 2.1: g_k may be another function) ----

def test_maximum_layer_closed_form():
    """A node that takes the element-wise maximum of a diagonal, an identity and a delayed
    identity connection, with fixed numbers: values, the routing of the error to the connection
    that holds the maximum (the first one on a tie) and the diagonal weight gradient by hand."""
    g = wl.GraphSpec()
    x = g.add_node(wl.INPUT, wl.LINEAR, 2, name="x")
    u = g.add_node(wl.INPUT, wl.LINEAR, 2, name="u")
    mx = g.add_node(wl.MAX, wl.LINEAR, 2, name="mx")
    out = g.add_node(wl.ADD, wl.LINEAR, 2, is_output=wl.SQUARED_ERROR, name="out")
    e_d = g.add_edge(x, mx, wl.DIAG, 0)          # z0 = w * x(t)
    e_i = g.add_edge(u, mx, wl.IDENTITY, 0)      # z1 = u(t)
    e_p = g.add_edge(u, mx, wl.IDENTITY, 1)      # z2 = u(t - 1)
    e_o = g.add_edge(mx, out, wl.IDENTITY, 0)
    weights = [None] * 4; weights[e_d] = np.array([2.0, -1.0])
    X = np.array([[[1.0, 1.0]], [[0.5, -4.0]]])          # T = 2, N = 1
    U = np.array([[[2.0, 3.0]], [[0.0, 3.5]]])
    D = np.array([[[0.0, 0.0]], [[0.0, 0.0]]])
    # frame 0: z0 = (2, -1), z1 = (2, 3), z2 = (0, 0)   -> max (2, 3): unit 0 is a tie of z0 and z1 -> z0 takes it; unit 1 -> z1
    # frame 1: z0 = (1, 4),  z1 = (0, 3.5), z2 = (2, 3) -> max (2, 4): unit 0 -> z2; unit 1 -> z0
    r = go.forward_bptt(g.nodes, g.edges, weights, [None] * 4, {x: X, u: U}, {out: D}, 2, 1)
    np.testing.assert_array_equal(r["y"][mx], np.array([[[2.0, 3.0]], [[2.0, 4.0]]]))
    assert r["loss"] == pytest.approx(0.5 * (4 + 9 + 4 + 16))
    # dE/ds_mx = y - d = (2, 3), (2, 4); the diagonal weight sees it where z0 holds the maximum:
    # unit 0 at frame 0 (x = 1) and unit 1 at frame 1 (x = -4)
    np.testing.assert_allclose(r["grad_w"][e_d], np.array([2.0 * 1.0, 4.0 * -4.0]))


def test_maximum_of_one_connection_is_the_connection_itself():
    """With a single incoming connection the maximum node is an additive node without bias."""
    def net(kind):
        g = wl.GraphSpec()
        x = g.add_node(wl.INPUT, wl.LINEAR, 4, name="x")
        h = g.add_node(wl.ADD, wl.TANH, 4, has_bias=True, name="h")
        m = g.add_node(kind, wl.SIGMOID, 4, name="m")
        out = g.add_node(wl.ADD, wl.SOFTMAX, 3, has_bias=True, is_output=True, name="out")
        g.add_edge(x, h, wl.FULL, 0); g.add_edge(h, h, wl.FULL, 1); g.add_edge(h, m, wl.DIAG, 0); g.add_edge(m, out, wl.FULL, 0)
        g.add_edge(m, h, wl.IDENTITY, 2)
        return g
    wa = wl.make_workload("one_add", net(wl.ADD), T=7, N=2, seed=51, scale=0.6, bias_scale=0.3)
    wm = wl.make_workload("one_max", net(wl.MAX), T=7, N=2, seed=51, scale=0.6, bias_scale=0.3)
    ra, rm = run_oracle(wa), run_oracle(wm)
    assert ra["loss"] == rm["loss"]
    for a, b in zip(ra["grad_w"], rm["grad_w"]):
        if a is not None:
            np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("seed", [0, 1, 2, 4, 5, 7, 9, 10])
def test_finite_differences_random_graphs_with_maximum_nodes(seed):
    """Random recurrent graphs in which about half of the inner nodes take the maximum of one to
    seven connections: every gradient against central differences (the probes' steps of 1e-5 do not
    change which connection holds a maximum for these seeds), forward + BPTT and a carried window."""
    rng = np.random.default_rng(950 + seed)
    spec = wl.random_graph(rng, n_inner=6 + seed % 3, max_delay=3, max_fraction=0.5)
    assert any(n["kind"] == wl.MAX for n in spec.nodes)
    w = wl.make_workload("rand_max", spec, T=6, N=2, seed=seed, scale=0.8, bias_scale=0.5, masked_fraction=0.2 if seed % 2 else 0.0)
    check_finite_differences(w, n_probe=4, seed=seed)
    check_truncated_gradient_by_finite_differences(w, t_first=2, n_probe=3)
