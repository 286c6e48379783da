"""TEST INFRASTRUCTURE -- slow float64 CPU oracle for forward + BPTT on a generalized RNN graph.

This file is the checker, not the product: only tests, the smoke entry and the
benchmark's CPU-baseline leg may import it.  It shares no code with the HIP path.

It is the plain definition written out, frame by frame (no SCC analysis, no batching
over frames, no reordering): the paper's Section 2.1 forward equations and Section 2.2
training equations, evaluated for N independent streams at once (Section 3.2 says the
multi-stream mode equals N independent copies with gradients summed), each stream
being one row of an [N x dim] matrix.

Readings where the paper is silent (all listed in the design notes of the repository):
  * optional bias per additive node, added to the state s_k (a full edge from a constant-1
    input would be the same thing inside the paper's model);
  * a third weight kind "diagonal" besides "full" and "identity" (needed for peepholes);
  * y_k = f_k(s_k) is applied to multiplicative nodes too (Section 2.2's delta equation
    uses f_k' for any layer);
  * a third aggregation function g_k besides sum and product (Section 2.1 allows "other"
    functions there): the element-wise maximum of the incoming connection outputs, node kind 3;
    its error terms go to the connection that holds the maximum, to the first one (lowest edge
    index) if several do;
  * the activation functions f_k (Section 2.1 leaves them open): linear, logistic sigmoid, tanh,
    and the rectifier max(0, s), whose derivative at s = 0 is taken as 0;
  * a fresh window starts from zero activations (frame index <= 0); a window that carries
    state (BPTT(h; h') of Section 3.2) starts from the activations the earlier frames left,
    and its backward pass follows the last two equations of Section 2.2 literally: delta and
    epsilon are propagated only while t > t0', but the connection outputs z_n(t) and the
    weight-gradient terms eps_m(t) y_k(t - d_m)^T of the frames t > t0' use the real
    y_k(t - d_m), also where t - d_m <= t0'; error terms from frames after the window are zero;
  * E_total = sum over frames, streams and output nodes of E(t) (no averaging).  Two error
    criteria (Section 2.2: the initial delta of an output layer depends on the criterion E(t) and
    on the layer's activation function): is_output = 1, softmax with minimum
    cross-entropy, E = -ln y_target (natural log), class targets, -1 masks the frame; is_output = 2,
    squared error E = 1/2 sum_j (d_j - y_j)^2 (the MSE criterion Section 4 names) on a linear,
    sigmoid, tanh or rectifier output layer, dense targets, a NaN target element has no error;
  * the functions return dE_total/dW (the paper's nabla W = -sum eps y^T with
    eps = -dE/dz is exactly that).

Parity pins (tests/, `-m "not gpu"`): a separately written textbook peephole LSTM and
Elman net (tanh and rectifier) with hand-derived full BPTT, central finite differences of E_total,
stream-independence, delay-line, unreachable-node and relabelling invariants; forward with a
carried history against one forward pass over the whole sequence; bptt_window against bptt itself
(whole sequence), against central finite differences of the window's error with the pre-window
activations held constant (which is the truncated gradient), against a textbook LSTM / Elman
BPTT started from a non-zero state, against a hand-derived one-frame window, and against the
window alone on a delay-free graph.
"""
from __future__ import annotations

import numpy as np

INPUT, ADD, MUL, MAX = 0, 1, 2, 3
CROSS_ENTROPY, SQUARED_ERROR = 1, 2          # values of a node's is_output
LINEAR, SIGMOID, TANH, SOFTMAX, RELU = 0, 1, 2, 3, 4
FULL, DIAG, IDENTITY = 0, 1, 2


def delay0_topological_order(nodes, edges):
    """Any topological order of the graph restricted to its delay-0 edges (Section 3.1
    requires that what remains after setting the delayed connections aside is a DAG).
    Kahn's algorithm, smallest node id first.  Raises if a delay-0 cycle exists."""
    K = len(nodes)
    indeg = [0] * K
    succ = [[] for _ in range(K)]
    for e in edges:
        if e["delay"] == 0:
            indeg[e["dst"]] += 1
            succ[e["src"]].append(e["dst"])
    ready = sorted(k for k in range(K) if indeg[k] == 0)
    order = []
    while ready:
        k = ready.pop(0)
        order.append(k)
        for v in succ[k]:
            indeg[v] -= 1
            if indeg[v] == 0:
                ready.append(v)
        ready.sort()
    if len(order) != K:
        raise ValueError("delay-0 edges form a cycle")
    return order


def _apply_weight(e, w, y):
    """z = W y for one connection (Section 2.1, first equation); rows of y are streams."""
    if e["wkind"] == FULL:
        return y @ w.T
    if e["wkind"] == DIAG:
        return y * w
    return y


def _apply_weight_transposed(e, w, eps):
    """W^T eps for one connection (matrix form of the delta equation, Section 2.2)."""
    if e["wkind"] == FULL:
        return eps @ w
    if e["wkind"] == DIAG:
        return eps * w
    return eps


def _activation(act, s):
    if act == LINEAR:
        return s
    if act == SIGMOID:
        return 1.0 / (1.0 + np.exp(-s))
    if act == TANH:
        return np.tanh(s)
    if act == RELU:
        return np.maximum(s, 0.0)
    if act == SOFTMAX:
        m = s.max(axis=-1, keepdims=True)
        ex = np.exp(s - m)
        return ex / ex.sum(axis=-1, keepdims=True)
    raise ValueError(act)


def _activation_derivative(act, y):
    if act == LINEAR:
        return np.ones_like(y)
    if act == SIGMOID:
        return y * (1.0 - y)
    if act == TANH:
        return 1.0 - y * y
    if act == RELU:
        return (y > 0.0).astype(y.dtype)
    raise ValueError(act)


def forward(nodes, edges, weights, biases, inputs, T, N, history=None):
    """Forward pass over frames 1..T (stored at index 0..T-1).

    weights[m]: float array [n_dst, n_src] (full), [dim] (diagonal) or None (identity).
    biases[k]:  float array [dim] or None.   inputs[k]: [T, N, dim] for every input node.
    history[k] (optional, every node): [Hh, N, dim], the activations of the Hh frames in front of
    the window (its last row is the frame right before the window), as left by an earlier
    forward pass (Section 3.2: the forward pass of BPTT(h; h') continues from the carried
    state); frames further back, and all of them without a history, are zero.
    Returns (y, z): y[k] is [T, N, dim] for every node; z[m] is [T, N, dim] for every edge
    (the connection outputs, which the multiplicative layers' backward pass needs)."""
    W = [None if w is None else np.asarray(w, dtype=np.float64) for w in weights]
    B = [None if b is None else np.asarray(b, dtype=np.float64) for b in biases]
    order = delay0_topological_order(nodes, edges)
    anterior = [[] for _ in nodes]
    for m, e in enumerate(edges):
        anterior[e["dst"]].append(m)
    y = [np.zeros((T, N, n["dim"])) for n in nodes]
    z = [np.zeros((T, N, nodes[e["dst"]]["dim"])) for e in edges]
    for k, n in enumerate(nodes):
        if n["kind"] == INPUT:
            y[k][:] = np.asarray(inputs[k], dtype=np.float64)
    def source_activation(k, tau):
        """y_k(tau); tau < 0 lies before the window: the carried history, else zero."""
        if tau >= 0:
            return y[k][tau]
        if history is not None and -tau <= len(history[k]):
            return np.asarray(history[k][len(history[k]) + tau], dtype=np.float64)
        return None

    for t in range(T):
        for k in order:
            n = nodes[k]
            if n["kind"] == INPUT:
                continue
            for m in anterior[k]:
                e = edges[m]
                ysrc = source_activation(e["src"], t - e["delay"])
                if ysrc is not None:
                    z[m][t] = _apply_weight(e, W[m], ysrc)
                # else: the source activation before the window is zero, so z stays zero
            if n["kind"] == ADD:
                s = np.zeros((N, n["dim"]))
                for m in anterior[k]:
                    s = s + z[m][t]
                if B[k] is not None:
                    s = s + B[k]
            elif n["kind"] == MAX:
                s = z[anterior[k][0]][t]
                for m in anterior[k][1:]:
                    s = np.maximum(s, z[m][t])
            else:
                s = np.ones((N, n["dim"]))
                for m in anterior[k]:
                    s = s * z[m][t]
            y[k][t] = _activation(n["act"], s)
    return y, z


def loss(nodes, y, targets):
    """E_total: the error criterion of every output node summed over frames and streams."""
    total = 0.0
    for k, n in enumerate(nodes):
        if not n["is_output"]:
            continue
        if n["is_output"] == SQUARED_ERROR:
            d = np.asarray(targets[k], dtype=np.float64)
            err = np.where(np.isnan(d), 0.0, d - y[k])
            total += 0.5 * float((err * err).sum())
            continue
        tg = np.asarray(targets[k])
        T, N = tg.shape
        for t in range(T):
            for s in range(N):
                c = int(tg[t, s])
                if c >= 0:
                    total -= np.log(y[k][t, s, c])
    return float(total)


def bptt(nodes, edges, weights, biases, y, z, targets, T, N, t_first=0):
    """Backward pass over frames T..t_first+1 (indices T-1 .. t_first) in reverse delay-0
    topological order; t_first is the paper's truncation point t0' (Section 2.2).

    Works in the paper's variables: delta_k(t) = -dE/ds_k(t), eps_m(t) = -dE/dz_m(t);
    output nodes start from delta = d - y (softmax with cross-entropy) or, under the squared
    error, delta = (d - y) f'(s).  delta and eps are
    back-propagated only while t > t0': nothing is handed to a frame before t_first.  The
    gradient sums run over t0' < t <= t1 with the real y_src(t - d_m) and the real connection
    outputs z_n(t), also where t - d_m lies at or before t0' (frames before index 0 do not
    exist: zero).  Returns
    (grad_w, grad_b, delta): grad_w[m] = -sum_t eps_m(t) y_src(t - d_m)^T summed over
    streams (None for identity edges), grad_b[k] = -sum_t delta_k(t), and delta[k] as
    [T, N, dim] for every non-input node (zero before t_first)."""
    W = [None if w is None else np.asarray(w, dtype=np.float64) for w in weights]
    order = delay0_topological_order(nodes, edges)
    anterior = [[] for _ in nodes]
    for m, e in enumerate(edges):
        anterior[e["dst"]].append(m)
    acc = [np.zeros((T, N, n["dim"])) for n in nodes]       # sum_n W_n^T eps_n(t + d_n)
    delta = [np.zeros((T, N, n["dim"])) for n in nodes]
    grad_w = [None if w is None else np.zeros_like(w) for w in W]
    grad_b = [None if b is None else np.zeros(nodes[k]["dim"]) for k, b in enumerate(biases)]
    for t in range(T - 1, t_first - 1, -1):
        for k in reversed(order):
            n = nodes[k]
            if n["kind"] == INPUT:
                continue
            if n["is_output"] == SQUARED_ERROR:
                # E(t) = 1/2 sum_j (d_j - y_j)^2, so -dE/ds_j = (d_j - y_j) f'(s_j)
                d = np.asarray(targets[k], dtype=np.float64)[t]
                delta[k][t] = np.where(np.isnan(d), 0.0, d - y[k][t]) * _activation_derivative(n["act"], y[k][t])
            elif n["is_output"]:
                d = np.zeros((N, n["dim"]))
                tg = np.asarray(targets[k])[t]
                for s in range(N):
                    c = int(tg[s])
                    if c >= 0:
                        d[s, c] = 1.0
                        d[s] -= y[k][t, s]
                delta[k][t] = d
            else:
                delta[k][t] = acc[k][t] * _activation_derivative(n["act"], y[k][t])
            if grad_b[k] is not None:
                grad_b[k] -= delta[k][t].sum(axis=0)
            for m in anterior[k]:
                e = edges[m]
                if n["kind"] == ADD:
                    eps = delta[k][t]
                elif n["kind"] == MAX:
                    # ds/dz_m is 1 where connection m holds the maximum (the first one, if several do), else 0
                    eps = delta[k][t].copy()
                    for other in anterior[k]:
                        if other < m:
                            eps = eps * (z[m][t] > z[other][t])
                        elif other > m:
                            eps = eps * (z[m][t] >= z[other][t])
                else:
                    eps = delta[k][t].copy()
                    for other in anterior[k]:
                        if other != m:
                            eps = eps * z[other][t]
                tau = t - e["delay"]
                if tau < 0:
                    continue            # no such frame: its activation is zero
                ysrc = y[e["src"]][tau]
                if e["wkind"] == FULL:
                    grad_w[m] -= eps.T @ ysrc
                elif e["wkind"] == DIAG:
                    grad_w[m] -= (eps * ysrc).sum(axis=0)
                if tau >= t_first and nodes[e["src"]]["kind"] != INPUT:
                    acc[e["src"]][tau] += _apply_weight_transposed(e, W[m], eps)
    return grad_w, grad_b, delta


def bptt_window(nodes, edges, weights, biases, y_long, z_long, targets_long, t_first, T, N):
    """BPTT(h; h') of Section 3.2: the forward pass has run over a longer sequence (y_long, z_long
    from `forward`), the backward pass covers only its T frames [t_first, t_first + T), truncated
    at t0' = t_first as the last two equations of Section 2.2 say: errors stop at the window
    start, while the frames inside the window see the real activations of the frames before it.
    The error counts the window's frames only.  With t_first = 0 and T the whole sequence this is
    `bptt`.  Returned arrays cover the window's T frames."""
    t_end = t_first + T
    y_cut = [a[:t_end] for a in y_long]
    z_cut = [a[:t_end] for a in z_long]
    targets = {k: np.asarray(v)[:t_end] for k, v in targets_long.items()}
    E = loss(nodes, [a[t_first:] for a in y_cut], {k: v[t_first:] for k, v in targets.items()})
    grad_w, grad_b, delta = bptt(nodes, edges, weights, biases, y_cut, z_cut, targets, t_end, N, t_first)
    return dict(y=[a[t_first:] for a in y_cut], z=[a[t_first:] for a in z_cut], loss=E, grad_w=grad_w, grad_b=grad_b,
                delta=[a[t_first:] for a in delta])


def forward_bptt(nodes, edges, weights, biases, inputs, targets, T, N):
    """Convenience wrapper: one window of forward + BPTT.  Returns a dict."""
    y, z = forward(nodes, edges, weights, biases, inputs, T, N)
    E = loss(nodes, y, targets)
    grad_w, grad_b, delta = bptt(nodes, edges, weights, biases, y, z, targets, T, N)
    return dict(y=y, z=z, loss=E, grad_w=grad_w, grad_b=grad_b, delta=delta)
