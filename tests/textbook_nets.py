"""Textbook recurrent nets written out separately from the graph oracle: a stacked LSTM with
forget gates and peephole connections, and an Elman network, each with a softmax output
layer, cross-entropy loss and a hand-derived *full-gradient* BPTT (every path through
h(t-1), c(t-1) and the peepholes is differentiated; no truncation inside the window).
A sequence may start from a given state (h0, c0), which is then a constant of the window: the
usual truncated BPTT over consecutive windows of one long sequence.

The paper states that its generalized graph equations represent these networks and their
BPTT training exactly (Sections 1, 2 and 4), so the graph oracle must agree with this file
to float64 round-off.  Nothing here knows about nodes, edges or delays.  One stream at a time.
"""
import numpy as np


def _sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def _softmax(a):
    e = np.exp(a - a.max())
    return e / e.sum()


class PeepholeLSTMLayer:
    """Parameter names: Wx*, Wh* [H, I] / [H, H] for * in i, f, g, o; peepholes wci, wcf, wco [H];
    biases b* [H].  use_h selects whether h(t-1) feeds the gates at all (the paper's
    language-model LSTM has no such connection)."""

    def __init__(self, p, use_h=True):
        self.p = {k: np.asarray(v, dtype=np.float64) for k, v in p.items()}
        self.use_h = use_h

    def forward(self, xs, h0=None, c0=None):
        p = self.p
        T = xs.shape[0]
        H = p["bi"].shape[0]
        self.xs = xs
        self.i = np.zeros((T, H)); self.f = np.zeros((T, H)); self.g = np.zeros((T, H))
        self.c = np.zeros((T, H)); self.o = np.zeros((T, H)); self.h = np.zeros((T, H))
        self.h0 = np.zeros(H) if h0 is None else np.asarray(h0, dtype=np.float64)
        self.c0 = np.zeros(H) if c0 is None else np.asarray(c0, dtype=np.float64)
        h_prev = self.h0; c_prev = self.c0
        for t in range(T):
            x = xs[t]
            rec = (lambda name: p["Wh" + name] @ h_prev) if self.use_h else (lambda name: 0.0)
            self.i[t] = _sigmoid(p["Wxi"] @ x + rec("i") + p["wci"] * c_prev + p["bi"])
            self.f[t] = _sigmoid(p["Wxf"] @ x + rec("f") + p["wcf"] * c_prev + p["bf"])
            self.g[t] = np.tanh(p["Wxg"] @ x + rec("g") + p["bg"])
            self.c[t] = self.i[t] * self.g[t] + self.f[t] * c_prev
            self.o[t] = _sigmoid(p["Wxo"] @ x + rec("o") + p["wco"] * self.c[t] + p["bo"])
            self.h[t] = self.o[t] * np.tanh(self.c[t])
            h_prev, c_prev = self.h[t], self.c[t]
        return self.h

    def backward(self, dh_above):
        """dh_above[t] = dE/dh(t) coming from the layers above.  Returns (dE/dx [T, I], grads)."""
        p = self.p
        T, H = self.h.shape
        G = {k: np.zeros_like(v) for k, v in p.items()}
        dx = np.zeros_like(self.xs)
        dh_next = np.zeros(H)      # dE/dh(t) through the gates of frame t+1
        dc_next = np.zeros(H)      # dE/dc(t) through frame t+1 (cell carry and peepholes)
        for t in range(T - 1, -1, -1):
            c_prev = self.c[t - 1] if t > 0 else self.c0
            h_prev = self.h[t - 1] if t > 0 else self.h0
            dh = dh_above[t] + dh_next
            tc = np.tanh(self.c[t])
            dao = dh * tc * self.o[t] * (1 - self.o[t])
            dc = dh * self.o[t] * (1 - tc * tc) + p["wco"] * dao + dc_next
            dai = dc * self.g[t] * self.i[t] * (1 - self.i[t])
            daf = dc * c_prev * self.f[t] * (1 - self.f[t])
            dag = dc * self.i[t] * (1 - self.g[t] ** 2)
            x = self.xs[t]
            for name, da in (("i", dai), ("f", daf), ("g", dag), ("o", dao)):
                G["Wx" + name] += np.outer(da, x)
                G["b" + name] += da
                if self.use_h:
                    G["Wh" + name] += np.outer(da, h_prev)
                dx[t] += p["Wx" + name].T @ da
            G["wci"] += dai * c_prev
            G["wcf"] += daf * c_prev
            G["wco"] += dao * self.c[t]
            dh_next = np.zeros(H)
            if self.use_h:
                for name, da in (("i", dai), ("f", daf), ("g", dag), ("o", dao)):
                    dh_next += p["Wh" + name].T @ da
            dc_next = dc * self.f[t] + p["wci"] * dai + p["wcf"] * daf
        return dx, G


def lstm_stack_loss_and_grads(layer_params, Wy, by, xs, targets, use_h=True, state0=None):
    """Stacked peephole LSTM + softmax/cross-entropy for one stream.  state0: per layer (h0, c0),
    the state the sequence starts from (default zero).
    Returns (loss, probs [T, C], per-layer grads list, dWy, dby, per-layer h list)."""
    layers = [PeepholeLSTMLayer(p, use_h) for p in layer_params]
    a = np.asarray(xs, dtype=np.float64)
    hs = []
    for l, L in enumerate(layers):
        a = L.forward(a) if state0 is None else L.forward(a, state0[l][0], state0[l][1])
        hs.append(a)
    Wy = np.asarray(Wy, dtype=np.float64); by = np.asarray(by, dtype=np.float64)
    T = a.shape[0]
    probs = np.zeros((T, by.shape[0]))
    loss = 0.0
    dlogit = np.zeros_like(probs)
    for t in range(T):
        probs[t] = _softmax(Wy @ a[t] + by)
        if targets[t] >= 0:
            loss -= np.log(probs[t, targets[t]])
            dlogit[t] = probs[t]
            dlogit[t, targets[t]] -= 1.0
    dWy = dlogit.T @ a
    dby = dlogit.sum(axis=0)
    d = dlogit @ Wy
    grads = [None] * len(layers)
    for l in range(len(layers) - 1, -1, -1):
        d, grads[l] = layers[l].backward(d)
    return loss, probs, grads, dWy, dby, hs


def elman_loss_and_grads(Wx, Wh, bh, Wy, by, xs, targets, h0=None, rectifier=False):
    """h(t) = tanh(Wx x(t) + Wh h(t-1) + bh), or max(0, .) with rectifier=True; p(t) =
    softmax(Wy h(t) + by); one stream; h(-1) = h0 (a constant of the window; default zero)."""
    Wx, Wh, bh, Wy, by = (np.asarray(a, dtype=np.float64) for a in (Wx, Wh, bh, Wy, by))
    xs = np.asarray(xs, dtype=np.float64)
    T = xs.shape[0]
    H = bh.shape[0]
    h0 = np.zeros(H) if h0 is None else np.asarray(h0, dtype=np.float64)
    h = np.zeros((T, H)); probs = np.zeros((T, by.shape[0]))
    loss = 0.0
    for t in range(T):
        hp = h[t - 1] if t > 0 else h0
        a = Wx @ xs[t] + Wh @ hp + bh
        h[t] = np.where(a > 0, a, 0.0) if rectifier else np.tanh(a)
        probs[t] = _softmax(Wy @ h[t] + by)
        if targets[t] >= 0:
            loss -= np.log(probs[t, targets[t]])
    G = dict(Wx=np.zeros_like(Wx), Wh=np.zeros_like(Wh), bh=np.zeros_like(bh),
             Wy=np.zeros_like(Wy), by=np.zeros_like(by))
    dh_next = np.zeros(H)
    for t in range(T - 1, -1, -1):
        dl = np.zeros_like(by)
        if targets[t] >= 0:
            dl = probs[t].copy(); dl[targets[t]] -= 1.0
        G["Wy"] += np.outer(dl, h[t]); G["by"] += dl
        da = (Wy.T @ dl + dh_next) * (np.where(h[t] > 0, 1.0, 0.0) if rectifier else 1 - h[t] ** 2)
        hp = h[t - 1] if t > 0 else h0
        G["Wx"] += np.outer(da, xs[t]); G["Wh"] += np.outer(da, hp); G["bh"] += da
        dh_next = Wh.T @ da
    return loss, probs, G, h
