"""Device-memory plumbing around the binding: torch tensors hold weights, inputs, targets,
workspace and gradients; every computation happens inside librnngraph.so."""
from __future__ import annotations

import numpy as np
import torch

from .binding import Graph


class Window:
    """One graph + one window shape (T, N) with all device buffers allocated."""

    def __init__(self, node_array, edge_array, T, N, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("rnngraph needs a GPU: there is no CPU path")
        self.g = Graph(node_array, edge_array)
        self.T, self.N = T, N
        self.dev = torch.device(device)
        self.ws_bytes = self.g.workspace_bytes(T, N)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.dev)
        self.ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256
        self.n_params = self.g.param_count()
        self.weights = torch.zeros(self.n_params, dtype=torch.float32, device=self.dev)
        self.grads = torch.empty(self.n_params, dtype=torch.float32, device=self.dev)
        self.inputs = {}
        self.targets = {}

    def set_params(self, weights, biases):
        self.weights.copy_(torch.from_numpy(self.g.pack_params(weights, biases)))

    def set_inputs(self, inputs):
        for k in self.g.input_nodes:
            a = np.ascontiguousarray(inputs[k], dtype=np.float32)
            assert a.shape == (self.T, self.N, int(self.g.nodes[k, 2])), a.shape
            self.inputs[k] = torch.from_numpy(a).to(self.dev)

    def set_onehot_inputs(self, indices):
        """indices[k]: int [T][N] class indices of input node k, given instead of its dense tensor."""
        self.onehot = getattr(self, "onehot", {})
        for k, a in indices.items():
            a = np.ascontiguousarray(a, dtype=np.int32)
            assert a.shape == (self.T, self.N)
            self.onehot[k] = torch.from_numpy(a).to(self.dev)
            self.g.set_onehot_input(self.g.input_nodes.index(k), self.onehot[k].data_ptr())
            self.inputs.pop(k, None)

    def _input_ptrs(self):
        return [self.inputs[k].data_ptr() if k in self.inputs else 0 for k in self.g.input_nodes]

    def set_targets(self, targets):
        for k in self.g.output_nodes:
            if int(self.g.nodes[k, 4]) == 2:      # squared-error output: dense target vectors
                a = np.ascontiguousarray(targets[k], dtype=np.float32)
                assert a.shape == (self.T, self.N, int(self.g.nodes[k, 2]))
            else:
                a = np.ascontiguousarray(targets[k], dtype=np.int32)
                assert a.shape == (self.T, self.N)
            self.targets[k] = torch.from_numpy(a).to(self.dev)

    def _stream(self):
        return torch.cuda.current_stream(self.dev).cuda_stream

    def forward(self):
        self.g.forward(self.weights.data_ptr(), self._input_ptrs(),
                       self.T, self.N, self.ws_ptr, self.ws_bytes, self._stream())

    def forward_range(self, t_begin, t_end):
        """Frames [t_begin, t_end) of the window; the frames before them come from earlier calls."""
        self.g.forward_range(self.weights.data_ptr(), self._input_ptrs(),
                             self.T, self.N, t_begin, t_end, self.ws_ptr, self.ws_bytes, self._stream())

    def advance(self, new_inputs, new_targets):
        """Moves the window ahead by the number of frames in new_inputs ([frames][N][dim] per input
        node; new_targets [frames][N] per output node): shifts the activations and the caller-owned
        input / target tensors, then computes the new frames from the carried state."""
        frames = int(next(iter(new_inputs.values())).shape[0])
        self.g.shift_window(frames, self._stream())
        for k in self.g.input_nodes:
            x = self.inputs[k]
            x[:self.T - frames] = x[frames:].clone()
            x[self.T - frames:] = torch.from_numpy(np.ascontiguousarray(new_inputs[k], dtype=np.float32)).to(self.dev)
        for k in self.g.output_nodes:
            d = self.targets[k]
            d[:self.T - frames] = d[frames:].clone()
            d[self.T - frames:] = torch.from_numpy(np.ascontiguousarray(new_targets[k])).to(self.dev).to(d.dtype)
        self.forward_range(self.T - frames, self.T)

    def bptt(self):
        self.g.bptt(self.weights.data_ptr(), [self.targets[k].data_ptr() for k in self.g.output_nodes], self._stream())

    def compute_grads(self, want_loss=False):
        return self.g.grads(self.grads.data_ptr(), want_loss, self._stream())

    def check(self):
        """Waits for the stream; raises if a kernel of the current window has flagged an error."""
        self.g.check(self._stream())

    def step(self):
        """One pass of the whole hot path: forward, BPTT, weight gradients (asynchronous)."""
        self.forward()
        self.bptt()
        self.compute_grads(False)

    # ---- read-back helpers for tests ---------------------------------------------------
    def _view(self, ptr, dim):
        n = self.T * self.N * dim
        if ptr >= self.ws.data_ptr() and ptr < self.ws.data_ptr() + self.ws.numel():
            off = ptr - self.ws.data_ptr()
            return self.ws[off:off + 4 * n].view(torch.float32).view(self.T, self.N, dim)
        raise ValueError("pointer outside the workspace")

    def node_output(self, k):
        dim = int(self.g.nodes[k, 2])
        if k in self.inputs:
            return self.inputs[k].cpu().numpy()
        torch.cuda.synchronize(self.dev)
        return self._view(self.g.output_ptr(k), dim).cpu().numpy()

    def node_state_grad(self, k):
        dim = int(self.g.nodes[k, 2])
        torch.cuda.synchronize(self.dev)
        return self._view(self.g.state_grad_ptr(k), dim).cpu().numpy()

    def grads_unpacked(self):
        torch.cuda.synchronize(self.dev)
        return self.g.unpack_params(self.grads.cpu().numpy())


def window_for(workload, device="cuda:0"):
    w = Window(workload.spec.node_array(), workload.spec.edge_array(), workload.T, workload.N, device)
    w.set_params(workload.weights, workload.biases)
    w.set_inputs(workload.inputs)
    w.set_targets(workload.targets)
    return w
