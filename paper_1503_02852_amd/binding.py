"""Thin ctypes binding of librnngraph.so: argument marshalling only.

Every step of the forward / BPTT path runs in the library's HIP kernels; PyTorch is used by
callers for device memory and streams.  There is no CPU fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librnngraph.so")

EXPORTS = ["rnn_graph_create", "rnn_graph_destroy", "rnn_graph_schedule", "rnn_param_count",
           "rnn_edge_param_offset", "rnn_bias_param_offset", "rnn_workspace_bytes", "rnn_forward",
           "rnn_forward_range", "rnn_shift_window", "rnn_set_onehot_input",
           "rnn_output", "rnn_bptt", "rnn_state_grad", "rnn_grads", "rnn_check", "rnn_set_deterministic", "rnn_specialise",
           "rnn_forward_static", "rnn_last_error"]
# measurement and inspection aids (include/rnngraph_aux.h)
AUX_EXPORTS = ["rnn_step_build", "rnn_debug_read_control", "rnn_profile_enable", "rnn_profile_read", "rnn_plan_work"]
BUILD_NAMES = {0: "none", 1: "wave", 2: "matrix", 3: "matrix_2d", 4: "lds", 5: "interpreted", 6: "per_frame", 7: "streaming"}

_lib = None


class RnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"rnngraph error {code}: {msg}")
        self.code = code


def load_library(build_if_missing=True):
    """Loads the built library; builds it with hipcc if it does not exist yet."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _build
        _build.build()
    lib = C.CDLL(LIB_PATH)
    i32p, i64p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.c_void_p
    lib.rnn_graph_create.argtypes = [vp, C.c_int32, vp, C.c_int32, C.POINTER(vp)]
    lib.rnn_graph_create.restype = C.c_int
    lib.rnn_graph_destroy.argtypes = [vp]
    lib.rnn_graph_destroy.restype = None
    lib.rnn_graph_schedule.argtypes = [vp, i32p, i32p, i32p, i32p, i32p, i32p]
    lib.rnn_graph_schedule.restype = C.c_int
    lib.rnn_param_count.argtypes = [vp]
    lib.rnn_param_count.restype = C.c_int64
    lib.rnn_edge_param_offset.argtypes = [vp, C.c_int32, i64p, i64p]
    lib.rnn_edge_param_offset.restype = C.c_int
    lib.rnn_bias_param_offset.argtypes = [vp, C.c_int32, i64p, i64p]
    lib.rnn_bias_param_offset.restype = C.c_int
    lib.rnn_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32]
    lib.rnn_workspace_bytes.restype = C.c_int64
    lib.rnn_forward.argtypes = [vp, vp, C.POINTER(vp), C.c_int32, C.c_int32, vp, C.c_int64, vp]
    lib.rnn_forward.restype = C.c_int
    lib.rnn_forward_range.argtypes = [vp, vp, C.POINTER(vp), C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, C.c_int64, vp]
    lib.rnn_forward_range.restype = C.c_int
    lib.rnn_forward_static.argtypes = [vp, vp, C.POINTER(vp), C.POINTER(vp), C.c_int32, C.c_int32, vp]
    lib.rnn_forward_static.restype = C.c_int
    lib.rnn_set_onehot_input.argtypes = [vp, C.c_int32, vp]
    lib.rnn_set_onehot_input.restype = C.c_int
    lib.rnn_shift_window.argtypes = [vp, C.c_int32, vp]
    lib.rnn_shift_window.restype = C.c_int
    lib.rnn_output.argtypes = [vp, C.c_int32, C.POINTER(vp)]
    lib.rnn_output.restype = C.c_int
    lib.rnn_bptt.argtypes = [vp, vp, C.POINTER(vp), vp]
    lib.rnn_bptt.restype = C.c_int
    lib.rnn_state_grad.argtypes = [vp, C.c_int32, C.POINTER(vp)]
    lib.rnn_state_grad.restype = C.c_int
    lib.rnn_grads.argtypes = [vp, vp, C.POINTER(C.c_double), vp]
    lib.rnn_grads.restype = C.c_int
    lib.rnn_set_deterministic.argtypes = [vp, C.c_int32]
    lib.rnn_set_deterministic.restype = C.c_int
    lib.rnn_check.argtypes = [vp, vp]
    lib.rnn_check.restype = C.c_int
    lib.rnn_step_build.argtypes = [vp, C.c_int32, C.c_int32, i32p]
    lib.rnn_step_build.restype = C.c_int
    lib.rnn_plan_work.argtypes = [vp, C.c_int32, C.c_int32, i64p, i64p]
    lib.rnn_plan_work.restype = C.c_int
    lib.rnn_specialise.argtypes = [vp, C.c_int32]
    lib.rnn_specialise.restype = C.c_int
    lib.rnn_debug_read_control.argtypes = [vp, vp, C.c_int32]
    lib.rnn_debug_read_control.restype = C.c_int
    lib.rnn_profile_enable.argtypes = [vp, C.c_int32]
    lib.rnn_profile_enable.restype = C.c_int
    lib.rnn_profile_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), i64p]
    lib.rnn_profile_read.restype = C.c_int
    lib.rnn_last_error.argtypes = []
    lib.rnn_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(code):
    if code < 0:
        raise RnnError(code, load_library().rnn_last_error().decode())
    return code


class Graph:
    """Handle of one network.  Node / edge descriptors are int32 arrays [K, 5] / [M, 4] in the
    header's rnn_node_desc / rnn_edge_desc field order."""

    def __init__(self, node_array, edge_array):
        self.lib = load_library()
        self.nodes = np.ascontiguousarray(node_array, dtype=np.int32).reshape(-1, 5)
        self.edges = np.ascontiguousarray(edge_array, dtype=np.int32).reshape(-1, 4)
        self.handle = C.c_void_p()
        _check(self.lib.rnn_graph_create(self.nodes.ctypes.data, self.nodes.shape[0],
                                         self.edges.ctypes.data if self.edges.size else None,
                                         self.edges.shape[0], C.byref(self.handle)))
        self.n_nodes, self.n_edges = self.nodes.shape[0], self.edges.shape[0]
        self.input_nodes = [k for k in range(self.n_nodes) if self.nodes[k, 0] == 0]
        self.output_nodes = [k for k in range(self.n_nodes) if self.nodes[k, 4] != 0]
        self._keep = None

    def close(self):
        if self.handle:
            self.lib.rnn_graph_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- host-only queries -------------------------------------------------------------
    def schedule(self):
        K, M = self.n_nodes, self.n_edges
        arrs = [np.zeros(K, np.int32) for _ in range(4)] + [np.zeros(max(M, 1), np.int32)]
        nc = C.c_int32()
        ptr = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
        _check(self.lib.rnn_graph_schedule(self.handle, *[ptr(a) for a in arrs], C.byref(nc)))
        return dict(node_comp=arrs[0].tolist(), node_level=arrs[1].tolist(), comp_level=arrs[2].tolist(),
                    comp_recurrent=arrs[3].tolist(), edge_class=arrs[4][:M].tolist(), n_comps=nc.value)

    def param_count(self):
        return int(_check(self.lib.rnn_param_count(self.handle)))

    def edge_param(self, m):
        off, ln = C.c_int64(), C.c_int64()
        _check(self.lib.rnn_edge_param_offset(self.handle, m, C.byref(off), C.byref(ln)))
        return off.value, ln.value

    def bias_param(self, k):
        off, ln = C.c_int64(), C.c_int64()
        _check(self.lib.rnn_bias_param_offset(self.handle, k, C.byref(off), C.byref(ln)))
        return off.value, ln.value

    def workspace_bytes(self, T, N):
        return int(_check(self.lib.rnn_workspace_bytes(self.handle, T, N)))

    def pack_params(self, weights, biases):
        """Per-edge / per-node float arrays -> flat float32 vector in the library's layout."""
        flat = np.zeros(self.param_count(), dtype=np.float32)
        for m, w in enumerate(weights):
            if w is not None:
                off, ln = self.edge_param(m)
                assert ln == w.size
                flat[off:off + ln] = np.asarray(w, dtype=np.float32).reshape(-1)
        for k, b in enumerate(biases):
            if b is not None:
                off, ln = self.bias_param(k)
                assert ln == b.size
                flat[off:off + ln] = np.asarray(b, dtype=np.float32).reshape(-1)
        return flat

    def unpack_params(self, flat):
        """Flat vector -> (per-edge list, per-node bias list) of views shaped like the parameters."""
        ws, bs = [], []
        for m in range(self.n_edges):
            off, ln = self.edge_param(m)
            if ln == 0:
                ws.append(None)
            elif self.edges[m, 3] == 0:
                ws.append(flat[off:off + ln].reshape(self.nodes[self.edges[m, 1], 2], self.nodes[self.edges[m, 0], 2]))
            else:
                ws.append(flat[off:off + ln])
        for k in range(self.n_nodes):
            off, ln = self.bias_param(k)
            bs.append(flat[off:off + ln] if ln else None)
        return ws, bs

    # ---- device calls (raw pointers; tensors are the caller's) ----------------------------
    def forward(self, d_weights, d_inputs, T, N, d_workspace, ws_bytes, stream=0):
        arr = (C.c_void_p * max(1, len(d_inputs)))(*d_inputs)
        _check(self.lib.rnn_forward(self.handle, d_weights, arr, T, N, d_workspace, ws_bytes, stream))

    def forward_range(self, d_weights, d_inputs, T, N, t_begin, t_end, d_workspace, ws_bytes, stream=0):
        arr = (C.c_void_p * max(1, len(d_inputs)))(*d_inputs)
        _check(self.lib.rnn_forward_range(self.handle, d_weights, arr, T, N, t_begin, t_end, d_workspace, ws_bytes, stream))

    def forward_static(self, d_weights, d_inputs, d_outputs, T, N, stream=0):
        arr = (C.c_void_p * max(1, len(d_inputs)))(*d_inputs)
        out = (C.c_void_p * max(1, len(d_outputs)))(*d_outputs)
        _check(self.lib.rnn_forward_static(self.handle, d_weights, arr, out, T, N, stream))

    def set_onehot_input(self, input_index, d_indices):
        _check(self.lib.rnn_set_onehot_input(self.handle, input_index, d_indices))

    def shift_window(self, frames, stream=0):
        _check(self.lib.rnn_shift_window(self.handle, frames, stream))

    def output_ptr(self, node):
        p = C.c_void_p()
        _check(self.lib.rnn_output(self.handle, node, C.byref(p)))
        return p.value

    def bptt(self, d_weights, d_targets, stream=0):
        arr = (C.c_void_p * max(1, len(d_targets)))(*d_targets)
        _check(self.lib.rnn_bptt(self.handle, d_weights, arr, stream))

    def state_grad_ptr(self, node):
        p = C.c_void_p()
        _check(self.lib.rnn_state_grad(self.handle, node, C.byref(p)))
        return p.value

    def specialise(self, N):
        return _check(self.lib.rnn_specialise(self.handle, N))

    def set_deterministic(self, on=True):
        _check(self.lib.rnn_set_deterministic(self.handle, 1 if on else 0))

    def check(self, stream=0):
        _check(self.lib.rnn_check(self.handle, stream))

    def step_build(self, node, backward=False):
        """(name of the step-kernel build that last ran the recurrent node of `node`, shared a chain launch)."""
        b = C.c_int32()
        _check(self.lib.rnn_step_build(self.handle, node, 1 if backward else 0, C.byref(b)))
        return BUILD_NAMES[b.value & 15], bool(b.value & 16)

    def step_build_has_helpers(self, node, backward=True):
        """True if the chain launch that last ran the recurrent node of `node` had helper members."""
        b = C.c_int32()
        _check(self.lib.rnn_step_build(self.handle, node, 1 if backward else 0, C.byref(b)))
        return bool(b.value & 32)

    def plan_work(self, T, N):
        fl, by = (C.c_int64 * 5)(), (C.c_int64 * 2)()
        _check(self.lib.rnn_plan_work(self.handle, T, N, fl, by))
        return dict(zip(("gemm_fwd", "gemm_bwd", "gemm_grad", "step_fwd", "step_bwd"), list(fl))), dict(step_fwd=by[0], step_bwd=by[1])

    def debug_read_control(self, nbytes=1024):
        buf = (C.c_ubyte * nbytes)()
        _check(self.lib.rnn_debug_read_control(self.handle, buf, nbytes))
        return bytes(buf)

    def profile_enable(self, class_mask):
        _check(self.lib.rnn_profile_enable(self.handle, class_mask))

    def profile_read(self, cls):
        ms, n = C.c_double(), C.c_int64()
        _check(self.lib.rnn_profile_read(self.handle, cls, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def grads(self, d_grads, want_loss=False, stream=0):
        if want_loss:
            loss = C.c_double()
            _check(self.lib.rnn_grads(self.handle, d_grads, C.byref(loss), stream))
            return loss.value
        _check(self.lib.rnn_grads(self.handle, d_grads, None, stream))
        return None
