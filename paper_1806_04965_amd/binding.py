"""ctypes binding of include/sr.h.  Same names as the C ABI; argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

SR_F32, SR_BF16 = 0, 1
_KIND = {"conv": 0, "dense": 1, "gap_dense": 2}
SR_OPT_USE_HIPGRAPH, SR_OPT_FORCE_DIRECT, SR_OPT_FRAMES_PER_GRAPH = 0, 1, 2

EXPORTS = ["sr_analyze", "sr_count_valid_patterns", "sr_tableau", "sr_equally_model_parallel",
           "sr_pattern_count_bounds", "sr_graph_create", "sr_graph_set_weights",
           "sr_graph_set_bias", "sr_graph_configure", "sr_graph_info", "sr_reset", "sr_frame_step",
           "sr_frame_step_static", "sr_rollout", "sr_get_state", "sr_set_state", "sr_frame_index", "sr_frame_step_timed",
           "sr_graph_work", "sr_graph_traffic_model", "sr_graph_tile_kernel", "sr_graph_node_kernels", "sr_graph_health", "sr_window_gradients", "sr_rmsprop_step", "sr_graph_get_weights", "sr_graph_get_bias", "sr_graph_destroy", "sr_status_str", "sr_last_error"]


class NodeDesc(C.Structure):
    _fields_ = [("channels", C.c_int32), ("height", C.c_int32), ("width", C.c_int32), ("act", C.c_int32)]


class EdgeDesc(C.Structure):
    _fields_ = [("src", C.c_int32), ("dst", C.c_int32), ("kind", C.c_int32), ("kh", C.c_int32),
                ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32), ("upsample", C.c_int32),
                ("bridge", C.c_uint8)]


class SrError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name}: {detail}")
        self.status = status
        self.name = name


_lib = None


def lib_path() -> str:
    return os.path.join(HERE, "libsr.so")


def load_library():
    """Load libsr.so; fails loudly if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python -m paper_1806_04965_amd.build) first")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    P = C.POINTER
    lib.sr_analyze.argtypes = [i32, P(EdgeDesc), i32, P(i32), P(i32)]
    lib.sr_count_valid_patterns.argtypes = [i32, P(EdgeDesc), i32, P(C.c_uint64)]
    lib.sr_graph_create.argtypes = [P(NodeDesc), i32, P(EdgeDesc), i32, i32, i32, vp, P(vp)]
    lib.sr_graph_set_weights.argtypes = [vp, i32, P(C.c_float), C.c_size_t]
    lib.sr_graph_set_bias.argtypes = [vp, i32, P(C.c_float), C.c_size_t]
    lib.sr_graph_configure.argtypes = [vp, i32, i64]
    lib.sr_graph_info.argtypes = [vp, P(i32), P(i32), P(i32)]
    lib.sr_reset.argtypes = [vp, P(vp)]
    lib.sr_frame_step.argtypes = [vp, P(vp)]
    lib.sr_frame_step_static.argtypes = [vp, P(vp)]
    lib.sr_rollout.argtypes = [vp, P(vp), i32, i32, vp]
    lib.sr_get_state.argtypes = [vp, i32, vp, C.c_size_t]
    lib.sr_set_state.argtypes = [vp, i32, vp, C.c_size_t]
    lib.sr_frame_index.argtypes = [vp, P(i64)]
    lib.sr_frame_step_timed.argtypes = [vp, P(vp), P(C.c_float), P(i32), i32, P(i32)]
    lib.sr_graph_work.argtypes = [vp, P(C.c_double), P(i64), P(i64)]
    lib.sr_graph_traffic_model.argtypes = [vp, P(C.c_double)]
    lib.sr_graph_tile_kernel.argtypes = [vp, P(i32)]
    lib.sr_graph_node_kernels.argtypes = [vp, P(i32)]
    lib.sr_graph_health.argtypes = [vp, P(i64), P(i32)]
    lib.sr_window_gradients.argtypes = [vp, i32, P(vp), P(vp), vp, i32, vp, P(vp), P(vp)]
    lib.sr_rmsprop_step.argtypes = [vp, C.c_float, C.c_float, C.c_float, P(vp), P(vp)]
    lib.sr_graph_get_weights.argtypes = [vp, i32, P(C.c_float), C.c_size_t]
    lib.sr_graph_get_bias.argtypes = [vp, i32, P(C.c_float), C.c_size_t]
    lib.sr_graph_destroy.argtypes = [vp]
    lib.sr_graph_destroy.restype = None
    lib.sr_status_str.argtypes = [i32]
    lib.sr_status_str.restype = C.c_char_p
    lib.sr_last_error.argtypes = [vp]
    lib.sr_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("sr_graph_destroy", "sr_status_str", "sr_last_error"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _check(lib, status: int, handle=None):
    if status != 0:
        name = lib.sr_status_str(status).decode()
        detail = lib.sr_last_error(handle).decode()
        raise SrError(status, name, detail)


def _edge_array(edges):
    arr = (EdgeDesc * max(1, len(edges)))()
    for i, e in enumerate(edges):
        kind = _KIND[e.kind] if isinstance(e.kind, str) else int(e.kind)
        arr[i] = EdgeDesc(e.src, e.dst, kind, e.kh, e.kw, e.stride, e.pad, e.up, int(e.bridge))
    return arr


def analyze(n_nodes: int, edges) -> tuple:
    """sr_analyze: (levels, inference factor) of a network and rollout pattern (host only)."""
    lib = load_library()
    lv = (C.c_int32 * max(1, n_nodes))()
    f = C.c_int32(0)
    _check(lib, lib.sr_analyze(n_nodes, _edge_array(edges), len(edges), lv, C.byref(f)))
    return list(lv)[:n_nodes], f.value


def count_valid_patterns(n_nodes: int, edges) -> int:
    lib = load_library()
    c = C.c_uint64(0)
    _check(lib, lib.sr_count_valid_patterns(n_nodes, _edge_array(edges), len(edges), C.byref(c)))
    return c.value


def tableau(n_nodes: int, edges, W: int) -> list:
    """sr_tableau: inference tableau of the window of size W as W + 1 rows of n_nodes values."""
    lib = load_library()
    t = (C.c_int32 * max(1, (W + 1) * n_nodes))()
    _check(lib, lib.sr_tableau(n_nodes, _edge_array(edges), len(edges), W, t))
    flat = list(t)
    return [flat[i * n_nodes:(i + 1) * n_nodes] for i in range(W + 1)]


def equally_model_parallel(n_nodes: int, edges, bridge_a, bridge_b) -> bool:
    lib = load_library()
    a = (C.c_uint8 * max(1, len(edges)))(*[int(x) for x in bridge_a])
    b = (C.c_uint8 * max(1, len(edges)))(*[int(x) for x in bridge_b])
    eq = C.c_int32(0)
    _check(lib, lib.sr_equally_model_parallel(n_nodes, _edge_array(edges), len(edges), a, b, C.byref(eq)))
    return bool(eq.value)


def pattern_count_bounds(n_nodes: int, edges) -> tuple:
    """sr_pattern_count_bounds: (lower_forward, lower_cycles, upper) of Lemma 1."""
    lib = load_library()
    lo_f, lo_c, up = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0)
    _check(lib, lib.sr_pattern_count_bounds(n_nodes, _edge_array(edges), len(edges), C.byref(lo_f), C.byref(lo_c),
                                            C.byref(up)))
    return lo_f.value, lo_c.value, up.value


class SrGraph:
    """Owner of one sr_graph handle.  Tensors passed in are torch CUDA tensors (dense NHWC, graph
    dtype); they are kept alive by the caller until the stream has drained."""

    def __init__(self, graph, stream=None, dtype: Optional[str] = None, options: Optional[Dict[int, int]] = None):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.g = graph
        self.dtype = dtype or graph.dtype
        self.tdtype = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        self.stream = stream if stream is not None else torch.cuda.Stream()
        nodes = (NodeDesc * len(graph.nodes))()
        for i, n in enumerate(graph.nodes):
            nodes[i] = NodeDesc(n.channels, n.height, n.width, n.act)
        h = C.c_void_p()
        st = self.lib.sr_graph_create(nodes, len(graph.nodes), _edge_array(graph.edges), len(graph.edges),
                                      graph.batch, SR_BF16 if self.dtype == "bf16" else SR_F32,
                                      C.c_void_p(self.stream.cuda_stream), C.byref(h))
        _check(self.lib, st)
        self.h = h
        self.inputs = graph.input_nodes()
        for k, v in (options or {}).items():
            self.configure(k, v)

    # -- parameters -------------------------------------------------------
    def set_weights(self, edge: int, w: np.ndarray):
        w = np.ascontiguousarray(w, dtype=np.float32)
        _check(self.lib, self.lib.sr_graph_set_weights(self.h, edge, w.ctypes.data_as(C.POINTER(C.c_float)), w.size), self.h)

    def set_bias(self, node: int, b: np.ndarray):
        b = np.ascontiguousarray(b, dtype=np.float32)
        _check(self.lib, self.lib.sr_graph_set_bias(self.h, node, b.ctypes.data_as(C.POINTER(C.c_float)), b.size), self.h)

    def set_parameters(self, weights: Sequence[np.ndarray], biases: Sequence[np.ndarray]):
        for ei, w in enumerate(weights):
            self.set_weights(ei, w)
        for v, b in enumerate(biases):
            self.set_bias(v, b)

    def configure(self, option: int, value: int):
        _check(self.lib, self.lib.sr_graph_configure(self.h, option, value), self.h)

    def info(self):
        f = C.c_int32()
        lv = (C.c_int32 * len(self.g.nodes))()
        nl = C.c_int32()
        _check(self.lib, self.lib.sr_graph_info(self.h, C.byref(f), lv, C.byref(nl)), self.h)
        return {"inference_factor": f.value, "levels": list(lv), "launches_per_frame": nl.value}

    def work(self):
        fl, t, b = C.c_double(), C.c_int64(), C.c_int64()
        _check(self.lib, self.lib.sr_graph_work(self.h, C.byref(fl), C.byref(t), C.byref(b)), self.h)
        return {"flops_per_frame": fl.value, "mfma_tiles": t.value, "device_bytes": b.value}

    def traffic_model(self):
        """sr_graph_traffic_model: bytes per frame by class (no cache modelled)."""
        a = (C.c_double * 6)()
        _check(self.lib, self.lib.sr_graph_traffic_model(self.h, a), self.h)
        keys = ["states_read_once", "edge_source_reads", "tile_patch_loads", "weights_once", "tile_weight_reads", "states_written"]
        return dict(zip(keys, [float(x) for x in a]))

    def tile_kernel(self):
        k = C.c_int32()
        _check(self.lib, self.lib.sr_graph_tile_kernel(self.h, C.byref(k)), self.h)
        return k.value

    def health(self):
        """sr_graph_health: {'dependency_timeouts', 'dependency_driven'} (synchronises)."""
        t, d = C.c_int64(), C.c_int32()
        _check(self.lib, self.lib.sr_graph_health(self.h, C.byref(t), C.byref(d)), self.h)
        return {"dependency_timeouts": t.value, "dependency_driven": bool(d.value)}

    def node_kernels(self):
        """sr_graph_node_kernels: per node 0 input, 1 / 2 tile kernel (4 / 8 waves), 3 one thread per output, 4 head."""
        k = (C.c_int32 * len(self.g.nodes))()
        _check(self.lib, self.lib.sr_graph_node_kernels(self.h, k), self.h)
        return list(k)

    # -- frames -----------------------------------------------------------
    def _order(self, *tensors):
        """Stream ordering between torch and the library's stream: work already enqueued on torch's
        current stream (the producers of `tensors`) runs before what the library enqueues next, and
        torch's allocator is told that the tensors are in use on the library's stream."""
        cur = self.torch.cuda.current_stream()
        if cur != self.stream:
            self.stream.wait_stream(cur)
            for t in tensors:
                if t is not None:
                    t.record_stream(self.stream)

    def _publish(self):
        """The other direction: torch work enqueued from now on (on torch's current stream) runs after what
        the library has enqueued so far, so tensors the library has just been asked to fill can be used."""
        cur = self.torch.cuda.current_stream()
        if cur != self.stream:
            cur.wait_stream(self.stream)

    def _ptrs(self, tensors):
        arr = (C.c_void_p * max(1, len(self.inputs)))()
        for i, t in enumerate(tensors):
            if t is None:
                arr[i] = None
                continue
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype, "inputs must be dense device tensors of the graph dtype"
            arr[i] = t.data_ptr()
        self._order(*tensors)
        return arr

    def reset(self, inputs0=None):
        arr = self._ptrs(inputs0) if inputs0 is not None else None
        _check(self.lib, self.lib.sr_reset(self.h, arr), self.h)

    def frame_step(self, inputs_t):
        _check(self.lib, self.lib.sr_frame_step(self.h, self._ptrs(inputs_t)), self.h)

    def frame_step_static(self, inputs_t):
        _check(self.lib, self.lib.sr_frame_step_static(self.h, self._ptrs(inputs_t)), self.h)

    def frame_step_timed(self, inputs_t, cap=64):
        ms = (C.c_float * cap)()
        kind = (C.c_int32 * cap)()
        n = C.c_int32()
        _check(self.lib, self.lib.sr_frame_step_timed(self.h, self._ptrs(inputs_t), ms, kind, cap, C.byref(n)), self.h)
        return [(kind[i], ms[i]) for i in range(n.value)]

    def rollout(self, inputs, T: int, out_node: int = -1, outputs=None):
        """inputs: one tensor [T+1,B,H,W,C] per input node; outputs: tensor [T,B,H,W,C] or None."""
        optr = None
        if outputs is not None:
            assert outputs.is_cuda and outputs.is_contiguous() and outputs.dtype == self.tdtype
            optr = C.c_void_p(outputs.data_ptr())
            self._order(outputs)
        _check(self.lib, self.lib.sr_rollout(self.h, self._ptrs(inputs), T, out_node, optr), self.h)
        if outputs is not None:
            self._publish()

    def window_gradients(self, inputs, labels, W: int, out_node: Optional[int] = None, masks=None, into=None):
        """inputs: one float tensor [W+1,B,H,W,C] per input node; labels: int32 tensor [B] on the device;
        masks: None or {node: float tensor [W+1,B,H,W,C]} of dropout multipliers; into: None, or the tuple an
        earlier call returned, whose tensors are then written again (no allocation per step).
        Returns (loss tensor [1], dtheta list, dbias list) as device tensors (dbias of input nodes: None)."""
        torch = self.torch
        g = self.g
        out = g.out_node if out_node is None else out_node
        assert labels.is_cuda and labels.dtype == torch.int32 and labels.is_contiguous()
        if into is not None:
            loss, dth, dbs = into
            tarr = (C.c_void_p * len(g.edges))(*[t.data_ptr() for t in dth])
            barr = (C.c_void_p * len(g.nodes))(*[None if t is None else t.data_ptr() for t in dbs])
            return self._window_call(inputs, labels, W, out, masks, loss, dth, dbs, tarr, barr)
        loss = torch.empty(1, dtype=torch.float32, device="cuda")
        dth, dbs = [], []
        tarr = (C.c_void_p * len(g.edges))()
        for ei, e in enumerate(g.edges):
            s, d = g.nodes[e.src], g.nodes[e.dst]
            shape = {"conv": (e.kh, e.kw, s.channels, d.channels), "dense": (s.height, s.width, s.channels, d.channels),
                     "gap_dense": (1, 1, s.channels, d.channels)}[e.kind]
            t = torch.empty(shape, dtype=torch.float32, device="cuda")
            dth.append(t)
            tarr[ei] = t.data_ptr()
        barr = (C.c_void_p * len(g.nodes))()
        for v, n in enumerate(g.nodes):
            if v in self.inputs:
                dbs.append(None)
                barr[v] = None
                continue
            t = torch.empty(n.channels, dtype=torch.float32, device="cuda")
            dbs.append(t)
            barr[v] = t.data_ptr()
        return self._window_call(inputs, labels, W, out, masks, loss, dth, dbs, tarr, barr)

    def _window_call(self, inputs, labels, W, out, masks, loss, dth, dbs, tarr, barr):
        g = self.g
        torch = self.torch
        marr = None
        if masks:
            marr = (C.c_void_p * len(g.nodes))()
            for v in range(len(g.nodes)):
                t = masks.get(v)
                if t is not None:
                    n = g.nodes[v]
                    assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32
                    assert tuple(t.shape) == (W + 1, g.batch, n.height, n.width, n.channels), "mask shape"
                    marr[v] = t.data_ptr()
            self._order(*masks.values())
        self._order(labels, loss, *dth, *dbs)
        _check(self.lib, self.lib.sr_window_gradients(self.h, W, self._ptrs(inputs), marr, C.c_void_p(labels.data_ptr()), out,
                                                       C.c_void_p(loss.data_ptr()), tarr, barr), self.h)
        self._publish()
        return loss, dth, dbs

    def rmsprop_step(self, dtheta, dbias, lr: float, rho: float = 0.9, eps: float = 1e-7):
        """One RMSprop update of the graph's parameters from the gradients of window_gradients."""
        tarr = (C.c_void_p * len(dtheta))()
        for i, t in enumerate(dtheta):
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.torch.float32
            tarr[i] = t.data_ptr()
        barr = (C.c_void_p * len(self.g.nodes))()
        for v, t in enumerate(dbias):
            barr[v] = None if t is None else t.data_ptr()
        self._order(*dtheta, *dbias)
        _check(self.lib, self.lib.sr_rmsprop_step(self.h, lr, rho, eps, tarr, barr), self.h)

    def get_parameters(self):
        """(weights, biases) as the device holds them now, as float32 numpy arrays."""
        g = self.g
        ws, bs = [], []
        for ei, e in enumerate(g.edges):
            s, d = g.nodes[e.src], g.nodes[e.dst]
            shape = {"conv": (e.kh, e.kw, s.channels, d.channels), "dense": (s.height, s.width, s.channels, d.channels),
                     "gap_dense": (1, 1, s.channels, d.channels)}[e.kind]
            a = np.empty(shape, dtype=np.float32)
            _check(self.lib, self.lib.sr_graph_get_weights(self.h, ei, a.ctypes.data_as(C.POINTER(C.c_float)), a.size), self.h)
            ws.append(a)
        for v, n in enumerate(g.nodes):
            a = np.empty(n.channels, dtype=np.float32)
            _check(self.lib, self.lib.sr_graph_get_bias(self.h, v, a.ctypes.data_as(C.POINTER(C.c_float)), a.size), self.h)
            bs.append(a)
        return ws, bs

    def get_state(self, node: int):
        n = self.g.nodes[node]
        t = self.torch.empty((self.g.batch, n.height, n.width, n.channels), dtype=self.tdtype, device="cuda")
        self._order(t)
        _check(self.lib, self.lib.sr_get_state(self.h, node, C.c_void_p(t.data_ptr()), t.numel() * t.element_size()), self.h)
        self.stream.synchronize()
        return t

    def set_state(self, node: int, t):
        assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype
        self._order(t)
        _check(self.lib, self.lib.sr_set_state(self.h, node, C.c_void_p(t.data_ptr()), t.numel() * t.element_size()), self.h)

    def frame_index(self) -> int:
        f = C.c_int64()
        _check(self.lib, self.lib.sr_frame_index(self.h, C.byref(f)), self.h)
        return f.value

    def synchronize(self):
        self.stream.synchronize()

    def close(self):
        if getattr(self, "h", None):
            self.lib.sr_graph_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
