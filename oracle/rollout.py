"""CPU oracle, part 2: the frame update of a rolled-out network, in float64.

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product path never does, and it
shares no code with the GPU library.

What it computes (Eq. 2 for the time index, App. A1.2 for the node map):

    x_v(t) = sigma_v( b_v + sum_{e=(u,v)} f_e(theta_e, x_u(t - R(e))) ),  t = 1..T

with x_v(0) = 0 for every node that has incoming edges, x_v(t) given for the
input nodes at all t = 0..T (initial state of Sec. 3; zero initial state per the
training details of App. A2), and frame t's result becoming frame t-1 of the
next shallow window (Sec. 4: inference with W = 1 windows).  Within a frame the
nodes are visited in the order of the inference tableau of the size-1 window
(Eq. 5), so an edge with R(e) = 0 reads a state already computed in this frame.

f_e is a cross-correlation ("convolution" in the deep-learning sense) with zero
padding, no dilation, no groups:
    y[b,ho,wo,co] = sum_{i,j,ci} theta[i,j,ci,co] * x[b, ho*s+i-p, wo*s+j-p, ci]
optionally followed by nearest-neighbour upsampling of y by an integer factor;
or a dense map over the flattened (h,w,c) source; or the mean over (h,w)
followed by a dense map over channels.  Arrays are NHWC.

Modes
  'f64'   everything in float64 (inputs, weights and biases are float32 values
          and therefore exact).
  'bf16'  the storage format of the GPU's bf16 path is emulated at its declared
          rounding points and nowhere else: weights are rounded once to bfloat16
          (round to nearest even), every state (inputs included) is rounded to
          bfloat16 when it is stored, i.e. after sigma; biases stay float32
          values; all sums are float64.

Pins (tests/test_oracle_rollout.py): the convolution against a pure-Python loop
nest on tiny inputs and against torch's CPU conv2d; 1x1 convolution == matmul;
dense == valid convolution with a kernel as large as the source; sum of edges
== one convolution over concatenated sources (App. A2); chain equivalence,
first-response frame, DAG settling time and a hand-expanded 3-node rollout
(Sec. 4); bfloat16 rounding on hand-picked values and against torch's
conversion.
"""
from __future__ import annotations

import numpy as np

from . import theory

ACT_IDENTITY = 0
ACT_RELU = 1


# ----------------------------------------------------------------------------
# bfloat16 storage emulation
# ----------------------------------------------------------------------------

def round_bf16(x):
    """Round float64 values to the nearest bfloat16 (8 significant bits), ties to
    even, returned as float64.  Done directly on the float64 value: x = m * 2^e
    with 0.5 <= |m| < 1, keep round-half-even(m * 2^8) / 2^8.  Values in the
    subnormal or overflow range of bfloat16 are not treated specially (states
    and weights here are O(1))."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


# ----------------------------------------------------------------------------
# edge transformations
# ----------------------------------------------------------------------------

def conv_out_size(size, k, stride, pad):
    return (size + 2 * pad - k) // stride + 1


def conv2d_nhwc(x, theta, stride, pad):
    """Cross-correlation with zero padding.  x: (B,H,W,Cin), theta: (kh,kw,Cin,Cout).
    The patches P[b,ho,wo,i,j,ci] = x[b, ho*s+i-p, wo*s+j-p, ci] are gathered
    explicitly (zeros outside the image) and contracted with theta over (i,j,ci)."""
    B, H, W, Cin = x.shape
    kh, kw, cin2, Cout = theta.shape
    assert Cin == cin2
    Ho = conv_out_size(H, kh, stride, pad)
    Wo = conv_out_size(W, kw, stride, pad)
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    P = np.empty((B, Ho, Wo, kh, kw, Cin), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            P[:, :, :, i, j, :] = xp[:, i:i + (Ho - 1) * stride + 1:stride,
                                     j:j + (Wo - 1) * stride + 1:stride, :]
    y = P.reshape(B * Ho * Wo, kh * kw * Cin) @ theta.reshape(kh * kw * Cin, Cout).astype(np.float64)
    return y.reshape(B, Ho, Wo, Cout)


def upsample_nearest(y, up):
    """y_up[b,h,w,c] = y[b, h // up, w // up, c]."""
    if up == 1:
        return y
    return np.repeat(np.repeat(y, up, axis=1), up, axis=2)


def dense_nhwc(x, theta):
    """y[b,0,0,co] = sum_{h,w,ci} theta[h,w,ci,co] * x[b,h,w,ci]."""
    B = x.shape[0]
    K = x.shape[1] * x.shape[2] * x.shape[3]
    y = x.reshape(B, K) @ theta.reshape(K, -1).astype(np.float64)
    return y.reshape(B, 1, 1, -1)


def gap_dense_nhwc(x, theta):
    """y[b,0,0,co] = sum_ci theta[0,0,ci,co] * mean_{h,w} x[b,h,w,ci]."""
    mean = x.mean(axis=(1, 2))
    y = mean @ theta.reshape(theta.shape[2], theta.shape[3]).astype(np.float64)
    return y.reshape(x.shape[0], 1, 1, -1)


def edge_transform(edge, theta, x):
    """y_e = f_e(theta_e, x_u) (App. A1.2)."""
    if edge.kind == "conv":
        return upsample_nearest(conv2d_nhwc(x, theta, edge.stride, edge.pad), edge.up)
    if edge.kind == "dense":
        return dense_nhwc(x, theta)
    if edge.kind == "gap_dense":
        return gap_dense_nhwc(x, theta)
    raise ValueError(f"unknown edge kind {edge.kind!r}")


def edge_output_shape(graph, edge):
    s = graph.nodes[edge.src]
    d = graph.nodes[edge.dst]
    if edge.kind == "conv":
        return (conv_out_size(s.height, edge.kh, edge.stride, edge.pad) * edge.up,
                conv_out_size(s.width, edge.kw, edge.stride, edge.pad) * edge.up, d.channels)
    return (1, 1, d.channels)


def activation(act, a):
    if act == ACT_RELU:
        return np.maximum(a, 0.0)
    if act == ACT_IDENTITY:
        return a
    raise ValueError(f"unknown activation {act}")


# ----------------------------------------------------------------------------
# the rollout
# ----------------------------------------------------------------------------

class ShapeError(ValueError):
    """An edge's result does not have the shape of its target node."""


def check_graph(graph):
    """Reject what is not a network, an invalid rollout pattern, or edges whose
    results cannot be summed at their target (App. A1.2: compatible dimensions)."""
    n = len(graph.nodes)
    el = [(e.src, e.dst) for e in graph.edges]
    theory.check_network(n, el)
    R = [e.bridge for e in graph.edges]
    theory.check_rollout(n, el, R)
    for e in graph.edges:
        d = graph.nodes[e.dst]
        if edge_output_shape(graph, e) != (d.height, d.width, d.channels):
            raise ShapeError(f"edge {e.src}->{e.dst}: result {edge_output_shape(graph, e)} "
                             f"!= node {(d.height, d.width, d.channels)}")


def frame_schedule(graph):
    """Nodes grouped by the update step of the frame at which they are computed
    (tableau of the size-1 window); inputs are level 0."""
    n = len(graph.nodes)
    el = [(e.src, e.dst) for e in graph.edges]
    lv = theory.levels(n, el, [e.bridge for e in graph.edges])
    F = max(lv)
    return [[v for v in range(n) if lv[v] == step] for step in range(0, F + 1)]


class Rollout:
    """State of a stream: the frame most recently computed.  ``step`` advances one
    frame; ``run`` advances T frames and collects what the caller asks for."""

    def __init__(self, graph, weights, biases, mode="f64"):
        assert mode in ("f64", "bf16")
        check_graph(graph)
        self.g = graph
        self.mode = mode
        self.store = round_bf16 if mode == "bf16" else (lambda a: np.asarray(a, dtype=np.float64))
        self.theta = [self.store(w) for w in weights]
        self.bias = [np.asarray(b, dtype=np.float64) for b in biases]
        self.schedule = frame_schedule(graph)
        self.inputs = self.schedule[0]
        self.src_edges = [[ei for ei, e in enumerate(graph.edges) if e.dst == v]
                          for v in range(len(graph.nodes))]
        self.edge_evaluations = 0
        self.X = None

    def reset(self, inputs0):
        """Frame 0: given states for the input nodes, zeros elsewhere."""
        g = self.g
        self.X = []
        for v, n in enumerate(g.nodes):
            if v in self.inputs:
                self.X.append(self.store(inputs0[v]))
            else:
                self.X.append(np.zeros((g.batch, n.height, n.width, n.channels)))
        self.edge_evaluations = 0

    def step(self, inputs_t):
        """One frame update: X' from X (previous frame) and this frame's inputs."""
        g = self.g
        Xn = [None] * len(g.nodes)
        for v in self.inputs:
            Xn[v] = self.store(inputs_t[v])
        for level in self.schedule[1:]:
            for v in level:
                n = g.nodes[v]
                acc = np.zeros((g.batch, n.height, n.width, n.channels)) + self.bias[v]
                for ei in self.src_edges[v]:
                    e = g.edges[ei]
                    src = self.X[e.src] if e.bridge == 1 else Xn[e.src]
                    acc = acc + edge_transform(e, self.theta[ei], src)
                    self.edge_evaluations += 1
                Xn[v] = self.store(activation(n.act, acc))
        self.X = Xn
        return Xn

    def run(self, inputs, T=None, keep=None):
        """inputs[v]: (T+1,B,H,W,C).  Returns {v: (T,B,H,W,C)} for v in ``keep``
        (default: the graph's output node), frames 1..T."""
        g = self.g
        T = g.frames if T is None else T
        keep = [g.out_node] if keep is None else list(keep)
        self.reset({v: inputs[v][0] for v in self.inputs})
        out = {v: [] for v in keep}
        for t in range(1, T + 1):
            X = self.step({v: inputs[v][t] for v in self.inputs})
            for v in keep:
                out[v].append(X[v])
        return {v: np.stack(a) for v, a in out.items()}


def rollout(graph, weights, biases, inputs, T=None, keep=None, mode="f64"):
    return Rollout(graph, weights, biases, mode).run(inputs, T, keep)


# ----------------------------------------------------------------------------
# single-element evaluation (sampled checks at sizes where a full frame is slow)
# ----------------------------------------------------------------------------

def node_element(graph, weights, biases, v, b, h, w, c, prev_states, cur_states, mode="f64"):
    """x_v(t)[b,h,w,c] from explicit loops over edges, taps and channels, given the
    previous frame's states (read by bridging edges) and the current frame's
    (read by non-bridging edges).  States and weights are taken as stored (the
    caller passes bfloat16-exact arrays in 'bf16' mode); only the result is
    rounded."""
    g = graph
    n = g.nodes[v]
    acc = float(biases[v][c])
    for ei, e in enumerate(g.edges):
        if e.dst != v:
            continue
        x = prev_states[e.src] if e.bridge == 1 else cur_states[e.src]
        th = np.asarray(weights[ei], dtype=np.float64)
        if mode == "bf16":
            th = round_bf16(th)
        s = g.nodes[e.src]
        if e.kind == "conv":
            ho, wo = h // e.up, w // e.up
            for i in range(e.kh):
                for j in range(e.kw):
                    iy, ix = ho * e.stride + i - e.pad, wo * e.stride + j - e.pad
                    if 0 <= iy < s.height and 0 <= ix < s.width:
                        acc += float(np.dot(np.asarray(x[b, iy, ix, :], dtype=np.float64), th[i, j, :, c]))
        elif e.kind == "dense":
            acc += float(np.sum(np.asarray(x[b], dtype=np.float64) * th[:, :, :, c]))
        elif e.kind == "gap_dense":
            mean = np.asarray(x[b], dtype=np.float64).mean(axis=(0, 1))
            acc += float(np.dot(mean, th[0, 0, :, c]))
        else:
            raise ValueError(e.kind)
    val = max(acc, 0.0) if n.act == ACT_RELU else acc
    return float(round_bf16(val)) if mode == "bf16" else val
