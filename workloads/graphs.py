"""Network graphs and rollout patterns used as workloads.

Pure data: nodes (layers), edges (transformations) and the per-edge bridging
bit R(e) of a rollout pattern (Sec. 3, definition of rollout pattern and
window).  Nothing here evaluates a network; both the CPU oracle and the GPU
library are driven from these descriptions.

Conventions
-----------
* node 0.. are listed in a forward order (inputs first); the ids are plain
  indices into ``Graph.nodes``.
* an edge is a convolution (``kind='conv'``: kh, kw, stride, pad, optional
  nearest-neighbour upsampling of its result by ``up``), a dense map over the
  flattened (h, w, c) source (``'dense'``) or a global average pool followed by
  a dense map (``'gap_dense'``)  (App. A2: edges are convolutions or fully
  connected layers).
* ``bridge`` is R(e): 1 = the edge reads its source at frame t-1, 0 = at
  frame t.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Sequence

ACT_IDENTITY = 0
ACT_RELU = 1

KIND_CONV = "conv"
KIND_DENSE = "dense"
KIND_GAP_DENSE = "gap_dense"


@dataclass(frozen=True)
class Node:
    name: str
    channels: int
    height: int
    width: int
    act: int = ACT_RELU


@dataclass(frozen=True)
class Edge:
    src: int
    dst: int
    kind: str = KIND_CONV
    kh: int = 3
    kw: int = 3
    stride: int = 1
    pad: int = 1
    up: int = 1
    bridge: int = 1


@dataclass
class Graph:
    name: str
    nodes: List[Node]
    edges: List[Edge]
    batch: int = 1
    frames: int = 1          # T: number of frame updates of a rollout
    dtype: str = "f32"       # arithmetic/storage type on the GPU path: 'f32' | 'bf16'
    out_node: int = -1
    notes: dict = field(default_factory=dict)

    def with_pattern(self, bits: Sequence[int], name: str | None = None) -> "Graph":
        assert len(bits) == len(self.edges)
        edges = [replace(e, bridge=int(b)) for e, b in zip(self.edges, bits)]
        return Graph(name or self.name, list(self.nodes), edges, self.batch, self.frames,
                     self.dtype, self.out_node, dict(self.notes))

    def input_nodes(self) -> List[int]:
        has_in = {e.dst for e in self.edges}
        return [v for v in range(len(self.nodes)) if v not in has_in]


# ----------------------------------------------------------------------------
# rollout patterns
# ----------------------------------------------------------------------------

def streaming_pattern(g: Graph) -> List[int]:
    """R == 1 on every edge (the streaming rollout)."""
    return [1] * len(g.edges)


def sequential_pattern(g: Graph) -> List[int]:
    """Bridge only where a cycle forces it: self-edges and edges that point
    from a later node back to an earlier one (recurrent / top-down edges).
    All other edges, including those leaving the input and the head, stay
    inside the frame.  Unique for graphs whose only cycles are closed by such
    backward edges (Sec. 4, footnote on the most sequential rollout)."""
    return [1 if e.src >= e.dst else 0 for e in g.edges]


def hybrid_pattern(g: Graph) -> List[int]:
    """Bridging on alternate layers: an edge bridges iff it is a backward or
    self edge, or its target node has an even index (the head, whose index is
    the last one, follows the same parity rule only if it is even)."""
    last = len(g.nodes) - 1
    bits = []
    for e in g.edges:
        if e.src >= e.dst:
            bits.append(1)
        elif e.dst == last:
            bits.append(0)
        else:
            bits.append(1 if e.dst % 2 == 0 else 0)
    return bits


# ----------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------

def conv_out(size: int, k: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - k) // stride + 1


def _conv_edge(nodes, src, dst, k=3, bridge=1):
    """3x3-style convolution whose stride is the size ratio of its end points
    (App. A2: skip connections use stride input size / output size); a source
    smaller than the target becomes a 1x1 convolution followed by upsampling."""
    hs, hd = nodes[src].height, nodes[dst].height
    if hs >= hd:
        stride = hs // hd
        return Edge(src, dst, KIND_CONV, k, k, stride, k // 2, 1, bridge)
    up = hd // hs
    return Edge(src, dst, KIND_CONV, 1, 1, 1, 0, up, bridge)


def _stack(name, in_shape, channels, stride_at, skips, recurrent, n_classes, batch, frames,
           dtype, feedback=()):
    """Input -> chain of 3x3 conv nodes -> GAP+dense head, plus skip edges
    (i -> i+d for d in skips, conv nodes only), self-recurrent edges and
    top-down feedback edges."""
    c_in, h, w = in_shape
    nodes = [Node("in", c_in, h, w, ACT_IDENTITY)]
    for i, c in enumerate(channels, start=1):
        if i in stride_at:
            h, w = conv_out(h, 3, 2, 1), conv_out(w, 3, 2, 1)
        nodes.append(Node(f"n{i}", c, h, w, ACT_RELU))
    n = len(channels)
    nodes.append(Node("out", n_classes, 1, 1, ACT_IDENTITY))
    edges = []
    for i in range(1, n + 1):                      # forward chain
        edges.append(_conv_edge(nodes, i - 1, i))
    for d in skips:                                # skip edges between conv nodes
        for i in range(1, n + 1 - d):
            edges.append(_conv_edge(nodes, i, i + d))
    for i in recurrent:                            # self-recurrent edges
        edges.append(_conv_edge(nodes, i, i))
    for (s, t) in feedback:                        # top-down edges
        edges.append(_conv_edge(nodes, s, t))
    edges.append(Edge(n, n + 1, KIND_GAP_DENSE, 1, 1, 1, 0, 1, 1))
    return Graph(name, nodes, edges, batch, frames, dtype, out_node=n + 1)


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------

def tiny_sr(batch=2, frames=8) -> Graph:
    """Tiny skip+recurrent net, fp32: in(1@28x28) -> c1(8) -> c2(8, s2) ->
    c3(16, s2) -> fc(10, dense over the flattened 7x7x16 state); skip in->c2
    (s2) and a self-recurrent edge on c2."""
    nodes = [Node("in", 1, 28, 28, ACT_IDENTITY), Node("c1", 8, 28, 28), Node("c2", 8, 14, 14),
             Node("c3", 16, 7, 7), Node("fc", 10, 1, 1, ACT_IDENTITY)]
    edges = [
        Edge(0, 1, KIND_CONV, 3, 3, 1, 1), Edge(1, 2, KIND_CONV, 3, 3, 2, 1),
        Edge(2, 3, KIND_CONV, 3, 3, 2, 1), Edge(0, 2, KIND_CONV, 3, 3, 2, 1),
        Edge(2, 2, KIND_CONV, 3, 3, 1, 1), Edge(3, 4, KIND_DENSE, 7, 7, 1, 0),
    ]
    return Graph("tiny_sr", nodes, edges, batch, frames, "f32", out_node=4)


def cifar_sr(batch=64, frames=16) -> Graph:
    """CIFAR-shaped skip+recurrent net, bf16: 6 conv nodes at 32/32/64/64/128/128
    channels, stride 2 entering nodes 3 and 5, skips i->i+2, recurrent edges on
    nodes 2, 4, 6, GAP -> fc(10)."""
    return _stack("cifar_sr", (3, 32, 32), [32, 32, 64, 64, 128, 128], {3, 5}, (2,), (2, 4, 6),
                  10, batch, frames, "bf16")


def gtsrb_sr(batch=128, frames=32) -> Graph:
    """GTSRB-shaped deeper net, bf16: 10 conv nodes (64x3, 128x3, 256x4 channels;
    stride 2 entering nodes 4, 7, 10), skips i->i+2 and i->i+3, recurrent edges on
    every second node, top-down feedback 8->4 (1x1 conv + x2 upsampling),
    GAP -> fc(43)."""
    ch = [64, 64, 64, 128, 128, 128, 256, 256, 256, 256]
    return _stack("gtsrb_sr", (3, 48, 48), ch, {4, 7, 10}, (2, 3), (2, 4, 6, 8, 10), 43, batch,
                  frames, "bf16", feedback=((8, 4),))


def hires_sr(batch=1, frames=64) -> Graph:
    """High-resolution latency net, bf16: 12 conv nodes (64, 128, 256, 512
    channels, three nodes each; stride 2 entering nodes 4, 7, 10), skips i->i+2,
    self-recurrent edges on all conv nodes, GAP -> fc(10)."""
    ch = [64] * 3 + [128] * 3 + [256] * 3 + [512] * 3
    return _stack("hires_sr", (3, 256, 256), ch, {4, 7, 10}, (2,), tuple(range(1, 13)), 10,
                  batch, frames, "bf16")


def cifar_patterns(batch=64, frames=16):
    """The CIFAR-shaped graph under the sequential, hybrid and streaming
    patterns (identical nodes, edges, weights and inputs)."""
    g = cifar_sr(batch, frames)
    return {
        "sequential": g.with_pattern(sequential_pattern(g), "cifar_sr/sequential"),
        "hybrid": g.with_pattern(hybrid_pattern(g), "cifar_sr/hybrid"),
        "streaming": g.with_pattern(streaming_pattern(g), "cifar_sr/streaming"),
    }


# ----------------------------------------------------------------------------
# small graphs from the paper, used by the tests
# ----------------------------------------------------------------------------

def paper_sr_net(batch=1, frames=4, hw=8, c=4) -> Graph:
    """The skip+recurrent example net of Fig. 1: I -> H1 -> H2 -> O with a skip
    edge H1 -> O and a self-recurrent edge H1 -> H1 (all edges 3x3 convs of one
    size here; the rollout-theoretic quantities depend on the graph only)."""
    nodes = [Node("I", c, hw, hw, ACT_IDENTITY), Node("H1", c, hw, hw), Node("H2", c, hw, hw),
             Node("O", c, hw, hw, ACT_IDENTITY)]
    edges = [Edge(0, 1), Edge(1, 2), Edge(2, 3), Edge(1, 3), Edge(1, 1)]
    return Graph("paper_sr", nodes, edges, batch, frames, "f32", out_node=3)


def chain(n_edges: int, batch=1, frames=6, hw=6, c=3, k=3) -> Graph:
    """Pure feed-forward chain of ``n_edges`` convolutions."""
    nodes = [Node("in", c, hw, hw, ACT_IDENTITY)]
    nodes += [Node(f"h{i}", c, hw, hw) for i in range(1, n_edges + 1)]
    edges = [Edge(i, i + 1, KIND_CONV, k, k, 1, k // 2) for i in range(n_edges)]
    return Graph(f"chain{n_edges}", nodes, edges, batch, frames, "f32", out_node=n_edges)


def mnist_net(variant="SR", batch=128, frames=8) -> Graph:
    """The MNIST nets of App. A2: I (28,28,1) -> H1 (7,7,16) by a 7x7 stride-4
    convolution, H1 -> H2 (128) and H2 -> O (10) fully connected; variant 'S' adds
    the fully connected skip H1 -> O, 'SR' also the 3x3 self-recurrence H1 -> H1;
    'FF' has neither."""
    nodes = [Node("I", 1, 28, 28, ACT_IDENTITY), Node("H1", 16, 7, 7), Node("H2", 128, 1, 1),
             Node("O", 10, 1, 1, ACT_IDENTITY)]
    edges = [Edge(0, 1, KIND_CONV, 7, 7, 4, 3), Edge(1, 2, KIND_DENSE, 7, 7, 1, 0),
             Edge(2, 3, KIND_DENSE, 1, 1, 1, 0)]
    if variant in ("S", "SR"):
        edges.append(Edge(1, 3, KIND_DENSE, 7, 7, 1, 0))
    if variant == "SR":
        edges.append(Edge(1, 1, KIND_CONV, 3, 3, 1, 1))
    return Graph(f"mnist_{variant.lower()}", nodes, edges, batch, frames, "f32", out_node=3)


_DSR_ORDER = ["I", "H1", "H11", "H12", "H13", "H2", "H21", "H22", "H23", "HD", "O"]
_DSR_ADDED = ["H11", "H21", "H12", "H22", "H13", "H23"]     # DSR1, DSR2, ... DSR6 each add one
_DSR_EDGES = [("I", "H1"), ("H1", "H11"), ("H11", "H12"), ("H12", "H13"), ("H13", "H2"),
              ("H2", "H21"), ("H21", "H22"), ("H22", "H23"), ("H23", "HD"), ("HD", "O"),
              ("H1", "H12"), ("H1", "H13"), ("H1", "H2"), ("H11", "H13"), ("H11", "H2"),
              ("H12", "H2"), ("H2", "H22"), ("H2", "H23"), ("H2", "HD"), ("H21", "H23"),
              ("H21", "HD"), ("H22", "HD"), ("H1", "H1")]


def dsr_net(k: int, batch=64, frames=16, self_recurrence=True, n_classes=10) -> Graph:
    """The CIFAR10 family DSR0..DSR6 of App. A2: DSR0 is I -> H1 -> H2 -> HD -> O
    with a self-recurrent H1; every further network adds one hidden layer to a
    block (H11, H21, H12, H22, H13, H23) and is wired densely inside its block.
    Sizes: I (32,32,3), H1* (32,32,32), H2* (16,16,64), HD (4,4,512), O (10).
    I-H1 is a 5x5 convolution, all others 3x3 with stride = size ratio, HD-O is
    fully connected.  The GTSRB experiment uses DSR4 without the self-recurrence
    and 43 classes."""
    assert 0 <= k <= 6
    present = ["I", "H1", "H2", "HD", "O"] + _DSR_ADDED[:k]
    names = [n for n in _DSR_ORDER if n in present]
    idx = {n: i for i, n in enumerate(names)}

    def mk(n):
        if n == "I":
            return Node(n, 3, 32, 32, ACT_IDENTITY)
        if n == "O":
            return Node(n, n_classes, 1, 1, ACT_IDENTITY)
        if n == "HD":
            return Node(n, 512, 4, 4)
        if n.startswith("H1"):
            return Node(n, 32, 32, 32)
        return Node(n, 64, 16, 16)

    nodes = [mk(n) for n in names]
    edges = []
    for (a, b) in _DSR_EDGES:
        if a not in idx or b not in idx:
            continue
        if a == b and not self_recurrence:
            continue
        if (a, b) == ("I", "H1"):
            edges.append(Edge(idx[a], idx[b], KIND_CONV, 5, 5, 1, 2))
        elif (a, b) == ("HD", "O"):
            edges.append(Edge(idx[a], idx[b], KIND_DENSE, 4, 4, 1, 0))
        else:
            edges.append(_conv_edge(nodes, idx[a], idx[b]))
    return Graph(f"dsr{k}", nodes, edges, batch, frames, "bf16", out_node=idx["O"])


BENCH_CONFIGS = {
    "tiny_sr": tiny_sr,
    "cifar_sr": cifar_sr,
    "gtsrb_sr": gtsrb_sr,
    "hires_sr": hires_sr,
}

# the paper's own network shapes (App. A2) with the batch sizes of Tab. A1, as further workloads
PAPER_CONFIGS = {
    "mnist_ff": lambda: mnist_net("FF", batch=128, frames=16),
    "mnist_s": lambda: mnist_net("S", batch=128, frames=16),
    "mnist_sr": lambda: mnist_net("SR", batch=128, frames=16),
    **{f"dsr{k}": (lambda k=k: dsr_net(k, batch=64, frames=16)) for k in range(7)},
    "gtsrb_dsr4": lambda: dsr_net(4, batch=16, frames=16, self_recurrence=False, n_classes=43),
}


def flops_per_frame(g: Graph) -> int:
    """Nominal direct-convolution work of one frame update of the whole batch:
    2 * B * sum_e Ho*Wo*Cout*Cin*kh*kw, counting padding taps, and counting the
    convolution of an upsampling edge at its source resolution."""
    total = 0
    for e in g.edges:
        s, d = g.nodes[e.src], g.nodes[e.dst]
        if e.kind == KIND_CONV:
            ho, wo = d.height // e.up, d.width // e.up
            total += ho * wo * d.channels * s.channels * e.kh * e.kw
        elif e.kind == KIND_DENSE:
            total += s.height * s.width * s.channels * d.channels
        else:
            total += s.channels * d.channels
    return 2 * g.batch * total
