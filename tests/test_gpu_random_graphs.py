"""GPU parity on seeded random networks: random shapes, kernel sizes, strides, up-sampling, channel
counts, skip / recurrent / feedback edges and random valid rollout patterns, through both tile kernels
and the direct kernel, against the CPU oracle."""
import numpy as np
import pytest

import workloads as W
from workloads.graphs import Node, Edge, Graph, ACT_IDENTITY, ACT_RELU
from oracle import theory as th
from gpu_util import gpu_states_by_steps, oracle_states, compare_all

pytestmark = pytest.mark.gpu


def random_graph(seed, dtype="bf16"):
    rng = np.random.default_rng(seed)
    n_conv = int(rng.integers(3, 7))
    size = int(rng.choice([6, 8, 12, 16, 20, 24]))
    cmul = 32 if dtype == "bf16" else 4
    nodes = [Node("in", int(rng.choice([1, 3, 4])), size, size, ACT_IDENTITY)]
    sizes = [size]
    for i in range(n_conv):
        s = int(rng.choice([1, 1, 2, 4])) if sizes[-1] % 4 == 0 and sizes[-1] >= 8 else (2 if sizes[-1] % 2 == 0 and sizes[-1] >= 4 and rng.random() < 0.3 else 1)
        sizes.append(sizes[-1] // s)
        nodes.append(Node(f"n{i + 1}", cmul * int(rng.integers(1, 4)), sizes[-1], sizes[-1], ACT_RELU))
    nodes.append(Node("out", int(rng.choice([5, 10, 40])), 1, 1, ACT_IDENTITY))

    def conv(a, b, bridge):
        ha, hb = nodes[a].height, nodes[b].height
        if ha >= hb:
            k = int(rng.choice([1, 3, 3, 5]))
            return Edge(a, b, "conv", k, k, ha // hb, k // 2, 1, bridge)
        return Edge(a, b, "conv", 1, 1, 1, 0, hb // ha, bridge)

    edges = [conv(i, i + 1, 1) for i in range(n_conv)]
    for _ in range(int(rng.integers(1, 5))):
        a, b = sorted(int(v) for v in rng.integers(1, n_conv + 1, size=2))
        kind = rng.random()
        if kind < 0.4 and a != b:
            edges.append(conv(a, b, 1))          # skip
        elif kind < 0.7:
            edges.append(conv(b, b, 1))          # recurrent
        elif a != b:
            edges.append(conv(b, a, 1))          # feedback (up-sampling 1x1 if needed)
    last = n_conv
    head = "gap_dense" if rng.random() < 0.5 or nodes[last].height * nodes[last].width * nodes[last].channels > 12000 else "dense"
    if head == "dense":
        edges.append(Edge(last, n_conv + 1, "dense", nodes[last].height, nodes[last].width, 1, 0, 1, 1))
    else:
        edges.append(Edge(last, n_conv + 1, "gap_dense", 1, 1, 1, 0, 1, 1))
    g = Graph(f"random{seed}", nodes, edges, int(rng.integers(1, 6)), 4, dtype, out_node=n_conv + 1)
    # a random valid pattern: start from streaming, clear bits while the pattern stays valid
    pairs = [(e.src, e.dst) for e in g.edges]
    bits = [1] * len(pairs)
    for i in rng.permutation(len(pairs)):
        if rng.random() < 0.4:
            trial = list(bits)
            trial[i] = 0
            if th.is_valid(len(nodes), pairs, trial):
                bits = trial
    return g.with_pattern(bits)


@pytest.mark.parametrize("seed", range(12))
def test_random_bf16_graph_both_tile_kernels(seed):
    g = random_graph(100 + seed)
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=g.frames, recipe="uniform")
    ref = oracle_states(g, w, b, x, g.frames, "bf16")
    for label, opts in (("4-wave", {4: 1}), ("8-wave", {4: 2})):
        got, info, work = gpu_states_by_steps(g, w, b, x, g.frames, opts)
        worst = compare_all(got, ref, 2e-2, f"{g.name}/{label}")
        print(f"[parity] {g.name}/{label}: worst {worst:.3e}, F(R)={info['inference_factor']}, tiles={work['mfma_tiles']}, "
              f"launches/frame={info['launches_per_frame']}", flush=True)


def scaled_up(g, seed):
    """The same topology, strides and pattern with 2-4x larger images and a batch of 6..32: hundreds
    of tiles, tiles that span several images, every XCD's share non-empty.  A dense head becomes
    GAP + dense (its flattened input would no longer fit a head item)."""
    rng = np.random.default_rng(seed + 7)
    f = int(rng.choice([2, 2, 4]))
    nodes = [Node(n.name, n.channels, n.height * f if n.height > 1 else 1, n.width * f if n.width > 1 else 1, n.act)
             for n in g.nodes]
    edges = [Edge(e.src, e.dst, "gap_dense", 1, 1, 1, 0, 1, e.bridge) if e.kind == "dense" else e for e in g.edges]
    return Graph(g.name + "_big", nodes, edges, int(rng.integers(6, 33)), 3, g.dtype, out_node=g.out_node)


@pytest.mark.parametrize("seed", [401, 405, 412, 429])
def test_random_bf16_graph_scaled_up(seed):
    g = scaled_up(random_graph(seed), seed)
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=g.frames, recipe="uniform")
    ref = oracle_states(g, w, b, x, g.frames, "bf16")
    for label, opts in (("4-wave", {4: 1}), ("8-wave", {4: 2})):
        got, info, work = gpu_states_by_steps(g, w, b, x, g.frames, opts)
        worst = compare_all(got, ref, 2e-2, f"{g.name}/{label}")
        print(f"[parity] {g.name}/{label}: worst {worst:.3e}, B={g.batch}, tiles={work['mfma_tiles']}", flush=True)


@pytest.mark.parametrize("seed", range(4))
def test_random_fp32_graph_direct_kernel(seed):
    g = random_graph(200 + seed, dtype="f32")
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=g.frames, recipe="uniform")
    ref = oracle_states(g, w, b, x, g.frames, "f64")
    got, info, work = gpu_states_by_steps(g, w, b, x, g.frames, None)
    compare_all(got, ref, 1e-4, g.name)
