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


def random_graph(seed, dtype="bf16", cmul=None):
    rng = np.random.default_rng(seed)
    n_conv = int(rng.integers(3, 7))
    size = int(rng.choice([6, 8, 12, 16, 20, 24]))
    cmul = cmul or (32 if dtype == "bf16" else 4)
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


@pytest.mark.parametrize("seed", range(6))
def test_random_bf16_graph_channel_counts_off_the_tile_width(seed):
    # channel counts 8..72 in steps of 8: not multiples of the 32-channel tile (nor, half of them, of the
    # 16-channel pitch); the tile kernels pad their weights and bias and store only the channels that exist
    import paper_1806_04965_amd as sr
    g = random_graph(300 + seed, cmul=8)
    g = Graph(g.name + "_c8", [Node(n.name, n.channels * (1 + (i + seed) % 3) if 0 < i < len(g.nodes) - 1 else n.channels,
                                    n.height, n.width, n.act) for i, n in enumerate(g.nodes)],
              g.edges, g.batch, g.frames, g.dtype, g.out_node)
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=g.frames, recipe="uniform")
    ref = oracle_states(g, w, b, x, g.frames, "bf16")
    for label, opts in (("4-wave", {4: 1}), ("8-wave", {4: 2})):
        got, info, work = gpu_states_by_steps(g, w, b, x, g.frames, opts)
        worst = compare_all(got, ref, 2e-2, f"{g.name}/{label}")
        # the planner treats the node as it would with its channel count rounded up to whole tiles
        g32 = Graph(g.name + "_c32", [Node(n.name, (n.channels + 31) // 32 * 32 if 0 < i < len(g.nodes) - 1 else n.channels,
                                           n.height, n.width, n.act) for i, n in enumerate(g.nodes)],
                    g.edges, g.batch, g.frames, g.dtype, g.out_node)
        kinds = []
        for gg in (g, g32):
            wg, bg, _ = W.make_case(gg, seed=seed, frames=1)
            dev = sr.SrGraph(gg, options=opts)
            dev.set_parameters(wg, bg)
            kinds.append(dev.node_kernels())
            dev.close()
        print(f"[parity] {g.name}/{label}: worst {worst:.3e}, channels {[n.channels for n in g.nodes]}, kernels {kinds[0]}", flush=True)
        assert kinds[0] == kinds[1] and work["mfma_tiles"] > 0


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
