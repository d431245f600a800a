"""sr_frame_step_static, the entry point that allocates nothing (K-split partial sums in the
library's static device array): through the C ABI, against sr_frame_step on the graph's own
scratch, bit for bit, every node after every frame -- on two graphs in a row, the second smaller
than the first (the array keeps the first one's contents)."""
import numpy as np
import pytest

import workloads as W
from workloads.graphs import Node, Graph
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def hires_at(size, frames):
    g = W.hires_sr(batch=1, frames=frames)
    f = 256 // size
    nodes = [n if n.name == "out" else Node(n.name, n.channels, n.height // f, n.width // f, n.act) for n in g.nodes]
    return Graph(f"hires_sr@{size}", nodes, g.edges, 1, frames, "bf16", g.out_node)


def run_pair(g, seed, T, options=None):
    """T frames through sr_frame_step (own scratch) and through sr_frame_step_static; returns the
    number of tiles with and without K-split."""
    import paper_1806_04965_amd as sr
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=T)
    ins = g.input_nodes()
    xd = [to_device(x[v], g.dtype) for v in ins]
    own = sr.SrGraph(g, options=options)
    stat = sr.SrGraph(g, options=options)
    nosplit = sr.SrGraph(g, options={**(options or {}), 3: 0})
    for d in (own, stat, nosplit):
        d.set_parameters(w, b)
    tiles, tiles_nosplit = own.work()["mfma_tiles"], nosplit.work()["mfma_tiles"]
    nosplit.close()
    with pytest.raises(sr.SrError) as ei:          # not planned / reset yet
        stat.frame_step_static([xi[1] for xi in xd])
    assert ei.value.name == "SR_ERR_STATE"
    own.reset([xi[0] for xi in xd])
    stat.reset([xi[0] for xi in xd])
    for t in range(1, T + 1):
        own.frame_step([xi[t] for xi in xd])
        stat.frame_step_static([xi[t] for xi in xd])
        own.synchronize()
        stat.synchronize()
        for v in range(len(g.nodes)):
            a = own.get_state(v).float().cpu().numpy()
            s = stat.get_state(v).float().cpu().numpy()
            assert np.isfinite(s).all()
            np.testing.assert_array_equal(s, a, err_msg=f"{g.name} node {v} frame {t}")
        assert float(np.abs(stat.get_state(g.out_node).float().cpu().numpy()).max()) > 0
    assert stat.frame_index() == T
    own.close()
    stat.close()
    return tiles, tiles_nosplit


def test_static_scratch_matches_own_scratch_two_graphs_second_smaller():
    # first the full 256x256 high-resolution graph (about 300 parts, 38 MiB of partial sums), then
    # the same graph at 64x64 and the CIFAR-shaped one at batch 4, both much smaller
    t_big, t_big_ns = run_pair(W.hires_sr(batch=1, frames=3), seed=3, T=3)
    assert t_big > t_big_ns, "the first graph must have K-split tiles"
    t_small, t_small_ns = run_pair(hires_at(64, 3), seed=4, T=3)
    assert t_small > t_small_ns, "the second graph must have K-split tiles"
    assert t_small < t_big
    t_c, t_c_ns = run_pair(W.cifar_sr(batch=4, frames=4), seed=5, T=4)
    assert t_c > t_c_ns


def test_static_scratch_with_a_dependency_driven_graph():
    # sequential pattern: all update steps of a frame in one launch, ordered by completion counters
    import paper_1806_04965_amd as sr
    g0 = W.cifar_sr(batch=4, frames=3)
    g = g0.with_pattern(W.sequential_pattern(g0))
    dev = sr.SrGraph(g)
    w, b, _ = W.make_case(g, seed=7)
    dev.set_parameters(w, b)
    assert dev.health()["dependency_driven"]
    dev.close()
    run_pair(g, seed=7, T=3)


def test_static_scratch_with_the_eight_wave_kernel():
    run_pair(hires_at(64, 2), seed=6, T=2, options={4: 2})


def test_static_scratch_refuses_what_does_not_fit():
    # 200 nodes of 4x4 pixels, each fed by four 512-channel inputs through 3x3 edges: 200 one-tile nodes
    # with a contraction of 18432, every one cut into parts -- more partial sums than the array holds.
    # The call must say so, leave the graph as it was, and sr_frame_step must still serve it.
    import paper_1806_04965_amd as sr
    from workloads.graphs import Edge, ACT_IDENTITY
    n_in, n_hidden = 4, 200
    nodes = [Node(f"in{i}", 512, 4, 4, ACT_IDENTITY) for i in range(n_in)]
    nodes += [Node(f"h{i}", 32, 4, 4) for i in range(n_hidden)]
    nodes.append(Node("out", 10, 1, 1, ACT_IDENTITY))
    edges = [Edge(i, n_in + h) for h in range(n_hidden) for i in range(n_in)]
    edges.append(Edge(n_in, n_in + n_hidden, "gap_dense", 1, 1, 1, 0))
    g = Graph("many_deep_nodes", nodes, edges, 1, 1, "bf16", out_node=n_in + n_hidden)
    w, b, x = W.make_case(g, seed=7, frames=1)
    xd = [to_device(x[v], g.dtype) for v in g.input_nodes()]
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    dev.reset([xi[0] for xi in xd])
    with pytest.raises(sr.SrError) as ei:
        dev.frame_step_static([xi[1] for xi in xd])
    assert ei.value.name == "SR_ERR_ARG" and "static scratch holds" in str(ei.value), str(ei.value)
    assert dev.frame_index() == 0
    dev.frame_step([xi[1] for xi in xd])
    dev.synchronize()
    assert dev.frame_index() == 1
    assert float(dev.get_state(n_in + 1).float().abs().max()) > 0
    dev.close()
