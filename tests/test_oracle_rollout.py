"""Pins for the oracle's frame update against library routines, closed forms,
brute force and the behaviour the paper states (Sec. 4, App. A1.2, App. A2)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import rollout as orc
from oracle import theory as th
import workloads as W
from workloads.graphs import Node, Edge, Graph, ACT_IDENTITY, ACT_RELU

HERE = os.path.dirname(os.path.abspath(__file__))


def loop_conv(x, theta, stride, pad):
    """Pure-Python loop nest of the cross-correlation definition."""
    B, H, Wd, Cin = x.shape
    kh, kw, _, Cout = theta.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    y = np.zeros((B, Ho, Wo, Cout))
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Cout):
                    s = 0.0
                    for i in range(kh):
                        for j in range(kw):
                            iy, ix = ho * stride + i - pad, wo * stride + j - pad
                            if iy < 0 or iy >= H or ix < 0 or ix >= Wd:
                                continue
                            for ci in range(Cin):
                                s += theta[i, j, ci, co] * x[b, iy, ix, ci]
                    y[b, ho, wo, co] = s
    return y


@pytest.mark.parametrize("k,stride,pad,H,Wd", [(3, 1, 1, 5, 6), (3, 2, 1, 6, 6), (3, 2, 1, 7, 5),
                                               (1, 1, 0, 4, 3), (5, 1, 2, 6, 6), (7, 4, 3, 12, 12),
                                               (3, 4, 1, 8, 8), (3, 1, 0, 5, 5)])
def test_conv_against_loop_nest(k, stride, pad, H, Wd):
    rng = np.random.default_rng(k * 100 + stride * 10 + pad)
    x = rng.standard_normal((2, H, Wd, 3))
    theta = rng.standard_normal((k, k, 3, 4))
    np.testing.assert_allclose(orc.conv2d_nhwc(x, theta, stride, pad), loop_conv(x, theta, stride, pad),
                               rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 1, 0), (5, 1, 2), (7, 4, 3), (3, 4, 1)])
def test_conv_against_torch_conv2d(k, stride, pad):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 16, 12, 5))
    theta = rng.standard_normal((k, k, 5, 7))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2),
                                     torch.from_numpy(theta).permute(3, 2, 0, 1),
                                     stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()
    got = orc.conv2d_nhwc(x, theta, stride, pad)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-11)


def test_asymmetric_kernel_is_not_transposed():
    # a single non-zero tap at (i=0, j=2) must shift the image up by pad and left by pad-2
    x = np.arange(2 * 5 * 5 * 1, dtype=np.float64).reshape(2, 5, 5, 1)
    theta = np.zeros((3, 3, 1, 1))
    theta[0, 2, 0, 0] = 1.0
    y = orc.conv2d_nhwc(x, theta, 1, 1)
    assert y[0, 1, 1, 0] == x[0, 0, 2, 0]       # (ho + 0 - 1, wo + 2 - 1)
    assert y[1, 4, 0, 0] == x[1, 3, 1, 0]
    assert y[0, 0, 0, 0] == 0.0                 # row -1 is padding


def test_one_by_one_conv_is_matmul_and_dense_is_full_valid_conv():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 4, 5, 6))
    t1 = rng.standard_normal((1, 1, 6, 3))
    np.testing.assert_allclose(orc.conv2d_nhwc(x, t1, 1, 0), x @ t1[0, 0], rtol=1e-12, atol=1e-12)
    td = rng.standard_normal((4, 5, 6, 3))
    np.testing.assert_allclose(orc.dense_nhwc(x, td), orc.conv2d_nhwc(x, td, 1, 0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.dense_nhwc(x, td)[:, 0, 0, :],
                               np.einsum("bhwc,hwco->bo", x, td), rtol=1e-12, atol=1e-12)


def test_gap_dense_closed_forms():
    rng = np.random.default_rng(3)
    theta = rng.standard_normal((1, 1, 4, 3))
    const = np.ones((2, 3, 5, 4)) * np.array([1.0, -2.0, 0.5, 4.0])
    np.testing.assert_allclose(orc.gap_dense_nhwc(const, theta)[0, 0, 0],
                               np.array([1.0, -2.0, 0.5, 4.0]) @ theta[0, 0], rtol=1e-12)
    x = rng.standard_normal((2, 3, 5, 4))
    # mean then dense == dense with every tap equal to theta / (H*W)
    td = np.broadcast_to(theta / 15.0, (3, 5, 4, 3))
    np.testing.assert_allclose(orc.gap_dense_nhwc(x, theta), orc.dense_nhwc(x, td), rtol=1e-12, atol=1e-12)


def test_upsampled_1x1_conv_commutes_with_upsampling_the_source():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 3, 4, 5))
    theta = rng.standard_normal((1, 1, 5, 2))
    e = Edge(0, 1, "conv", 1, 1, 1, 0, 2, 1)
    a = orc.edge_transform(e, theta, x)
    b = orc.conv2d_nhwc(orc.upsample_nearest(x, 2), theta, 1, 0)
    assert a.shape == (2, 6, 8, 2)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)
    assert a[1, 5, 7, 1] == a[1, 4, 6, 1] and a[0, 2, 3, 0] == orc.conv2d_nhwc(x, theta, 1, 0)[0, 1, 1, 0]


def test_bf16_rounding_hand_values_and_torch():
    cases = [(1.0, 1.0), (1.0 + 2.0 ** -8, 1.0), (1.0 + 3 * 2.0 ** -8, 1.015625),
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0078125), (3.14159, 3.140625), (-0.3, -0.30078125),
             (0.0, 0.0), (255.5, 256.0), (-1.0 - 2.0 ** -8, -1.0), (2.0 ** -20 * 1.00390625, 2.0 ** -20)]
    for x, want in cases:
        assert float(orc.round_bf16(x)) == want, (x, want)
    rng = np.random.default_rng(0)
    v = (rng.standard_normal(20000) * 10.0 ** rng.uniform(-3, 3, 20000)).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.round_bf16(v.astype(np.float64)), ref)


# ----------------------------------------------------------------------------
# rollout semantics
# ----------------------------------------------------------------------------

def feed_forward(g, weights, biases, x):
    """Plain layer-by-layer evaluation of a chain (no time): the sequential value."""
    cur = np.asarray(x, dtype=np.float64)
    for ei, e in enumerate(g.edges):
        n = g.nodes[e.dst]
        cur = orc.activation(n.act, orc.edge_transform(e, np.asarray(weights[ei], np.float64), cur) + biases[e.dst])
    return cur


def test_chain_streaming_is_sequential_delayed_by_L():
    # Sec. 4: without skip or recurrent edges streaming and sequential are the same function, pipelined
    L, T = 3, 7
    g = W.chain(L, batch=2, frames=T)
    w, b, x = W.make_case(g, seed=1, bias_scale=0.3)
    gs = g.with_pattern(W.streaming_pattern(g))
    gq = g.with_pattern(W.sequential_pattern(g))
    out_s = orc.rollout(gs, w, b, x)[g.out_node]
    out_q = orc.rollout(gq, w, b, x)[g.out_node]
    for t in range(1, T + 1):
        np.testing.assert_allclose(out_q[t - 1], feed_forward(g, w, b, x[0][t]), rtol=1e-12, atol=1e-12)
        if t >= L:
            np.testing.assert_allclose(out_s[t - 1], feed_forward(g, w, b, x[0][t - L]), rtol=1e-12, atol=1e-12)
    assert th.inference_factor(len(g.nodes), [(e.src, e.dst) for e in g.edges], W.sequential_pattern(g)) == L


@pytest.mark.parametrize("make", [W.tiny_sr, lambda: W.paper_sr_net(2, 6), lambda: W.mnist_net("SR", 2, 5),
                                  lambda: W.cifar_sr(1, 9)])
def test_first_response_frame_is_shortest_path(make):
    # Sec. 4: the streaming rollout first responds after shortest-path-many frames
    g = make()
    g = g.with_pattern(W.streaming_pattern(g))
    w, b, x = W.make_case(g, seed=2)
    n = len(g.nodes)
    el = [(e.src, e.dst) for e in g.edges]
    Lmin = th.shortest_path_length(n, el, g.out_node)
    T = Lmin + 2
    out = orc.rollout(g, w, b, x, T=T)[g.out_node]
    for t in range(1, T + 1):
        if t < Lmin:
            assert np.all(out[t - 1] == 0.0), t
    assert np.any(out[Lmin - 1] != 0.0)
    # changing only x(0) changes the output first at frame Lmin
    x2 = {v: a.copy() for v, a in x.items()}
    for v in x2:
        x2[v][0] += 1.0
    out2 = orc.rollout(g, w, b, x2, T=T)[g.out_node]
    for t in range(1, Lmin):
        np.testing.assert_array_equal(out[t - 1], out2[t - 1])
    assert np.any(out[Lmin - 1] != out2[Lmin - 1])


def test_sequential_pattern_responds_in_first_frame():
    g = W.paper_sr_net(1, 3)
    g = g.with_pattern(W.sequential_pattern(g))
    w, b, x = W.make_case(g, seed=3)
    out = orc.rollout(g, w, b, x)[g.out_node]
    assert np.any(out[0] != 0.0)


def test_dag_constant_input_settles_at_longest_path():
    # Sec. 4: after longest-path-many frames the streaming rollout uses the full network.
    # DAG with skips: in -> a -> b -> c, in -> b, a -> c
    nodes = [Node("in", 2, 6, 6, ACT_IDENTITY), Node("a", 3, 6, 6), Node("b", 3, 3, 3), Node("c", 4, 3, 3)]
    edges = [Edge(0, 1), Edge(1, 2, stride=2), Edge(2, 3), Edge(0, 2, stride=2), Edge(1, 3, stride=2)]
    g = Graph("dag", nodes, edges, batch=2, frames=6, out_node=3)
    w, b, _ = W.make_case(g, seed=4, bias_scale=0.2)
    rng = np.random.default_rng(0)
    x0 = rng.standard_normal((2, 6, 6, 2)).astype(np.float32)
    x = {0: np.stack([x0] * 7)}
    gs = g.with_pattern(W.streaming_pattern(g))
    gq = g.with_pattern(W.sequential_pattern(g))
    seq = orc.rollout(gq, w, b, x, keep=[1, 2, 3])
    st = orc.rollout(gs, w, b, x, keep=[1, 2, 3])
    longest = {1: 1, 2: 2, 3: 3}
    for v in (1, 2, 3):
        for t in range(1, 7):
            same = np.allclose(st[v][t - 1], seq[v][0], rtol=1e-12, atol=1e-12)
            if t >= longest[v]:
                assert same, (v, t)
        assert not np.allclose(st[3][1], seq[3][0])        # frame 2 < longest path 3: not yet settled


def test_cyclic_graph_patterns_share_the_fixed_point():
    # all rollout patterns of one network share x_v = sigma(b + sum f_e(x_u)); with contractive
    # weights streaming and sequential converge to it under constant input
    g = W.paper_sr_net(1, 60)
    w, b, _ = W.make_case(g, seed=5, bias_scale=0.1, gain=0.5)
    x0 = np.random.default_rng(1).standard_normal((1, 8, 8, 4)).astype(np.float32)
    x = {0: np.stack([x0] * 61)}
    a = orc.rollout(g.with_pattern(W.streaming_pattern(g)), w, b, x)[3][-1]
    c = orc.rollout(g.with_pattern(W.sequential_pattern(g)), w, b, x)[3][-1]
    np.testing.assert_allclose(a, c, rtol=1e-9, atol=1e-9)


def test_hand_expanded_three_node_rollout():
    with open(os.path.join(HERE, "golden", "three_node_rollout.json")) as f:
        gold = json.load(f)
    nodes = [Node("in", 1, 1, 1, ACT_IDENTITY), Node("a", 1, 1, 1, ACT_RELU), Node("b", 1, 1, 1, ACT_RELU)]
    base = [Edge(0, 1, "conv", 1, 1, 1, 0), Edge(1, 2, "conv", 1, 1, 1, 0), Edge(0, 2, "conv", 1, 1, 1, 0),
            Edge(1, 1, "conv", 1, 1, 1, 0)]
    wt = [np.full((1, 1, 1, 1), gold["weights"][k], np.float32) for k in gold["edge_order"]]
    bias = [np.zeros(1, np.float32), np.array([gold["bias"]["a"]], np.float32),
            np.array([gold["bias"]["b"]], np.float32)]
    x = {0: np.array(gold["x"], np.float32).reshape(5, 1, 1, 1, 1)}
    for name, case in gold["cases"].items():
        g = Graph(name, nodes, base, batch=1, frames=4, out_node=2).with_pattern(case["R"])
        out = orc.rollout(g, wt, bias, x, keep=[1, 2])
        assert out[1].ravel().tolist() == case["a"], name
        assert out[2].ravel().tolist() == case["b"], name


def test_sum_of_edges_equals_conv_over_concatenation():
    # App. A2: summing incoming transformations == one convolution on the concatenated inputs
    rng = np.random.default_rng(6)
    xa, xb = rng.standard_normal((2, 6, 6, 3)), rng.standard_normal((2, 6, 6, 5))
    ta, tb = rng.standard_normal((3, 3, 3, 4)), rng.standard_normal((3, 3, 5, 4))
    lhs = orc.conv2d_nhwc(xa, ta, 1, 1) + orc.conv2d_nhwc(xb, tb, 1, 1)
    rhs = orc.conv2d_nhwc(np.concatenate([xa, xb], -1), np.concatenate([ta, tb], 2), 1, 1)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    nodes = [Node("i1", 3, 6, 6, ACT_IDENTITY), Node("i2", 5, 6, 6, ACT_IDENTITY), Node("o", 4, 6, 6)]
    g = Graph("two_in", nodes, [Edge(0, 2), Edge(1, 2)], batch=2, frames=1, out_node=2)
    bias = [np.zeros(3), np.zeros(5), rng.standard_normal(4)]
    x = {0: np.stack([xa, xa]), 1: np.stack([xb, xb])}
    out = orc.rollout(g, [ta, tb], bias, x)[2][0]
    np.testing.assert_allclose(out, np.maximum(rhs + bias[2], 0.0), rtol=1e-12, atol=1e-12)


def test_linearity_with_identity_activation():
    g = W.paper_sr_net(1, 4)
    nodes = [Node(n.name, n.channels, n.height, n.width, ACT_IDENTITY) for n in g.nodes]
    g = Graph("lin", nodes, g.edges, 1, 4, out_node=3)
    w, b, x = W.make_case(g, seed=7)
    _, _, x2 = W.make_case(g, seed=8)
    f = lambda xx: orc.rollout(g, w, b, xx)[3]
    mix = {0: 2.0 * x[0].astype(np.float64) - 3.0 * x2[0].astype(np.float64)}
    np.testing.assert_allclose(f(mix), 2.0 * f(x) - 3.0 * f(x2), rtol=1e-10, atol=1e-10)


def test_window_chaining_and_edge_count():
    # Sec. 4 / Sec. 5: W = 1 windows chained; every pattern evaluates |E| edges per frame
    g0 = W.tiny_sr(2, 6)
    w, b, x = W.make_case(g0, seed=9, bias_scale=0.1)
    for bits in (W.streaming_pattern(g0), W.sequential_pattern(g0), W.hybrid_pattern(g0)):
        g = g0.with_pattern(bits)
        full = orc.Rollout(g, w, b)
        ref = full.run(x, keep=range(len(g.nodes)))
        assert full.edge_evaluations == 6 * len(g.edges)
        part = orc.Rollout(g, w, b)
        part.reset({0: x[0][0]})
        for t in range(1, 4):
            part.step({0: x[0][t]})
        saved = [a.copy() for a in part.X]
        cont = orc.Rollout(g, w, b)
        cont.X = saved
        for t in range(4, 7):
            X = cont.step({0: x[0][t]})
        for v in range(len(g.nodes)):
            np.testing.assert_array_equal(X[v], ref[v][-1])


def test_node_element_matches_full_frame():
    for mode in ("f64", "bf16"):
        g = W.tiny_sr(2, 3).with_pattern(W.hybrid_pattern(W.tiny_sr()))
        w, b, x = W.make_case(g, seed=10, bias_scale=0.2)
        r = orc.Rollout(g, w, b, mode)
        r.reset({0: x[0][0]})
        r.step({0: x[0][1]})
        prev = [a.copy() for a in r.X]
        cur = r.step({0: x[0][2]})
        rng = np.random.default_rng(0)
        for v in range(1, len(g.nodes)):
            n = g.nodes[v]
            for _ in range(5):
                bi, h, wd, c = rng.integers(2), rng.integers(n.height), rng.integers(n.width), rng.integers(n.channels)
                got = orc.node_element(g, w, b, v, bi, h, wd, c, prev, cur, mode)
                assert abs(got - cur[v][bi, h, wd, c]) <= 1e-12 * max(1.0, abs(got)), (mode, v)


def test_bf16_mode_is_close_to_f64_and_exactly_representable():
    g = W.tiny_sr(2, 5)
    w, b, x = W.make_case(g, seed=11)
    a = orc.rollout(g, w, b, x, keep=range(1, 5), mode="f64")
    c = orc.rollout(g, w, b, x, keep=range(1, 5), mode="bf16")
    for v in range(1, 5):
        assert np.array_equal(orc.round_bf16(c[v]), c[v])
        scale = np.abs(a[v]).max()
        assert np.abs(a[v] - c[v]).max() / scale < 3e-2
        assert np.abs(a[v] - c[v]).max() > 0


def test_shape_and_rollout_errors():
    g = W.tiny_sr()
    bad = Graph("bad", g.nodes, [Edge(0, 1), Edge(1, 2, stride=1)], 1, 1, out_node=2)
    with pytest.raises(orc.ShapeError):
        orc.check_graph(bad)
    with pytest.raises(th.RolloutError):
        orc.check_graph(g.with_pattern([1, 1, 1, 1, 0, 1]))


def test_input_recipes_are_seeded_and_shaped():
    for name, f in W.BENCH_CONFIGS.items():
        g = f()
        small = Graph(g.name, g.nodes, g.edges, 2, 3, g.dtype, g.out_node)
        if name == "hires_sr":
            small.nodes = [Node("in", 3, 32, 32, ACT_IDENTITY)] + small.nodes[1:]
        x1 = W.make_inputs(small, seed=0)
        x2 = W.make_inputs(small, seed=0)
        x3 = W.make_inputs(small, seed=1)
        n = small.nodes[0]
        assert x1[0].shape == (4, 2, n.height, n.width, n.channels) and x1[0].dtype == np.float32
        np.testing.assert_array_equal(x1[0], x2[0])
        assert np.any(x1[0] != x3[0])
