"""Pins of the training-window oracle (oracle/training.py): loss of a rollout window of size W and
its BPTT gradients.  None of these checks re-uses the oracle's own backward code: central finite
differences of its forward loss, torch's CPU autograd on the same window rebuilt from torch
operators, closed forms, the adjoint identity, and the first-response property of Sec. 4."""
import numpy as np
import pytest

import workloads as W
from workloads.graphs import Node, Edge, Graph, ACT_IDENTITY, ACT_RELU
from oracle import rollout as ro
from oracle import training as tr
from oracle import theory as th


def small_sr_graph(batch=2, classes=5, channels=(2, 3, 4), hw=6):
    """in(c0 @ hw x hw) -> a(c1 @ hw x hw) -> b(c2 @ hw/2 x hw/2, stride 2) -> out(classes, dense); skip in -> b
    (stride 2), self-recurrent a -> a, top-down b -> a (1x1 + x2 up-sampling), GAP+dense skip a -> out."""
    c0, c1, c2 = channels
    h2 = hw // 2
    nodes = [Node("in", c0, hw, hw, ACT_IDENTITY), Node("a", c1, hw, hw), Node("b", c2, h2, h2),
             Node("out", classes, 1, 1, ACT_IDENTITY)]
    edges = [Edge(0, 1, "conv", 3, 3, 1, 1), Edge(1, 2, "conv", 3, 3, 2, 1), Edge(2, 3, "dense", h2, h2, 1, 0),
             Edge(0, 2, "conv", 3, 3, 2, 1), Edge(1, 1, "conv", 3, 3, 1, 1), Edge(2, 1, "conv", 1, 1, 1, 0, 2),
             Edge(1, 3, "gap_dense", 1, 1, 1, 0)]
    return Graph("small_sr", nodes, edges, batch, 4, "f32", out_node=3)


def patterns(g):
    return {"streaming": g.with_pattern(W.streaming_pattern(g)), "hybrid": g.with_pattern(W.hybrid_pattern(g)),
            "sequential": g.with_pattern(W.sequential_pattern(g))}


def case(g, seed, frames):
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.3, frames=frames, recipe="uniform")
    labels = np.random.default_rng(seed + 5).integers(0, g.nodes[g.out_node].channels, g.batch)
    return [wi.astype(np.float64) for wi in w], [bi.astype(np.float64) for bi in b], x, labels


def loss_of(g, w, b, x, labels, Wn):
    win = tr.Window(g, w, b)
    win.forward(x, Wn)
    return win.loss(labels)


@pytest.mark.parametrize("pattern", ["streaming", "hybrid", "sequential"])
def test_gradients_match_central_finite_differences(pattern):
    g = patterns(small_sr_graph())[pattern]
    Wn = 4
    w, b, x, labels = case(g, 3, Wn)
    loss, dth, db = tr.window_gradients(g, w, b, x, labels, Wn)
    assert loss > 0
    rng = np.random.default_rng(0)
    h = 1e-5
    for ei in range(len(w)):
        idx = [tuple(rng.integers(0, s) for s in w[ei].shape) for _ in range(6)]
        for k in idx:
            wp = [wi.copy() for wi in w]; wm = [wi.copy() for wi in w]
            wp[ei][k] += h; wm[ei][k] -= h
            fd = (loss_of(g, wp, b, x, labels, Wn) - loss_of(g, wm, b, x, labels, Wn)) / (2 * h)
            assert abs(fd - dth[ei][k]) <= 1e-6 + 1e-5 * abs(fd), (pattern, "edge", ei, k, fd, dth[ei][k])
    for v in range(len(b)):
        if v in g.input_nodes():
            assert np.all(db[v] == 0)
            continue
        for c in range(len(b[v])):
            bp = [bi.copy() for bi in b]; bm = [bi.copy() for bi in b]
            bp[v][c] += h; bm[v][c] -= h
            fd = (loss_of(g, w, bp, x, labels, Wn) - loss_of(g, w, bm, x, labels, Wn)) / (2 * h)
            assert abs(fd - db[v][c]) <= 1e-6 + 1e-5 * abs(fd), (pattern, "bias", v, c, fd, db[v][c])


def torch_window_loss(g, w, b, x, labels, Wn, flips=(), masks=None):
    """The same window built from torch's CPU operators (float64); returns loss and autograd gradients.
    flips: (frame, node, flat index) at which the rectifier keeps its value but passes the other derivative."""
    import torch
    import torch.nn.functional as F
    tw = [torch.tensor(wi, dtype=torch.float64, requires_grad=True) for wi in w]
    tb = [torch.tensor(bi, dtype=torch.float64, requires_grad=True) for bi in b]
    n = len(g.nodes)
    pairs = [(e.src, e.dst) for e in g.edges]
    lv = th.levels(n, pairs, [e.bridge for e in g.edges])
    order = sorted(range(n), key=lambda v: lv[v])
    ins = g.input_nodes()
    X = [[None] * n for _ in range(Wn + 1)]
    for v, nd in enumerate(g.nodes):
        if v in ins:
            for i in range(Wn + 1):
                X[i][v] = torch.tensor(x[v][i], dtype=torch.float64)
        else:
            X[0][v] = torch.zeros((g.batch, nd.height, nd.width, nd.channels), dtype=torch.float64)
    for i in range(1, Wn + 1):
        for v in order:
            if v in ins:
                continue
            a = tb[v].reshape(1, 1, 1, -1)
            for ei, e in enumerate(g.edges):
                if e.dst != v:
                    continue
                src = X[i - e.bridge][e.src]
                if e.kind == "conv":
                    y = F.conv2d(src.permute(0, 3, 1, 2), tw[ei].permute(3, 2, 0, 1), stride=e.stride, padding=e.pad)
                    if e.up > 1:
                        y = y.repeat_interleave(e.up, dim=2).repeat_interleave(e.up, dim=3)
                    y = y.permute(0, 2, 3, 1)
                elif e.kind == "dense":
                    y = (src.reshape(g.batch, -1) @ tw[ei].reshape(-1, tw[ei].shape[3])).reshape(g.batch, 1, 1, -1)
                else:
                    y = (src.mean(dim=(1, 2)) @ tw[ei].reshape(tw[ei].shape[2], -1)).reshape(g.batch, 1, 1, -1)
                a = a + y
            if g.nodes[v].act == ACT_RELU:
                mask = (a.detach() > 0).to(torch.float64)
                for (fi, fv, fk) in flips:
                    if (fi, fv) == (i, v):
                        mask.view(-1)[fk] = 1.0 - mask.view(-1)[fk]
                X[i][v] = torch.relu(a).detach() + (a - a.detach()) * mask    # value of the rectifier, derivative = mask
            else:
                X[i][v] = a
            if masks is not None and masks.get(v) is not None:
                X[i][v] = X[i][v] * torch.tensor(masks[v][i], dtype=torch.float64)
    lab = torch.tensor(labels, dtype=torch.long)
    loss = sum(F.cross_entropy(X[i][g.out_node].reshape(g.batch, -1), lab) for i in range(1, Wn + 1)) / Wn
    loss.backward()
    return float(loss.detach()), [t.grad.numpy() if t.grad is not None else np.zeros(t.shape) for t in tw], \
        [t.grad.numpy() if t.grad is not None else np.zeros(t.shape) for t in tb]


@pytest.mark.parametrize("pattern", ["streaming", "hybrid", "sequential"])
@pytest.mark.parametrize("Wn", [1, 3, 6])
def test_gradients_match_torch_autograd_on_the_rebuilt_window(pattern, Wn):
    g = patterns(small_sr_graph(batch=3))[pattern]
    w, b, x, labels = case(g, 7 + Wn, Wn)
    loss, dth, db = tr.window_gradients(g, w, b, x, labels, Wn)
    tl, tdw, tdb = torch_window_loss(g, w, b, x, labels, Wn)
    assert abs(loss - tl) <= 1e-12 * max(1.0, abs(tl))
    for ei in range(len(w)):
        np.testing.assert_allclose(dth[ei], tdw[ei], rtol=1e-9, atol=1e-12, err_msg=f"edge {ei}")
    for v in range(len(b)):
        np.testing.assert_allclose(db[v], tdb[v], rtol=1e-9, atol=1e-12, err_msg=f"bias {v}")


def test_the_paper_mnist_net_window_against_torch():
    # MNIST SR net of App. A2 (7x7 stride-4 convolution, dense edges, dense skip, 3x3 self-recurrence), W = 4
    g = W.mnist_net("SR", batch=2, frames=4)
    w, b, x, labels = case(g, 11, 4)
    loss, dth, db = tr.window_gradients(g, w, b, x, labels, 4)
    tl, tdw, tdb = torch_window_loss(g, w, b, x, labels, 4)
    assert abs(loss - tl) <= 1e-12
    for a, c in zip(dth + db, tdw + tdb):
        np.testing.assert_allclose(a, c, rtol=1e-9, atol=1e-12)


def test_softmax_cross_entropy_closed_form():
    z = np.array([[1.0, 2.0, 0.5], [0.0, 0.0, 0.0]])
    labels = np.array([1, 2])
    loss, dz = tr.softmax_cross_entropy(z, labels)
    p = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    assert abs(loss - (-(np.log(p[0, 1]) + np.log(p[1, 2])) / 2)) < 1e-15
    onehot = np.eye(3)[labels]
    np.testing.assert_allclose(dz, (p - onehot) / 2, atol=1e-15)
    assert abs(loss - (np.log(3.0) + (-np.log(p[0, 1]))) / 2) < 1e-12      # uniform logits: log(number of classes)
    # invariance to a shift of the logits, and no overflow for large ones
    l2, d2 = tr.softmax_cross_entropy(z + 1000.0, labels)
    assert abs(l2 - loss) < 1e-9 and np.allclose(d2, dz)


@pytest.mark.parametrize("kind,geom", [("conv", (3, 3, 1, 1, 1)), ("conv", (3, 3, 2, 1, 1)), ("conv", (5, 5, 1, 2, 1)),
                                       ("conv", (7, 7, 4, 3, 1)), ("conv", (1, 1, 1, 0, 2)), ("conv", (3, 2, 2, 1, 1)),
                                       ("dense", None), ("gap_dense", None)])
def test_edge_adjoint_identity(kind, geom):
    # f_e is linear in x and in theta: <f_e(theta, x), y> = <x, dx(y)> = <theta, dtheta(y)>
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 8, 8, 3))
    if kind == "conv":
        kh, kw, s, p, up = geom
        e = Edge(0, 1, "conv", kh, kw, s, p, up)
        theta = rng.standard_normal((kh, kw, 3, 4))
    elif kind == "dense":
        e = Edge(0, 1, "dense", 8, 8, 1, 0)
        theta = rng.standard_normal((8, 8, 3, 4))
    else:
        e = Edge(0, 1, "gap_dense", 1, 1, 1, 0)
        theta = rng.standard_normal((1, 1, 3, 4))
    y = ro.edge_transform(e, theta, x)
    dy = rng.standard_normal(y.shape)
    dx, dth = tr.edge_backward(e, theta, x, dy)
    lhs = float((y * dy).sum())
    assert abs(lhs - float((x * dx).sum())) <= 1e-9 * max(1.0, abs(lhs))
    assert abs(lhs - float((theta * dth).sum())) <= 1e-9 * max(1.0, abs(lhs))


def test_window_shorter_than_the_shortest_path_leaves_input_edges_without_gradient():
    # Sec. 4: under the streaming rollout the output first depends on the input after
    # shortest-path-many frames.  A chain of 4 edges, W = 3: the loss cannot depend on the input, so the
    # edge that leaves the input has zero gradient; with W = 4 it has not.  Under the sequential
    # pattern already W = 1 informs the output.
    g0 = W.chain(4, batch=2, frames=4, hw=4, c=2)
    g0 = Graph(g0.name, g0.nodes[:-1] + [Node("out", 2, 4, 4, ACT_IDENTITY)], g0.edges, 2, 4, "f32", out_node=4)
    # classification head over the last node's pixels: flatten (h, w, c) as classes
    labels = np.array([3, 17])
    for pattern, Wn, informed in (("streaming", 3, False), ("streaming", 4, True), ("sequential", 1, True)):
        g = patterns(g0)[pattern]
        w, b, x = W.make_case(g, seed=2, bias_scale=0.2, frames=Wn, recipe="uniform")
        w = [np.abs(wi).astype(np.float64) for wi in w]          # positive weights: no unit dies
        b = [np.abs(bi).astype(np.float64) for bi in b]
        loss, dth, db = tr.window_gradients(g, w, b, x, labels, Wn)
        assert (np.abs(dth[0]).max() > 0) == informed, (pattern, Wn)
        assert np.abs(dth[3]).max() > 0                           # the last edge always sees the loss


def test_gradient_is_the_mean_of_the_single_frame_gradients():
    # The loss is a mean over frames.  The loss of frame k alone is k * (loss of the window of size k)
    # - (k-1) * (loss of the window of size k-1), both from the zero state; the same holds for the
    # gradients, and their mean over k = 1..W is the gradient of the window of size W.
    g = patterns(small_sr_graph())["streaming"]
    Wn = 3
    w, b, x, labels = case(g, 13, Wn)
    _, dth, _ = tr.window_gradients(g, w, b, x, labels, Wn)

    def grads(k):
        if k == 0:
            return [np.zeros_like(t) for t in w]
        return tr.window_gradients(g, w, b, {v: x[v][:k + 1] for v in x}, labels, k)[1]

    acc = [np.zeros_like(t) for t in w]
    for k in range(1, Wn + 1):
        gk, gkm = grads(k), grads(k - 1)
        acc = [a + (k * p - (k - 1) * q) / Wn for a, p, q in zip(acc, gk, gkm)]
    for a, c in zip(acc, dth):
        np.testing.assert_allclose(a, c, rtol=1e-9, atol=1e-12)


def test_toggled_rectifier_derivatives_against_torch():
    g = patterns(small_sr_graph(batch=2))["hybrid"]
    Wn = 4
    w, b, x, labels = case(g, 17, Wn)
    win = tr.Window(g, w, b)
    win.forward(x, Wn)
    base = win.backward(labels)
    rng = np.random.default_rng(3)
    flips = [(int(rng.integers(1, Wn + 1)), v, int(rng.integers(0, win.X[1][v].size))) for v in (1, 2) for _ in range(4)]
    dth, db, _ = win.backward(labels, flips=flips)
    _, tdw, tdb = torch_window_loss(g, w, b, x, labels, Wn, flips=flips)
    for a, c in zip(dth + db, tdw + tdb):
        np.testing.assert_allclose(a, c, rtol=1e-9, atol=1e-12)
    assert any(np.abs(a - c).max() > 1e-9 for a, c in zip(dth, base[0]))     # the toggles do change the gradient
    none = win.backward(labels, flips=[])
    for a, c in zip(none[0], base[0]):
        assert np.array_equal(a, c)


def test_near_kink_lists_exactly_the_small_preactivations():
    g = patterns(small_sr_graph(batch=2))["streaming"]
    w, b, x, labels = case(g, 19, 3)
    win = tr.Window(g, w, b)
    win.forward(x, 3)
    got = set(win.near_kink(1e-2))
    assert got
    for v in (1, 2):
        scale = max(np.abs(win.X[i][v]).max() for i in range(1, 4))
        for i in range(1, 4):
            a = win.A[i][v].ravel()
            for k in range(a.size):
                assert ((i, v, k) in got) == (abs(a[k]) <= 1e-2 * scale)
    assert all(v in (1, 2) for (_, v, _) in got)          # the output node has no rectifier
    assert win.near_kink(0.0) == [] or all(win.A[i][v].ravel()[k] == 0 for (i, v, k) in win.near_kink(0.0))


def test_kink_matching_recovers_planted_toggles():
    # the helper the GPU tests use to decide which near-kink elements carry the other derivative:
    # plant toggles on the oracle's side, add float32-sized noise, and ask for them back
    import gpu_util
    g = patterns(small_sr_graph(batch=2))["sequential"]
    Wn = 4
    w, b, x, labels = case(g, 23, Wn)
    win = tr.Window(g, w, b)
    win.forward(x, Wn)
    _, base_db, _ = win.backward(labels)
    old = gpu_util.KINK_TAU
    gpu_util.KINK_TAU = 1e-2              # wide enough to have candidates on this tiny window
    try:
        cand = win.near_kink(gpu_util.KINK_TAU)
        assert 3 <= len(cand) <= gpu_util.KINK_MAX
        planted = [cand[0], cand[-1]]
        dth, db, _ = win.backward(labels, flips=planted)
        base = win.backward(labels)[:2]
        rng = np.random.default_rng(0)
        noise = lambda t: t * (1 + 1e-6 * rng.standard_normal(t.shape))
        noisy = ([noise(t) for t in dth], [None if v in g.input_nodes() else noise(t) for v, t in enumerate(db)])
        found = gpu_util.match_kinks(win, labels, noisy, base)
        assert found and set(found) <= set(cand)
        # the same gradient as with the planted toggles (a toggle where no gradient arrives is not found
        # and does not matter)
        dth2, db2, _ = win.backward(labels, flips=found)
        for t, u in zip(dth + db, dth2 + db2):
            np.testing.assert_allclose(t, u, rtol=0, atol=1e-12)
        assert any(np.abs(t - u).max() > 1e-6 for t, u in zip(db, base_db))
        clean = (base[0], [None if v in g.input_nodes() else t for v, t in enumerate(base[1])])
        assert gpu_util.match_kinks(win, labels, clean, base) == []
    finally:
        gpu_util.KINK_TAU = old


def test_rmsprop_step_closed_forms_and_torch():
    import torch
    rng = np.random.default_rng(1)
    theta = rng.standard_normal((3, 4))
    g = rng.standard_normal((3, 4))
    lr, rho, eps = 1e-2, 0.9, 1e-7
    # first step from a = 0: theta - lr * g / (sqrt(1 - rho) |g| + eps)
    t1, a1 = tr.rmsprop_step(theta, np.zeros_like(theta), g, lr, rho, eps)
    np.testing.assert_allclose(a1, (1 - rho) * g * g, rtol=1e-15)
    np.testing.assert_allclose(t1, theta - lr * g / (np.sqrt(1 - rho) * np.abs(g) + eps), rtol=1e-14)
    # a constant gradient: a -> g^2, the step tends to lr * g / (|g| + eps), i.e. lr * sign(g)
    t, a = theta, np.zeros_like(theta)
    for _ in range(400):
        prev = t
        t, a = tr.rmsprop_step(t, a, g, lr, rho, eps)
    np.testing.assert_allclose(a, g * g, rtol=1e-12)
    np.testing.assert_allclose(prev - t, lr * g / (np.abs(g) + eps), rtol=1e-10)
    # several steps with changing gradients against torch's optimiser
    p = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.RMSprop([p], lr=lr, alpha=rho, eps=eps)
    t, a = theta, np.zeros_like(theta)
    for k in range(5):
        gk = rng.standard_normal((3, 4))
        p.grad = torch.tensor(gk, dtype=torch.float64)
        opt.step()
        t, a = tr.rmsprop_step(t, a, gk, lr, rho, eps)
        np.testing.assert_allclose(t, p.detach().numpy(), rtol=1e-13, atol=1e-15)


def dropout_masks(g, Wn, seed, rates):
    """{node: (W+1,B,H,W,C)} of 0 or 1/(1 - rate), drawn afresh per frame (the caller's business: the
    method's random numbers are inputs of both sides)."""
    rng = np.random.default_rng(seed)
    out = {}
    for v, rate in rates.items():
        n = g.nodes[v]
        keep = rng.random((Wn + 1, g.batch, n.height, n.width, n.channels)) >= rate
        out[v] = keep.astype(np.float64) / (1.0 - rate)
    return out


@pytest.mark.parametrize("pattern", ["streaming", "hybrid", "sequential"])
def test_dropout_masks_against_finite_differences_and_torch(pattern):
    g = patterns(small_sr_graph(batch=3))[pattern]
    Wn = 4
    w, b, x, labels = case(g, 29, Wn)
    masks = dropout_masks(g, Wn, 30, {1: 0.25, 2: 0.5})        # App. A2: 0.25, and 0.5 on the last hidden layer
    loss, dth, db = tr.window_gradients(g, w, b, x, labels, Wn, masks=masks)
    tl, tdw, tdb = torch_window_loss(g, w, b, x, labels, Wn, masks=masks)
    assert abs(loss - tl) <= 1e-12 * max(1.0, abs(tl))
    for a, c in zip(dth + db, tdw + tdb):
        np.testing.assert_allclose(a, c, rtol=1e-9, atol=1e-12)
    rng = np.random.default_rng(2)
    h = 1e-5

    def loss_at(ws):
        win = tr.Window(g, ws, b)
        win.forward(x, Wn, masks=masks)
        return win.loss(labels)

    for ei in range(len(w)):
        for _ in range(3):
            k = tuple(rng.integers(0, s) for s in w[ei].shape)
            wp = [t.copy() for t in w]; wm = [t.copy() for t in w]
            wp[ei][k] += h; wm[ei][k] -= h
            fd = (loss_at(wp) - loss_at(wm)) / (2 * h)
            assert abs(fd - dth[ei][k]) <= 1e-6 + 1e-5 * abs(fd), (pattern, ei, k, fd, dth[ei][k])
    # the masks matter, masks of ones do not, and a node that is dropped entirely passes nothing on
    base = tr.window_gradients(g, w, b, x, labels, Wn)
    assert any(np.abs(a - c).max() > 1e-6 for a, c in zip(dth, base[1]))
    ones = {v: np.ones_like(m) for v, m in masks.items()}
    same = tr.window_gradients(g, w, b, x, labels, Wn, masks=ones)
    for a, c in zip(same[1] + same[2], base[1] + base[2]):
        assert np.array_equal(a, c)
    cut = tr.window_gradients(g, w, b, x, labels, Wn, masks={2: np.zeros_like(masks[2])})
    for ei, e in enumerate(g.edges):
        if e.dst == 2:
            assert np.all(cut[1][ei] == 0), ei            # edges into the dropped node get no gradient
