"""GPU parity of one training window (Sec. 3 rollout window of size W, Sec. 2 backpropagation through
it, loss of App. A2): loss and every weight and bias gradient from the C-ABI library against the
float64 oracle on the same seeded arrays, under the streaming, hybrid and sequential patterns.

Tolerance.  Both sides compute the same sums, the library in float32: a gradient element is a sum of
n = W * B * Ho * Wo (weights) or taps * Cout (states) products, each term already carrying the
float32 error of the forward pass and of the gradient it was built from.  With sequential float32
summation the error is about sqrt(n) * 2^-24 of the sum of magnitudes, n <= 3e5 here: up to a few
1e-6 of the tensor's largest element (measured: 1e-7 .. 6e-7).  GRAD_TOL = 2e-5 of max|reference| per
tensor leaves a factor of about 30 and is printed next to what was measured.  Rectifier elements whose
pre-activation is zero to float32 accuracy may carry either derivative: see gpu_util.match_kinks.
"""
from dataclasses import replace

import numpy as np
import pytest

import workloads as W
from oracle import training as tr
from gpu_util import to_device, max_abs_rel, match_kinks
from test_oracle_training import small_sr_graph

pytestmark = pytest.mark.gpu

GRAD_TOL = 2e-5
LOSS_TOL = 1e-5
PATTERNS = {"streaming": W.streaming_pattern, "hybrid": W.hybrid_pattern, "sequential": W.sequential_pattern}


def cases():
    return {
        # every edge kind: strided and plain convolutions, skip, self-recurrence, 1x1 + up-sampling, dense, GAP+dense
        "small_sr": (lambda: small_sr_graph(batch=3), 4),
        # the same wiring wide enough for the tiled matrix-core gradient kernels (32 and 64 channels at 16x16 / 8x8,
        # batch 8); its input and 1x1 edges stay on the one-thread-per-output kernels
        "mid_sr": (lambda: small_sr_graph(batch=8, classes=10, channels=(8, 32, 64), hw=16), 4),
        "tiny_sr": (lambda: W.tiny_sr(batch=2, frames=5), 5),
        # App. A2: MNIST net with skip and self-recurrence, 7x7 stride-4 convolution and dense edges
        "mnist_sr": (lambda: W.mnist_net("SR", batch=16, frames=4), 4),
        # ... at the paper's batch size (Tab. A1): its strided 7x7 convolution and dense edges on the tiled kernels
        "mnist_sr_b128": (lambda: W.mnist_net("SR", batch=128, frames=3), 3),
        # App. A2: CIFAR10 family member (10 nodes, 64-channel 3x3 convolutions at 32x32 and 16x16)
        "dsr2": (lambda: replace(W.dsr_net(2, batch=2, frames=6), dtype="f32"), 6),
    }


def run_case(g, Wn, seed, dev=None):
    import torch
    import paper_1806_04965_amd as sr
    w, b, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=Wn, recipe="uniform")
    labels = np.random.default_rng(seed + 1).integers(0, g.nodes[g.out_node].channels, g.batch).astype(np.int32)
    own = dev is None
    if own:
        dev = sr.SrGraph(g)
        dev.set_parameters(w, b)
    ins = g.input_nodes()
    xd = [to_device(x[v][:Wn + 1], "f32") for v in ins]
    loss, dth, dbs = dev.window_gradients(xd, torch.from_numpy(labels).to("cuda"), Wn)
    dev.synchronize()
    got = (float(loss.cpu()[0]), [t.cpu().numpy() for t in dth], [None if t is None else t.cpu().numpy() for t in dbs])
    if own:
        dev.close()
    return got, (w, b, x, labels)


def check_against_oracle(g, Wn, got, data, label, may_be_zero=False):
    w, b, x, labels = data
    loss, dth, dbs = got
    win = tr.Window(g, w, b)
    win.forward({v: x[v][:Wn + 1] for v in x}, Wn)
    ref_loss = win.loss(labels)
    ref_dth, ref_db, _ = win.backward(labels)
    assert ref_loss > 0
    assert abs(loss - ref_loss) <= LOSS_TOL * max(1.0, abs(ref_loss)), (label, loss, ref_loss)

    def errors(rd, rb):
        out = {}
        for ei in range(len(g.edges)):
            assert dth[ei].shape == rd[ei].shape
            if may_be_zero and np.abs(rd[ei]).max() == 0:       # a window too short to inform this edge (Sec. 4)
                assert np.abs(dth[ei]).max() == 0, (label, "edge", ei)
                continue
            assert np.abs(rd[ei]).max() > 0, (label, "edge", ei, "reference gradient is all zero")
            out[f"dtheta[{ei}]"] = max_abs_rel(dth[ei], rd[ei])
        for v in range(len(g.nodes)):
            if dbs[v] is not None:
                if may_be_zero and np.abs(rb[v]).max() == 0:
                    assert np.abs(dbs[v]).max() == 0, (label, "bias", v)
                    continue
                assert np.abs(rb[v]).max() > 0, (label, "bias", v)
                out[f"dbias[{v}]"] = max_abs_rel(dbs[v], rb[v])
        return out

    err = errors(ref_dth, ref_db)
    flips = []
    if max(err.values()) > GRAD_TOL:
        # elements at the rectifier's kink may carry either derivative (see gpu_util.match_kinks)
        flips = match_kinks(win, labels, (dth, dbs), (ref_dth, ref_db), verbose=label)
        assert flips, f"{label}: {max(err, key=err.get)} max-abs-rel {max(err.values()):.3e} > {GRAD_TOL}, no element at the kink"
        ref_dth, ref_db, _ = win.backward(labels, flips=flips)
        err = errors(ref_dth, ref_db)
    worst = max(err, key=err.get)
    assert err[worst] <= GRAD_TOL, f"{label} {worst}: max-abs-rel {err[worst]:.3e} > {GRAD_TOL} (kink elements taken: {flips})"
    print(f"[train] {label}: W={Wn}, loss {loss:.6f} (oracle {ref_loss:.6f}), worst gradient max-abs-rel {err[worst]:.2e} "
          f"(tol {GRAD_TOL}), rectifier elements taken on the other side of the kink: {len(flips)}", flush=True)
    return err[worst]


@pytest.mark.parametrize("pattern", list(PATTERNS))
@pytest.mark.parametrize("name", list(cases()))
def test_window_gradients_match_the_oracle(name, pattern):
    mk, Wn = cases()[name]
    g0 = mk()
    g = g0.with_pattern(PATTERNS[pattern](g0))
    got, data = run_case(g, Wn, seed=41)
    check_against_oracle(g, Wn, got, data, f"{name}/{pattern}")


def test_window_sizes_on_one_graph_and_reproducible_bits():
    # one graph object, windows of size 3, then 1, then 6 (its arena grows), then 3 again: every call
    # stands alone (zero initial state) and the same call gives the same bits
    import paper_1806_04965_amd as sr
    g0 = small_sr_graph(batch=4)
    g = g0.with_pattern(W.streaming_pattern(g0))
    w, b, _ = W.make_case(g, seed=41, bias_scale=0.1, frames=6, recipe="uniform")
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    first = None
    for Wn in (3, 1, 6, 3):
        got, data = run_case(g, Wn, seed=41, dev=dev)
        check_against_oracle(g, Wn, got, data, f"small_sr W={Wn}", may_be_zero=Wn < 3)
        if Wn == 3:
            if first is None:
                first = got
            else:
                assert got[0] == first[0]
                for a, c in zip(got[1] + [t for t in got[2] if t is not None],
                                first[1] + [t for t in first[2] if t is not None]):
                    assert np.array_equal(a, c)
    dev.close()


def test_window_shorter_than_the_shortest_path_gives_the_first_edge_no_gradient():
    # Sec. 4 on the device: chain of 4 edges under the streaming pattern, W = 3 < shortest path
    from workloads.graphs import Node, Graph, ACT_IDENTITY
    g0 = W.chain(3, batch=2, frames=4, hw=4, c=2)
    nodes = g0.nodes + [Node("out", 5, 1, 1, ACT_IDENTITY)]
    edges = g0.edges + [W.Edge(3, 4, "dense", 4, 4, 1, 0)]
    g0 = Graph("chain_head", nodes, edges, 2, 4, "f32", out_node=4)
    g = g0.with_pattern(W.streaming_pattern(g0))
    for Wn, informed in ((3, False), (4, True)):
        got, _ = run_case(g, Wn, seed=5)
        assert (np.abs(got[1][0]).max() > 0) == informed, Wn
        assert np.abs(got[1][3]).max() > 0


def test_refusals():
    import torch
    import paper_1806_04965_amd as sr
    g = W.tiny_sr(batch=2, frames=2)
    w, b, x = W.make_case(g, seed=1, frames=2)
    labels = torch.zeros(2, dtype=torch.int32, device="cuda")
    dev = sr.SrGraph(g, dtype="bf16")
    dev.set_parameters(w, b)
    xd = [to_device(x[v], "bf16") for v in g.input_nodes()]
    with pytest.raises(sr.SrError) as ei:
        dev.window_gradients(xd, labels, 2)
    assert "SR_F32" in str(ei.value)
    dev.close()
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    xd = [to_device(x[v], "f32") for v in g.input_nodes()]
    for bad in (0, 1):      # an input node; a node that is not 1x1
        with pytest.raises(sr.SrError):
            dev.window_gradients(xd, labels, 2, out_node=bad)
    with pytest.raises(sr.SrError):
        dev.window_gradients(xd, labels, 0)
    dev.close()


def test_rmsprop_step_on_given_gradients():
    # the update itself, on seeded gradients handed to both sides (App. A2: RMSprop); three steps so that the
    # running mean of the squared gradient is carried over
    import torch
    import paper_1806_04965_amd as sr
    g0 = small_sr_graph(batch=2)
    g = g0.with_pattern(W.streaming_pattern(g0))
    w, b, _ = W.make_case(g, seed=9, bias_scale=0.1, frames=1)
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    ins = g.input_nodes()
    rng = np.random.default_rng(10)
    th = [wi.astype(np.float64) for wi in w]
    bs = [bi.astype(np.float64) for bi in b]
    a_w = [np.zeros_like(t) for t in th]
    a_b = [np.zeros_like(t) for t in bs]
    lr, rho, eps = 1e-2, 0.9, 1e-7
    for step in range(3):
        gw = [(rng.standard_normal(t.shape) * 10.0 ** rng.integers(-6, 1)).astype(np.float32) for t in th]
        gb = [None if v in ins else rng.standard_normal(t.shape).astype(np.float32) for v, t in enumerate(bs)]
        dev.rmsprop_step([torch.from_numpy(t).to("cuda") for t in gw],
                         [None if t is None else torch.from_numpy(t).to("cuda") for t in gb], lr / (1 + 1e-6 * step), rho, eps)
        for i in range(len(th)):
            th[i], a_w[i] = tr.rmsprop_step(th[i], a_w[i], gw[i], lr / (1 + 1e-6 * step), rho, eps)
        for v in range(len(bs)):
            if gb[v] is not None:
                bs[v], a_b[v] = tr.rmsprop_step(bs[v], a_b[v], gb[v], lr / (1 + 1e-6 * step), rho, eps)
        got_w, got_b = dev.get_parameters()
        for i in range(len(th)):
            assert np.abs(got_w[i] - th[i]).max() <= 1e-6 * max(1.0, np.abs(th[i]).max()), (step, i)
        for v in range(len(bs)):
            assert np.abs(got_b[v] - bs[v]).max() <= 1e-6 * max(1.0, np.abs(bs[v]).max()), (step, v)
            if v in ins:
                assert np.array_equal(got_b[v], b[v])          # input nodes have no parameters to update
    dev.close()


def test_training_steps_follow_the_oracle_and_lower_the_loss():
    # window gradients + RMSprop, five steps on the same batch (the paper's MNIST SR net, B = 16, W = 4):
    # the loss falls, and the parameters follow the oracle's loop.  RMSprop divides a gradient by its own
    # running magnitude, so an element whose gradient is below the float32 noise of its tensor moves by
    # up to lr / sqrt(1 - rho) in either direction: such elements are only held to that bound.
    import torch
    import paper_1806_04965_amd as sr
    g0 = W.mnist_net("SR", batch=16, frames=4)
    g = g0.with_pattern(W.streaming_pattern(g0))
    Wn = 4
    w, b, x = W.make_case(g, seed=12, bias_scale=0.1, frames=Wn, recipe="uniform")
    labels = np.random.default_rng(13).integers(0, 10, g.batch).astype(np.int32)
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    ins = g.input_nodes()
    xd = [to_device(x[v][:Wn + 1], "f32") for v in ins]
    ld = torch.from_numpy(labels).to("cuda")
    th = [wi.astype(np.float64) for wi in w]
    bs = [bi.astype(np.float64) for bi in b]
    a_w = [np.zeros_like(t) for t in th]
    a_b = [np.zeros_like(t) for t in bs]
    lr, rho, eps = 1e-3, 0.9, 1e-7
    losses, ref_losses = [], []
    for step in range(5):
        loss, dth, dbs = dev.window_gradients(xd, ld, Wn)
        dev.rmsprop_step(dth, dbs, lr, rho, eps)
        losses.append(float(loss.cpu()[0]))
        rl, rdth, rdb = tr.window_gradients(g, th, bs, {v: x[v][:Wn + 1] for v in x}, labels, Wn)
        ref_losses.append(rl)
        noisy = []
        for i in range(len(th)):
            noisy.append(np.abs(rdth[i]) < 1e-3 * np.abs(rdth[i]).max())
            th[i], a_w[i] = tr.rmsprop_step(th[i], a_w[i], rdth[i], lr, rho, eps)
        for v in range(len(bs)):
            if v not in ins:
                bs[v], a_b[v] = tr.rmsprop_step(bs[v], a_b[v], rdb[v], lr, rho, eps)
        got_w, _ = dev.get_parameters()
        bound = (step + 1) * 2 * lr / np.sqrt(1 - rho) * 1.01
        for i in range(len(th)):
            d = np.abs(got_w[i] - th[i])
            assert d[~noisy[i]].max() <= 2e-2 * lr * (step + 1), (step, i, d[~noisy[i]].max())
            assert d.max() <= bound, (step, i, d.max())
    assert all(abs(a - c) <= 1e-4 * max(1.0, abs(c)) for a, c in zip(losses, ref_losses)), (losses, ref_losses)
    assert losses[-1] < losses[0] - 0.05, losses
    print(f"[train] mnist_sr, 5 RMSprop steps: loss {losses[0]:.4f} -> {losses[-1]:.4f} (oracle {ref_losses[0]:.4f} -> {ref_losses[-1]:.4f})", flush=True)
    dev.close()


def test_two_inputs_batch_of_one_odd_channel_counts_and_clamped_labels():
    # degenerate shapes of a window: two input nodes, a batch of one, channel counts 3 / 2 / 5 / 7, 5x5 states, and
    # labels outside the class range, which the library clamps to it
    import torch
    import paper_1806_04965_amd as sr
    from workloads.graphs import Node, Edge, Graph, ACT_IDENTITY
    nodes = [Node("in0", 3, 5, 5, ACT_IDENTITY), Node("in1", 2, 5, 5, ACT_IDENTITY), Node("a", 5, 5, 5),
             Node("out", 7, 1, 1, ACT_IDENTITY)]
    edges = [Edge(0, 2, "conv", 3, 3, 1, 1), Edge(1, 2, "conv", 1, 1, 1, 0), Edge(2, 2, "conv", 3, 3, 1, 1),
             Edge(2, 3, "dense", 5, 5, 1, 0), Edge(1, 3, "gap_dense", 1, 1, 1, 0)]
    g0 = Graph("two_inputs", nodes, edges, 1, 3, "f32", out_node=3)
    for pattern in ("streaming", "sequential"):
        g = g0.with_pattern(PATTERNS[pattern](g0))
        got, data = run_case(g, 3, seed=77)
        check_against_oracle(g, 3, got, data, f"two_inputs/{pattern}")
    g = g0.with_pattern(W.streaming_pattern(g0))
    g = Graph(g.name, g.nodes, g.edges, 2, 3, "f32", out_node=3)
    w, b, x = W.make_case(g, seed=78, bias_scale=0.1, frames=3, recipe="uniform")
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    xd = [to_device(x[v][:4], "f32") for v in g.input_nodes()]
    loss, dth, dbs = dev.window_gradients(xd, torch.tensor([-3, 99], dtype=torch.int32, device="cuda"), 3)
    dev.synchronize()
    ref_loss, ref_dth, _ = tr.window_gradients(g, w, b, {v: x[v][:4] for v in x}, np.array([0, 6]), 3)
    assert abs(float(loss.cpu()[0]) - ref_loss) <= LOSS_TOL * max(1.0, ref_loss)
    for ei in range(len(g.edges)):
        assert max_abs_rel(dth[ei].cpu().numpy(), ref_dth[ei]) <= GRAD_TOL, ei
    dev.close()


@pytest.mark.parametrize("name", ["small_sr", "mid_sr", "mnist_sr"])
def test_window_gradients_with_dropout_masks(name):
    # App. A2, training details: dropout 0.25, and 0.5 on the last hidden layer; the masks are drawn here, once,
    # and handed to both sides
    import torch
    import paper_1806_04965_amd as sr
    from test_oracle_training import dropout_masks
    mk, Wn = cases()[name]
    g0 = mk()
    g = g0.with_pattern(W.hybrid_pattern(g0))
    hidden = [v for v in range(len(g.nodes)) if v not in g.input_nodes() and v != g.out_node]
    rates = {v: (0.5 if v == hidden[-1] else 0.25) for v in hidden}
    masks = dropout_masks(g, Wn, 91, rates)
    w, b, x = W.make_case(g, seed=92, bias_scale=0.1, frames=Wn, recipe="uniform")
    labels = np.random.default_rng(93).integers(0, g.nodes[g.out_node].channels, g.batch).astype(np.int32)
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    xd = [to_device(x[v][:Wn + 1], "f32") for v in g.input_nodes()]
    md = {v: torch.from_numpy(m.astype(np.float32)).to("cuda").contiguous() for v, m in masks.items()}
    loss, dth, dbs = dev.window_gradients(xd, torch.from_numpy(labels).to("cuda"), Wn, masks=md)
    dev.synchronize()
    ref_loss, ref_dth, ref_db = tr.window_gradients(g, w, b, {v: x[v][:Wn + 1] for v in x}, labels, Wn, masks=masks)
    no_drop = tr.window_gradients(g, w, b, {v: x[v][:Wn + 1] for v in x}, labels, Wn)[0]
    assert abs(ref_loss - no_drop) > 1e-3                      # the masks do change the window
    assert abs(float(loss.cpu()[0]) - ref_loss) <= LOSS_TOL * max(1.0, ref_loss)
    worst = 0.0
    for ei in range(len(g.edges)):
        assert np.abs(ref_dth[ei]).max() > 0
        worst = max(worst, max_abs_rel(dth[ei].cpu().numpy(), ref_dth[ei]))
    for v in range(len(g.nodes)):
        if dbs[v] is not None:
            worst = max(worst, max_abs_rel(dbs[v].cpu().numpy(), ref_db[v]))
    print(f"[train] {name}/hybrid with dropout: loss {float(loss.cpu()[0]):.6f} (oracle {ref_loss:.6f}), worst gradient "
          f"max-abs-rel {worst:.2e}", flush=True)
    assert worst <= GRAD_TOL
    dev.close()


@pytest.mark.parametrize("name", ["mid_sr", "mnist_sr_b128"])
def test_windows_into_the_same_buffers_follow_their_new_contents(name):
    # A training loop keeps its buffers.  Three calls into the same tensors, with new inputs and labels written
    # into them in between (and unrelated torch work and synchronisations between the calls), then one call with
    # other buffers: each must equal, bit for bit, what a second graph object gives for the same data in fresh
    # tensors (the launches of a window run on four streams: their sums must not depend on how those interleave),
    # and the oracle within the tolerance.
    import torch
    import paper_1806_04965_amd as sr
    mk, Wn = cases()[name]
    g0 = mk()
    g = g0.with_pattern(W.hybrid_pattern(g0))
    w, b, _ = W.make_case(g, seed=61, bias_scale=0.1, frames=Wn, recipe="uniform")
    dev = sr.SrGraph(g)
    plain = sr.SrGraph(g)
    for d in (dev, plain):
        d.set_parameters(w, b)
    ins = g.input_nodes()
    classes = g.nodes[g.out_node].channels
    xd = labels_d = res = None
    for call, seed in enumerate((62, 63, 64, 65)):
        _, _, x = W.make_case(g, seed=seed, bias_scale=0.1, frames=Wn, recipe="uniform")
        labels = np.random.default_rng(seed + 100).integers(0, classes, g.batch).astype(np.int32)
        fresh = [to_device(x[v][:Wn + 1], "f32") for v in ins]
        if call in (0, 3):           # new buffers
            xd, labels_d, res = fresh, torch.from_numpy(labels).to("cuda"), None
        else:                        # same buffers, new contents
            for t, f in zip(xd, fresh):
                t.copy_(f)
            labels_d.copy_(torch.from_numpy(labels))
        torch.cuda.synchronize()
        res = dev.window_gradients(xd, labels_d, Wn, into=res)
        dev.synchronize()
        filler = torch.randn(1 << 20, device="cuda").sum().item()   # the program's own work between the calls
        assert np.isfinite(filler)
        want = plain.window_gradients(fresh, torch.from_numpy(labels).to("cuda"), Wn)
        plain.synchronize()
        assert float(res[0].cpu()[0]) == float(want[0].cpu()[0]), f"call {call}: loss"
        for a, c in zip(res[1] + [t for t in res[2] if t is not None], want[1] + [t for t in want[2] if t is not None]):
            assert torch.equal(a, c), f"call {call}: the two graph objects' gradients differ"
        if call in (1, 3):
            got = (float(res[0].cpu()[0]), [t.cpu().numpy() for t in res[1]],
                   [None if t is None else t.cpu().numpy() for t in res[2]])
            check_against_oracle(g, Wn, got, (w, b, x, labels), f"{name} same buffers, call {call}")
    dev.close()
    plain.close()


def ragged_graph(batch=5, channels=(24, 40, 136)):
    """Channel counts and pixel counts that are multiples of no tile edge: 24 channels (32-wide column tiles, ragged),
    40 (64-wide), 136 (128-wide plus a ragged second column tile), 19 x 19 images (ragged row tiles), a stride-2 edge
    (phase planes of unequal size), a self-recurrent edge and a dense read-out."""
    from workloads.graphs import Node, Edge, Graph, ACT_IDENTITY
    ca, cb, cc = channels
    nodes = [Node("in", 3, 19, 19, ACT_IDENTITY), Node("a", ca, 19, 19), Node("b", cb, 10, 10), Node("c", cc, 10, 10),
             Node("out", 7, 1, 1, ACT_IDENTITY)]
    edges = [Edge(0, 1, "conv", 5, 5, 1, 2), Edge(1, 1, "conv", 3, 3, 1, 1), Edge(1, 2, "conv", 3, 3, 2, 1),
             Edge(2, 3, "conv", 3, 3, 1, 1), Edge(3, 2, "conv", 1, 1, 1, 0), Edge(3, 4, "dense", 10, 10, 1, 0)]
    return Graph("ragged", nodes, edges, batch, 3, "f32", out_node=4)


@pytest.mark.parametrize("channels", [(24, 40, 136), (22, 42, 134)])
@pytest.mark.parametrize("tall_from", [0, 2048, 1 << 30])
def test_every_tile_shape_on_ragged_sizes(tall_from, channels):
    # SR_OPT_TRAIN_TALL_TILES_FROM (option 8): 0 sends every tiled contraction to the taller of its two tile shapes
    # (128x128, 128x64, 256x32), 2^30 to the shorter (64x64, 128x32), the default chooses by the launch's size.
    # Channel counts that are multiples of four take the kernel that gathers 16 bytes at a time, the others the
    # one that gathers element by element.
    import paper_1806_04965_amd as sr
    g0 = ragged_graph(channels=channels)
    g = g0.with_pattern(W.hybrid_pattern(g0))
    Wn = 3
    w, b, _ = W.make_case(g, seed=71, bias_scale=0.1, frames=Wn, recipe="uniform")
    dev = sr.SrGraph(g, options={8: tall_from})
    dev.set_parameters(w, b)
    got, data = run_case(g, Wn, seed=71, dev=dev)
    check_against_oracle(g, Wn, got, data, f"ragged{channels}/hybrid tall_from={tall_from}")
    dev.close()


@pytest.mark.timeout(600)
def test_gtsrb_shaped_window_at_full_width():
    # The GTSRB-shaped benchmark graph as an fp32 graph with its real image sizes and channel counts (64 @ 48x48 ...
    # 256 @ 6x6, 32 edges: skips, self-recurrence, the 1x1 up-sampled feedback edge, GAP + dense head), hybrid
    # pattern, W = 3, at a batch of 8 so that the float64 oracle takes seconds: contractions of up to 2304 terms
    # and 18432 rows, where the partial sums of the weight gradients are many and long.
    g0 = replace(W.gtsrb_sr(batch=8, frames=3), dtype="f32")
    g = g0.with_pattern(W.hybrid_pattern(g0))
    got, data = run_case(g, 3, seed=5)
    check_against_oracle(g, 3, got, data, "gtsrb_sr B=8/hybrid")
