"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on
the same seeded inputs.  Tolerances: max-abs-rel <= 1e-4 for fp32 graphs (oracle in float64),
<= 2e-2 for bf16 graphs (oracle emulating the bf16 storage points)."""
import numpy as np
import pytest

import workloads as W
from workloads.graphs import Node, Edge, Graph, ACT_IDENTITY, ACT_RELU
from gpu_util import (gpu_states_by_steps, gpu_rollout, oracle_states, compare_all, max_abs_rel,
                      to_device as to_device_)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
MODE = {"f32": "f64", "bf16": "bf16"}
OPT_DIRECT = {1: 1}
OPT_EAGER = {0: 0}
OPT_WIDE = {4: 2}     # 8-wave tile kernel (both operands through LDS, stages loaded one ahead)


def check(g, seed=0, T=None, options=None, bias_scale=0.1, label=None):
    T = g.frames if T is None else T
    w, b, x = W.make_case(g, seed=seed, bias_scale=bias_scale, frames=T)
    got, info, work = gpu_states_by_steps(g, w, b, x, T, options)
    ref = oracle_states(g, w, b, x, T, MODE[g.dtype])
    worst = compare_all(got, ref, TOL[g.dtype], label or g.name)
    print(f"[parity] {label or g.name}: worst max-abs-rel {worst:.3e} (tol {TOL[g.dtype]}), "
          f"F(R)={info['inference_factor']}, mfma tiles={work['mfma_tiles']}", flush=True)
    return info, work


def test_tiny_sr_fp32_streaming_all_nodes_all_frames():
    g = W.tiny_sr()
    info, _ = check(g)
    assert info["inference_factor"] == 1


@pytest.mark.parametrize("pattern", ["sequential", "hybrid"])
def test_tiny_sr_fp32_other_patterns(pattern):
    g = W.tiny_sr()
    bits = W.sequential_pattern(g) if pattern == "sequential" else W.hybrid_pattern(g)
    check(g.with_pattern(bits), label=f"tiny_sr/{pattern}")


def test_mnist_sr_net_fp32_conv7_stride4_and_dense_edges():
    check(W.mnist_net("SR", batch=3, frames=5))


def test_cifar_small_bf16_direct_kernel():
    g = W.cifar_sr(batch=2, frames=4)
    _, work = check(g, options=OPT_DIRECT, label="cifar_sr/direct")
    assert work["mfma_tiles"] == 0


def test_cifar_small_bf16_mfma_streaming():
    g = W.cifar_sr(batch=4, frames=6)
    info, work = check(g)
    assert work["mfma_tiles"] > 0 and info["inference_factor"] == 1


def test_cifar_ragged_batch_bf16_mfma():
    # B=3: nodes 5 and 6 have 192 pixels, less than one 256-pixel tile; nodes 3, 4 end in a partial tile
    check(W.cifar_sr(batch=3, frames=4), seed=3, label="cifar_sr/B3")


@pytest.mark.parametrize("pattern", ["sequential", "hybrid"])
def test_cifar_patterns_bf16_mfma(pattern):
    g = W.cifar_patterns(batch=4, frames=5)[pattern]
    info, work = check(g, label=g.name)
    assert work["mfma_tiles"] > 0
    assert info["inference_factor"] == (7 if pattern == "sequential" else info["inference_factor"])


def test_gtsrb_small_bf16_mfma_feedback_and_long_skips():
    check(W.gtsrb_sr(batch=2, frames=4), seed=1)


def test_dsr2_bf16_conv5_and_stride4():
    check(W.dsr_net(2, batch=2, frames=5), seed=2)


def test_hires_reduced_bf16_mfma():
    # the high-resolution graph at 64x64 input (same nodes, edges and channel schedule)
    g = W.hires_sr(batch=1, frames=3)
    nodes = []
    for n in g.nodes:
        if n.name == "out":
            nodes.append(n)
        else:
            nodes.append(Node(n.name, n.channels, n.height // 4, n.width // 4, n.act))
    g2 = Graph("hires_sr", nodes, g.edges, 1, 3, "bf16", g.out_node)
    check(g2, seed=4, label="hires_sr/64x64")


def test_gap_head_with_several_pixel_slabs():
    # 24x24 source -> 576 pixels per image: the head sums 9 slabs, the last one to finish combines them
    nodes = [Node("in", 3, 24, 24, ACT_IDENTITY), Node("a", 32, 24, 24), Node("out", 7, 1, 1, ACT_IDENTITY)]
    edges = [Edge(0, 1), Edge(1, 1), Edge(1, 2, "gap_dense", 1, 1, 1, 0)]
    for dtype in ("bf16", "f32"):
        g = Graph("gap", nodes, edges, batch=3, frames=4, dtype=dtype, out_node=2)
        check(g, seed=8, label=f"gap_head/{dtype}")
        check(g.with_pattern([0, 1, 0]), seed=8, label=f"gap_head/{dtype}/sequential")


def test_k_split_on_and_off_agree_with_the_oracle():
    # deep nodes with few pixels are cut along the contraction; with the option off they are not
    g = W.cifar_sr(batch=4, frames=5)
    _, work_on = check(g, seed=11, label="cifar_sr/k-split on")
    _, work_off = check(g, seed=11, options={3: 0}, label="cifar_sr/k-split off")
    assert work_on["mfma_tiles"] > work_off["mfma_tiles"]


def test_recording_a_hidden_node():
    g = W.cifar_sr(batch=2, frames=5)
    w, b, x = W.make_case(g, seed=9)
    got = gpu_rollout(g, w, b, x, 5, out_node=3)
    ref = oracle_states(g, w, b, x, 5, "bf16", nodes=[3])[3]
    for t in range(5):
        assert max_abs_rel(got[t], ref[t]) <= 2e-2


def test_rollout_equals_frame_steps_and_hipgraph_equals_eager():
    g = W.cifar_sr(batch=2, frames=11)       # 11 frames: one 8-frame graph + 3 single frames
    w, b, x = W.make_case(g, seed=5, bias_scale=0.1)
    T = g.frames
    a = gpu_rollout(g, w, b, x, T)
    c = gpu_rollout(g, w, b, x, T, options=OPT_EAGER)
    steps, _, _ = gpu_states_by_steps(g, w, b, x, T, nodes=[g.out_node])
    np.testing.assert_array_equal(a, c)
    np.testing.assert_array_equal(a, np.stack(steps[g.out_node]))
    ref = oracle_states(g, w, b, x, T, "bf16", nodes=[g.out_node])[g.out_node]
    for t in range(T):
        assert max_abs_rel(a[t], ref[t]) <= 2e-2


def test_checkpoint_restore_continues_bit_exactly():
    import paper_1806_04965_amd as sr
    from gpu_util import to_device
    g = W.cifar_sr(batch=2, frames=6)
    w, b, x = W.make_case(g, seed=6)
    xd = to_device(x[0], "bf16")
    full, _, _ = gpu_states_by_steps(g, w, b, x, 6, nodes=range(len(g.nodes)))
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    dev.reset([xd[0]])
    for t in range(1, 4):
        dev.frame_step([xd[t]])
    saved = [dev.get_state(v) for v in range(len(g.nodes))]
    dev.close()
    dev2 = sr.SrGraph(g)
    dev2.set_parameters(w, b)
    dev2.reset(None)
    for v, s in enumerate(saved):
        dev2.set_state(v, s)
    for t in range(4, 7):
        dev2.frame_step([xd[t]])
    for v in range(1, len(g.nodes)):
        np.testing.assert_array_equal(dev2.get_state(v).float().cpu().numpy(), full[v][-1])
    dev2.close()


def test_first_response_frame_on_gpu():
    # exact zeros at the output until shortest-path-many frames have passed (zero bias)
    g = W.cifar_sr(batch=2, frames=7)
    w, b, x = W.make_case(g, seed=7)
    out = gpu_rollout(g, w, b, x, 7)
    for t in range(1, 5):
        assert np.all(out[t - 1] == 0.0)
    assert np.any(out[4] != 0.0)


def test_two_inputs_and_unordered_node_ids():
    # node ids in no particular order: outputs first, two input nodes last
    nodes = [Node("out", 5, 1, 1, ACT_IDENTITY), Node("b", 32, 8, 8), Node("a", 32, 16, 16),
             Node("in2", 4, 16, 16, ACT_IDENTITY), Node("in1", 3, 16, 16, ACT_IDENTITY)]
    edges = [Edge(4, 2), Edge(3, 2), Edge(2, 1, stride=2), Edge(1, 1), Edge(1, 0, "gap_dense", 1, 1, 1, 0),
             Edge(3, 1, stride=2)]
    for dtype in ("bf16", "f32"):
        g = Graph("two_in", nodes, edges, batch=3, frames=4, dtype=dtype, out_node=0)
        assert g.input_nodes() == [3, 4]
        check(g, seed=12, label=f"two_in/{dtype}")
        check(g.with_pattern([0, 1, 0, 1, 0, 1]), seed=12, label=f"two_in/{dtype}/hybrid")


def test_zero_frames_and_single_sample():
    import torch
    import paper_1806_04965_amd as sr
    from gpu_util import to_device
    g = W.cifar_sr(batch=1, frames=3)
    w, b, x = W.make_case(g, seed=13)
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    xd = to_device(x[0], "bf16")
    dev.rollout([xd], 0, g.out_node, None)          # T = 0: only the initial state
    dev.synchronize()
    assert dev.frame_index() == 0
    np.testing.assert_array_equal(dev.get_state(0).float().cpu().numpy(), xd[0].float().cpu().numpy())
    for v in range(1, len(g.nodes)):
        assert float(dev.get_state(v).float().abs().max()) == 0.0
    dev.close()
    check(g, seed=13, label="cifar_sr/B1")


def test_errors_on_the_device_path():
    import paper_1806_04965_amd as sr
    from gpu_util import to_device
    g = W.tiny_sr()
    w, b, x = W.make_case(g, seed=14)
    dev = sr.SrGraph(g)
    xd = to_device(x[0], "f32")
    with pytest.raises(sr.SrError) as ei:
        dev.frame_step([xd[1]])
    assert ei.value.name == "SR_ERR_STATE"          # no sr_reset yet
    with pytest.raises(sr.SrError) as ei:
        dev.reset([xd[0]])
    assert ei.value.name == "SR_ERR_STATE"          # weights missing
    dev.set_parameters(w, b)
    dev.reset([xd[0]])
    dev.frame_step([xd[1]])
    dev.synchronize()
    with pytest.raises(sr.SrError) as ei:
        dev.set_weights(0, np.zeros(5, np.float32))
    assert ei.value.name == "SR_ERR_ARG"
    dev.close()


@pytest.mark.parametrize("name", ["cifar", "cifar_ragged", "gtsrb", "hires"])
def test_eight_wave_tile_kernel_streaming(name):
    g = {"cifar": lambda: W.cifar_sr(batch=4, frames=4), "cifar_ragged": lambda: W.cifar_sr(batch=3, frames=3),
         "gtsrb": lambda: W.gtsrb_sr(batch=3, frames=3), "hires": lambda: W.hires_sr(batch=1, frames=2)}[name]()
    info, work = check(g, seed=21, options=OPT_WIDE, label=f"{name}/8-wave kernel")
    assert work["mfma_tiles"] > 0 and info["inference_factor"] == 1


def test_eight_wave_tile_kernel_sequential_pattern_and_no_split():
    g = W.cifar_sr(batch=4, frames=3)
    check(g.with_pattern(W.sequential_pattern(g)), seed=22, options=OPT_WIDE, label="cifar_sr/sequential/8-wave kernel")
    check(W.hires_sr(batch=1, frames=2), seed=23, options={4: 2, 3: 0}, label="hires_sr/8-wave kernel, no K-split")


def test_eight_wave_tile_kernel_rollout_in_hipgraph_matches_steps():
    g = W.gtsrb_sr(batch=2, frames=5)
    w, b, x = W.make_case(g, seed=24, bias_scale=0.1, frames=5)
    a = gpu_rollout(g, w, b, x, 5, options=OPT_WIDE)
    c = gpu_rollout(g, w, b, x, 5, options={4: 2, 0: 0})
    assert np.array_equal(a, c)
    ref = oracle_states(g, w, b, x, 5, "bf16", nodes=[g.out_node])
    for t in range(5):
        assert max_abs_rel(a[t], ref[g.out_node][t]) <= TOL["bf16"]


def test_tile_kernel_choice_is_reported():
    import paper_1806_04965_amd as sr
    # CIFAR-shaped: every patch fits the 4-wave kernel; DSR0 at its batch of 64: the stride-4 edges into the 4x4 node
    # fit as phase planes; fp32 graphs have no MFMA node; an explicit choice is reported back
    for g, options, want in ((W.cifar_sr(batch=2, frames=2), None, 1), (W.dsr_net(0, batch=64, frames=2), None, 1),
                             (W.tiny_sr(), None, 0), (W.cifar_sr(batch=2, frames=2), OPT_WIDE, 2)):
        dev = sr.SrGraph(g, options=options)
        w, b, _ = W.make_case(g, seed=1)
        dev.set_parameters(w, b)
        assert dev.tile_kernel() == want, (g.name, options)
        dev.close()


OPT_FLOW_ON, OPT_FLOW_OFF = {5: 1}, {5: 0}


@pytest.mark.parametrize("pattern", ["streaming", "hybrid", "sequential"])
def test_dependency_driven_execution_equals_one_launch_per_update_step(pattern):
    # The same rollout dependency-driven (one launch for every update step of up to 8 frames; a work item
    # waits for the nodes it reads) and with one launch per update step: bit-identical outputs over
    # 19 frames (two 8-frame launches + 3 single frames), every node's final state too, and no
    # dependency wait may have given up.  K-split tiles, head and input-staging items all take part.
    import paper_1806_04965_amd as sr
    g0 = W.cifar_sr(batch=6, frames=19)
    g = g0.with_pattern({"streaming": W.streaming_pattern, "hybrid": W.hybrid_pattern,
                         "sequential": W.sequential_pattern}[pattern](g0))
    w, b, x = W.make_case(g, seed=41, bias_scale=0.1)
    outs, finals = {}, {}
    for name, opt in (("flow", OPT_FLOW_ON), ("steps", OPT_FLOW_OFF)):
        res, dev = gpu_rollout(g, w, b, x, g.frames, options=opt, return_dev=True)
        health, info = dev.health(), dev.info()
        assert health["dependency_driven"] == (name == "flow")
        assert health["dependency_timeouts"] == 0
        assert info["launches_per_frame"] == (1 if name == "flow" else max(1, info["inference_factor"]))
        outs[name] = res
        finals[name] = [dev.get_state(v).float().cpu().numpy() for v in range(len(g.nodes))]
        dev.close()
    np.testing.assert_array_equal(outs["flow"], outs["steps"])
    for a, c in zip(finals["flow"], finals["steps"]):
        np.testing.assert_array_equal(a, c)
    ref = oracle_states(g, w, b, x, g.frames, "bf16", nodes=[g.out_node])[g.out_node]
    for t in range(g.frames):
        assert np.abs(ref[t]).max() > 0
        assert max_abs_rel(outs["flow"][t], ref[t]) <= TOL["bf16"]


def test_dependency_driven_default_and_larger_graphs():
    # default: dependency-driven exactly when a frame has more than one update step
    import paper_1806_04965_amd as sr
    for g, want in ((W.cifar_sr(batch=2, frames=2), False),
                    (W.cifar_patterns(batch=2, frames=2)["sequential"], True), (W.tiny_sr(), False)):
        dev = sr.SrGraph(g)
        w, b, _ = W.make_case(g, seed=1)
        dev.set_parameters(w, b)
        assert dev.health()["dependency_driven"] == want, g.name
        dev.close()
    # forced on for streaming graphs with feedback, long skips and K-split tiles: against the oracle
    for g, seed in ((W.gtsrb_sr(batch=3, frames=10), 43), (W.hires_sr(batch=1, frames=3), 44)):
        if g.name == "hires_sr":
            g = Graph("hires_sr", [n if n.name == "out" else Node(n.name, n.channels, n.height // 4, n.width // 4, n.act)
                                   for n in g.nodes], g.edges, 1, 3, "bf16", g.out_node)
        check(g, seed=seed, options=OPT_FLOW_ON, label=f"{g.name}/dependency-driven")
        hy = g.with_pattern(W.hybrid_pattern(g))
        check(hy, seed=seed, label=f"{g.name}/hybrid (dependency-driven by default)")


def test_tile_spanning_more_than_127_images():
    # a 1x3 node at batch 160: one 512-pixel tile would span 170 images, more than the tile kernels'
    # packed image offset holds; the planner has to choose a shape (or kernel) that stays within it
    nodes = [Node("in", 16, 1, 3, ACT_IDENTITY), Node("a", 32, 1, 3), Node("out", 5, 1, 1, ACT_IDENTITY)]
    edges = [Edge(0, 1, "conv", 3, 3, 1, 1), Edge(1, 1, "conv", 3, 3, 1, 1), Edge(1, 2, "gap_dense", 1, 1, 1, 0)]
    g = Graph("thin", nodes, edges, batch=160, frames=3, dtype="bf16", out_node=2)
    for options in (None, OPT_WIDE):
        check(g, seed=17, options=options, label=f"thin/B160/{options}")


def test_mfma_nodes_of_the_benchmark_configurations():
    # which kernel the planner gives every node: all convolution nodes of the three bf16 benchmark
    # configurations run on matrix-core tiles (4-wave kernel), their heads as head items
    import paper_1806_04965_amd as sr
    for g in (W.cifar_sr(), W.gtsrb_sr(), W.hires_sr()):
        dev = sr.SrGraph(g)
        w, b, _ = W.make_case(g, seed=1, frames=0)
        dev.set_parameters(w, b)
        kinds = dev.node_kernels()
        assert dev.tile_kernel() == 1
        dev.close()
        for v, n in enumerate(g.nodes):
            want = 0 if v in g.input_nodes() else (4 if v == g.out_node else 1)
            assert kinds[v] == want, (g.name, n.name, kinds)


def test_two_graphs_alive_interleaved_and_recreated():
    # Two graphs with K-split nodes live side by side, stepped alternately; then both are destroyed and
    # created again (the partial-sum scratch of the first pair is handed to the second).  Every
    # graph's output must match its own single-graph run bit for bit and the oracle within tolerance.
    import paper_1806_04965_amd as sr
    ga = W.cifar_sr(batch=4, frames=5)
    gb = W.gtsrb_sr(batch=2, frames=5)
    cases = []
    for g, seed in ((ga, 21), (gb, 22)):
        w, b, x = W.make_case(g, seed=seed)
        alone, _, work = gpu_states_by_steps(g, w, b, x, g.frames, nodes=[g.out_node])
        ref = oracle_states(g, w, b, x, g.frames, "bf16", nodes=[g.out_node])[g.out_node]
        cases.append((g, w, b, x, alone[g.out_node], ref))
    for round_ in range(2):
        devs = []
        for g, w, b, x, _, _ in cases:
            d = sr.SrGraph(g)
            d.set_parameters(w, b)
            ins = g.input_nodes()
            xd = {v: to_device_(x[v], g.dtype) for v in ins}
            d.reset([xd[v][0] for v in ins])
            devs.append((d, xd, ins))
        for t in range(1, 6):
            for (d, xd, ins), (g, _, _, _, alone, ref) in zip(devs, cases):
                d.frame_step([xd[v][t] for v in ins])
            for (d, xd, ins), (g, _, _, _, alone, ref) in zip(devs, cases):
                got = d.get_state(g.out_node).float().cpu().numpy().astype(np.float64)
                np.testing.assert_array_equal(got, alone[t - 1])
                assert max_abs_rel(got, ref[t - 1]) <= 2e-2
        for d, _, _ in devs:
            d.close()


def test_dependency_wait_that_gives_up_is_counted_and_every_kernel_ends():
    # failure path of the dependency-driven launch, forced from the host: with a spin limit of 0 a wait
    # gives up at its first unsatisfied poll; the work item goes on (results undefined), the kernels
    # end normally, and the graph reports the waits that gave up.  sr_reset clears the count.
    import paper_1806_04965_amd as sr
    g0 = W.cifar_sr(batch=4, frames=4)
    g = g0.with_pattern(W.sequential_pattern(g0))
    w, b, x = W.make_case(g, seed=3, bias_scale=0.1, frames=4)
    dev = sr.SrGraph(g, options={6: 0})
    dev.set_parameters(w, b)
    xd = [to_device_(x[v], g.dtype) for v in g.input_nodes()]
    dev.rollout(xd, 4)
    dev.synchronize()
    h = dev.health()
    assert h["dependency_driven"] and h["dependency_timeouts"] > 0, h
    dev.reset([xi[0] for xi in xd])
    assert dev.health()["dependency_timeouts"] == 0
    dev.close()
    with pytest.raises(sr.SrError):
        sr.SrGraph(g, options={6: -1})


@pytest.mark.parametrize("name", ["cifar_seq", "cifar_hybrid", "dsr2_seq", "hires_seq"])
def test_depth_ordered_multi_frame_launch_equals_frame_after_frame(name):
    # a dependency-driven rollout dispatches the work items of 8 frames in the order of their depth in the rollout
    # window of those frames (Eq. 5 over update steps); the arithmetic of every item is the same as when the frames
    # are dispatched one after the other, so the outputs are bit-identical -- and both match the oracle
    g0 = {"cifar_seq": lambda: W.cifar_sr(batch=4, frames=19), "cifar_hybrid": lambda: W.cifar_sr(batch=4, frames=19),
          "dsr2_seq": lambda: W.dsr_net(2, batch=8, frames=17), "hires_seq": lambda: W.hires_sr(batch=1, frames=16)}[name]()
    pat = W.hybrid_pattern if name.endswith("hybrid") else W.sequential_pattern
    g = g0.with_pattern(pat(g0))
    T = g.frames
    w, b, x = W.make_case(g, seed=61, bias_scale=0.1, frames=T)
    a, dev = gpu_rollout(g, w, b, x, T, return_dev=True)
    h = dev.health()
    dev.close()
    assert h["dependency_driven"] and h["dependency_timeouts"] == 0
    c = gpu_rollout(g, w, b, x, T, options={7: 0})
    assert np.array_equal(a, c)
    ref = oracle_states(g, w, b, x, T, "bf16", nodes=[g.out_node])
    for t in range(T):
        assert np.abs(ref[g.out_node][t]).max() > 0
        assert max_abs_rel(a[t], ref[g.out_node][t]) <= TOL["bf16"], (name, t)


@pytest.mark.parametrize("frames_per_launch", [1, 2, 5, 16])
def test_depth_ordered_launches_of_other_lengths(frames_per_launch):
    # the order table is built for the configured number of frames per launch; a rollout whose length is no
    # multiple of it finishes with single-frame launches.  All of them equal one launch per update step.
    g0 = W.cifar_sr(batch=3, frames=13)
    g = g0.with_pattern(W.sequential_pattern(g0))
    w, b, x = W.make_case(g, seed=62, bias_scale=0.1, frames=13)
    a = gpu_rollout(g, w, b, x, 13, options={2: frames_per_launch})
    c = gpu_rollout(g, w, b, x, 13, options={5: 0})
    assert np.array_equal(a, c)
    assert np.abs(a[-1]).max() > 0
