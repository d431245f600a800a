"""GPU parity on the paper's own networks (App. A2: the MNIST nets FF / S / SR and the CIFAR10 family
DSR0..DSR6, plus DSR4 without self-recurrence for GTSRB) at the batch sizes of Tab. A1 (128 / 64 /
16), under the streaming and the sequential rollout pattern, every node after every frame against
the CPU oracle; and the claim of Sec. 4 / Fig. 3f on the device: under the streaming rollout the
first output that depends on the input appears after shortest-path-many frames (4 for every DSRk),
under the sequential rollout after one frame."""
import numpy as np
import pytest

import workloads as W
from oracle import theory as th
from gpu_util import gpu_states_by_steps, gpu_rollout, oracle_states, compare_all, one_step_check

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
MODE = {"f32": "f64", "bf16": "bf16"}
PATTERNS = {"streaming": W.streaming_pattern, "sequential": W.sequential_pattern}


def longest_path(g):
    """Number of edges on the longest input-to-output path that uses no backward or self edge:
    the inference factor of the sequential pattern (Eq. 6)."""
    pairs = [(e.src, e.dst) for e in g.edges]
    return th.inference_factor(len(g.nodes), pairs, W.sequential_pattern(g))


@pytest.mark.parametrize("pattern", ["streaming", "sequential"])
@pytest.mark.parametrize("name", list(W.PAPER_CONFIGS))
def test_paper_network_at_paper_batch_size(name, pattern):
    import paper_1806_04965_amd as sr
    g0 = W.PAPER_CONFIGS[name]()
    g = g0.with_pattern(PATTERNS[pattern](g0))
    T = longest_path(g0) + 2            # every node informed through its longest path, plus two frames
    w, b, x = W.make_case(g, seed=31, bias_scale=0.1, frames=T)
    got, info, work = gpu_states_by_steps(g, w, b, x, T)
    ref = oracle_states(g, w, b, x, T, MODE[g.dtype])
    for v in ref:
        for t in range(T):
            assert np.abs(ref[v][t]).max() > 0, (name, v, t)
    worst = compare_all(got, ref, TOL[g.dtype], f"{name}/{pattern}")
    # the nodes of the first update step of frame 1 (all nodes, under the streaming pattern) are computed
    # from identical stored states on both sides (the inputs and zeros): within one bf16 step
    if g.dtype == "bf16":
        for v in ref:
            if info["levels"][v] == 1:
                one_step_check(got[v][0], ref[v][0], f"{name}/{pattern} frame 1 node {v}")
    # which kernel computed what: every convolution node of the bf16 nets runs on matrix-core tiles
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    kinds, tile_kernel = dev.node_kernels(), dev.tile_kernel()
    dev.close()
    conv_nodes = sorted({e.dst for e in g.edges if e.kind == "conv"})
    if g.dtype == "bf16":
        # the stride-4 edges into the 4x4x512 node HD are staged as phase planes by the 4-wave kernel;
        # with all nodes on it the sequential pattern runs dependency-driven: one launch per frame
        assert tile_kernel == 1, (name, tile_kernel)
        assert all(kinds[v] == 1 for v in conv_nodes), (name, kinds)
        assert info["launches_per_frame"] == 1, (name, info)
    else:
        assert tile_kernel == 0 and all(kinds[v] == 3 for v in conv_nodes), (name, kinds)
    assert info["inference_factor"] == (1 if pattern == "streaming" else longest_path(g0))
    print(f"[paper] {name}/{pattern} B={g.batch} T={T}: worst max-abs-rel {worst:.3e} (tol {TOL[g.dtype]}), "
          f"F(R)={info['inference_factor']}, launches/frame {info['launches_per_frame']}, node kernels {kinds}", flush=True)


@pytest.mark.parametrize("pattern", ["streaming", "sequential"])
@pytest.mark.parametrize("name", ["dsr2", "gtsrb_dsr4"])
def test_paper_network_on_the_eight_wave_kernel(name, pattern):
    # the second tile kernel cuts the stride-4 edges by row phase only; same networks, same bar
    g0 = W.PAPER_CONFIGS[name]()
    g = g0.with_pattern(PATTERNS[pattern](g0))
    T = longest_path(g0) + 2
    w, b, x = W.make_case(g, seed=33, bias_scale=0.1, frames=T)
    got, info, work = gpu_states_by_steps(g, w, b, x, T, options={4: 2})
    ref = oracle_states(g, w, b, x, T, "bf16")
    worst = compare_all(got, ref, TOL["bf16"], f"{name}/{pattern}/8-wave")
    assert info["launches_per_frame"] == info["inference_factor"]
    print(f"[paper] {name}/{pattern} on the 8-wave kernel: worst max-abs-rel {worst:.3e}", flush=True)


@pytest.mark.parametrize("k", range(7))
def test_first_response_frame_of_the_dsr_family(k):
    # zero biases and zero initial state: the output is exactly zero until the input has reached it
    g0 = W.dsr_net(k, batch=2, frames=6)
    pairs = [(e.src, e.dst) for e in g0.edges]
    assert th.shortest_path_length(len(g0.nodes), pairs, g0.out_node) == 4
    w, b, x = W.make_case(g0, seed=40 + k, frames=6)
    out = gpu_rollout(g0.with_pattern(W.streaming_pattern(g0)), w, b, x, 6)
    for t in range(1, 4):
        assert np.all(out[t - 1] == 0.0), (k, t)
    assert np.any(out[3] != 0.0), k
    out_seq = gpu_rollout(g0.with_pattern(W.sequential_pattern(g0)), w, b, x, 6)
    assert np.any(out_seq[0] != 0.0), k
