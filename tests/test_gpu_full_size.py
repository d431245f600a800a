"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times (sr_rollout through captured HIP graphs).  The oracle runs as many frames as it finishes in
about a minute on the host; every element of every node is compared at the last of those frames and
the output node at all of them."""
import sys
import time

import numpy as np
import pytest

import workloads as W
from gpu_util import to_device, max_abs_rel

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def run_full(g, T_check, seed=0):
    import torch
    import paper_1806_04965_amd as sr
    from oracle import rollout as orc
    w, b, x = W.make_case(g, seed=seed, frames=T_check)
    mode = "bf16" if g.dtype == "bf16" else "f64"
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    ins = g.input_nodes()
    xd = [to_device(x[v], g.dtype) for v in ins]
    n = g.nodes[g.out_node]
    out = torch.empty((T_check, g.batch, n.height, n.width, n.channels), dtype=dev.tdtype, device="cuda")
    dev.rollout(xd, T_check, g.out_node, out)
    dev.synchronize()
    got_out = out.float().cpu().numpy().astype(np.float64)
    # oracle, frame by frame (prints progress: a frame of the largest graph takes seconds)
    r = orc.Rollout(g, w, b, mode)
    r.reset({v: x[v][0] for v in ins})
    worst = 0.0
    for t in range(1, T_check + 1):
        t0 = time.time()
        X = r.step({v: x[v][t] for v in ins})
        e = max_abs_rel(got_out[t - 1], X[g.out_node])
        worst = max(worst, e)
        print(f"[full] {g.name} frame {t}/{T_check}: oracle {time.time() - t0:.1f} s, out-node err {e:.2e}", flush=True)
        assert e <= TOL[g.dtype], (g.name, t, e)
    for v in range(len(g.nodes)):
        gv = dev.get_state(v).float().cpu().numpy().astype(np.float64)
        e = max_abs_rel(gv, X[v])
        worst = max(worst, e)
        assert e <= TOL[g.dtype], (g.name, "node", v, e)
    info = dev.info()
    dev.close()
    print(f"[full] {g.name}: worst max-abs-rel {worst:.3e}, launches/frame {info['launches_per_frame']}", flush=True)
    sys.stdout.flush()
    return info


def test_tiny_sr_full():
    g = W.tiny_sr()
    run_full(g, g.frames)


def test_cifar_sr_full_streaming():
    g = W.cifar_sr()
    info = run_full(g, g.frames)
    assert info["launches_per_frame"] == 1


@pytest.mark.parametrize("pattern", ["sequential", "hybrid"])
def test_cifar_sr_full_patterns(pattern):
    g = W.cifar_patterns()[pattern]
    run_full(g, g.frames)


@pytest.mark.timeout(600)
def test_gtsrb_sr_full_batch():
    g = W.gtsrb_sr()
    info = run_full(g, 6)
    assert info["launches_per_frame"] == 1


@pytest.mark.timeout(600)
def test_hires_sr_full_resolution():
    g = W.hires_sr()
    run_full(g, 8)


def test_full_rollout_is_deterministic_and_matches_stepping():
    # all T frames of the largest configuration: two rollouts agree bit for bit, and so does
    # stepping frame by frame (properties that hold at any size)
    import torch
    import paper_1806_04965_amd as sr
    g = W.gtsrb_sr()
    w, b, x = W.make_case(g, seed=0)
    dev = sr.SrGraph(g)
    dev.set_parameters(w, b)
    xd = [to_device(x[v], g.dtype) for v in g.input_nodes()]
    n = g.nodes[g.out_node]
    outs = []
    for _ in range(2):
        out = torch.empty((g.frames, g.batch, 1, 1, n.channels), dtype=dev.tdtype, device="cuda")
        dev.rollout(xd, g.frames, g.out_node, out)
        dev.synchronize()
        outs.append(out.clone())
    assert torch.equal(outs[0], outs[1])
    dev.reset([xi[0] for xi in xd])
    for t in range(1, g.frames + 1):
        dev.frame_step([xi[t] for xi in xd])
    last = dev.get_state(g.out_node)
    assert torch.equal(last, outs[0][-1])
    assert torch.isfinite(outs[0].float()).all()
    dev.close()
