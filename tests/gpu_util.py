"""Helpers shared by the GPU parity tests: run a workload through the C-ABI library and through the
CPU oracle on the same seeded arrays, and compare with the max-abs-rel metric."""
from __future__ import annotations

import numpy as np


def to_device(x, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.float().contiguous()


def max_abs_rel(got, ref):
    """max |g - o| / max(max |o|, 1e-6) over one tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-6))


def gpu_states_by_steps(g, w, b, x, T, options=None, nodes=None):
    """reset + T frame_steps; returns {v: [T arrays]} of every requested node after every frame."""
    import paper_1806_04965_amd as sr
    dev = sr.SrGraph(g, options=options)
    dev.set_parameters(w, b)
    ins = g.input_nodes()
    xd = {v: to_device(x[v], g.dtype) for v in ins}
    nodes = list(range(len(g.nodes))) if nodes is None else list(nodes)
    dev.reset([xd[v][0] for v in ins])
    out = {v: [] for v in nodes}
    for t in range(1, T + 1):
        dev.frame_step([xd[v][t] for v in ins])
        for v in nodes:
            out[v].append(dev.get_state(v).float().cpu().numpy().astype(np.float64))
    info = dev.info()
    work = dev.work()
    dev.close()
    return out, info, work


def gpu_rollout(g, w, b, x, T, out_node=None, options=None, return_dev=False):
    import torch
    import paper_1806_04965_amd as sr
    out_node = g.out_node if out_node is None else out_node
    dev = sr.SrGraph(g, options=options)
    dev.set_parameters(w, b)
    ins = g.input_nodes()
    xd = [to_device(x[v], g.dtype) for v in ins]
    n = g.nodes[out_node]
    out = torch.empty((T, g.batch, n.height, n.width, n.channels), dtype=dev.tdtype, device="cuda")
    dev.rollout(xd, T, out_node, out)
    dev.synchronize()
    res = out.float().cpu().numpy().astype(np.float64)
    if return_dev:
        return res, dev
    dev.close()
    return res


def oracle_states(g, w, b, x, T, mode, nodes=None):
    from oracle import rollout as orc
    nodes = list(range(len(g.nodes))) if nodes is None else list(nodes)
    res = orc.rollout(g, w, b, x, T=T, keep=nodes, mode=mode)
    return {v: [res[v][t] for t in range(T)] for v in nodes}


def compare_all(got, ref, tol, label=""):
    worst = 0.0
    for v in ref:
        for t, (a, o) in enumerate(zip(got[v], ref[v])):
            e = max_abs_rel(a, o)
            worst = max(worst, e)
            assert e <= tol, f"{label} node {v} frame {t + 1}: max-abs-rel {e:.3e} > {tol}"
    return worst
