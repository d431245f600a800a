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


def bf16_ulp(a):
    """Spacing of bfloat16 values (8 significant bits) at the magnitude of each element."""
    _, e = np.frexp(np.maximum(np.abs(np.asarray(a, dtype=np.float64)), 2.0 ** -120))
    return np.ldexp(1.0, e - 8)


# One frame computed from IDENTICAL stored states differs between the library (products exact,
# float32 sums in the matrix cores' order) and the oracle (float64 sums) only where the float32
# sum error moves a value across a bfloat16 rounding boundary: such an element is then one
# bfloat16 step off, everything else is bit-identical.  The sum error itself is at most about
# K * 2^-24 * sum|w x| (K <= 14k terms) and typically sqrt(K) * 2^-24 of the tensor's scale, which
# is what the absolute floor below covers for elements much smaller than the tensor's scale
# (their own bfloat16 step is far finer than the sum's float32 error).
ONE_STEP_FLOOR = 1e-4        # absolute floor, as a fraction of max|ref|
ONE_STEP_MAX_FLIPS = 2e-2    # largest accepted fraction of elements that are not bit-identical


def one_step_check(got, ref, label=""):
    """Tight check of one teacher-forced frame (bf16 graphs): every element within one bfloat16
    step of the oracle's (plus the floor above) and at most ONE_STEP_MAX_FLIPS of them different at
    all.  Returns (fraction different, largest error in bfloat16 steps of the element)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = float(np.abs(ref).max())
    assert scale > 0, f"{label}: the reference tensor is all zero: nothing is being compared"
    d = np.abs(got - ref)
    step = bf16_ulp(np.maximum(np.abs(got), np.abs(ref)))
    bad = d > step + ONE_STEP_FLOOR * scale
    assert not bad.any(), (f"{label}: {int(bad.sum())} elements further than one bf16 step from the oracle, "
                           f"worst {float((d / step).max()):.1f} steps, max|d| {float(d.max()):.3e}, scale {scale:.3e}")
    flips = float((d > 0).mean())
    assert flips <= ONE_STEP_MAX_FLIPS, f"{label}: {flips:.2e} of the elements differ from the oracle"
    return flips, float((d / step).max())


def forced_step(dev, g, xd, X_prev, t):
    """One frame on the device from the ORACLE's frame t-1 states and input frame t: reset with
    input frame t-1, overwrite every other node's state with X_prev, step with input frame t.
    Returns the list of all node states (float64 arrays)."""
    import torch
    ins = g.input_nodes()
    dev.reset([xi[t - 1] for xi in xd])
    for v in range(len(g.nodes)):
        if v in ins:
            continue
        dev.set_state(v, torch.from_numpy(np.ascontiguousarray(X_prev[v])).to("cuda").to(dev.tdtype).contiguous())
    dev.frame_step([xi[t] for xi in xd])
    return [dev.get_state(v).float().cpu().numpy().astype(np.float64) for v in range(len(g.nodes))]


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


# ---------------------------------------------------------------------------
# training windows: the rectifier's kink
# ---------------------------------------------------------------------------
# A pre-activation that the float64 oracle computes as -1e-8 may come out of a float32 forward pass as
# +1e-8: the value of the rectifier is the same to rounding, its derivative is 0 on one side and 1 on
# the other, and the gradient of the window changes by a finite amount.  Both decisions are correct
# ones for a forward pass of finite precision; which elements are that close to zero is decided on the
# oracle's side alone (Window.near_kink with KINK_TAU, a few times the float32 forward error measured
# by the frame-update parity tests, <= 1.5e-6 of a tensor's largest element).  The library's gradients
# then have to equal the oracle's for ONE assignment of derivatives to those elements, to the same
# tolerance as everywhere else; the assignment is found by least squares on the bias gradients and
# then checked exactly on every tensor.
KINK_TAU = 4e-6
KINK_MAX = 32


def match_kinks(win, labels, got, base, verbose=None):
    """Which near-kink elements of the oracle's window carry the other derivative in the gradients
    `got` = (dtheta list, dbias list with None for input nodes)?  `base` = the oracle's (dtheta, dbias)
    without toggles.  Returns the (frame, node, flat index) list to pass to Window.backward(flips=...)."""
    cand = win.near_kink(KINK_TAU)
    assert len(cand) <= KINK_MAX, f"{len(cand)} elements within {KINK_TAU} of the rectifier's kink: case too large"
    if not cand:
        return []
    nodes = [v for v in range(len(base[1])) if got[1][v] is not None]

    def flat(dth, db):
        return np.concatenate([np.asarray(t, dtype=np.float64).ravel() for t in dth] +
                              [np.asarray(db[v], dtype=np.float64).ravel() for v in nodes])

    f0 = flat(*base)
    cols = []
    for c in cand:
        dth, db, _ = win.backward(labels, flips=[c])
        cols.append(flat(dth, db) - f0)
    A = np.stack(cols, axis=1)
    live = np.abs(A).max(axis=0) > 0          # a toggle where no gradient arrives changes nothing
    sol = np.zeros(len(cand))
    if live.any():
        sol[live] = np.linalg.lstsq(A[:, live], flat(got[0], got[1]) - f0, rcond=None)[0]
    chosen = [c for c, s in zip(cand, sol) if s > 0.5]
    if verbose is not None:
        print(f"[kink] {verbose}: {len(cand)} elements within {KINK_TAU:g} of the kink, {len(chosen)} taken on the other "
              f"side: {chosen}", flush=True)
    return chosen
