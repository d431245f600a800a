"""Seeded synthetic weights and input frame sequences.

Stand-ins for the noisy MNIST / CIFAR10 / GTSRB sequences of the paper's
experiments (Sec. 4, Tab. A1), which are not available offline: same shapes,
value ranges and per-frame perturbation structure, generated on the host from
``numpy.random.default_rng(seed)``.  The same arrays are handed to the CPU
oracle and to the GPU library; nothing here evaluates a network.
"""
from __future__ import annotations

import numpy as np

from .graphs import Graph, KIND_CONV, KIND_DENSE, KIND_GAP_DENSE


def edge_weight_shape(g: Graph, ei: int):
    """Weight layout of an edge: [kh][kw][Cin][Cout]; a dense edge is a valid
    convolution whose kernel covers the whole source, a GAP+dense edge has a
    1x1 kernel."""
    e = g.edges[ei]
    s, d = g.nodes[e.src], g.nodes[e.dst]
    if e.kind == KIND_CONV:
        return (e.kh, e.kw, s.channels, d.channels)
    if e.kind == KIND_DENSE:
        return (s.height, s.width, s.channels, d.channels)
    if e.kind == KIND_GAP_DENSE:
        return (1, 1, s.channels, d.channels)
    raise ValueError(e.kind)


def make_weights(g: Graph, seed: int = 0, bias_scale: float = 0.0, gain: float = 1.0):
    """He-normal weights with the fan-in of the node's concatenated incoming
    transformations: std = gain * sqrt(2 / sum_e Cin_e*kh_e*kw_e).  The sum over
    edges equals one convolution over the concatenated sources (App. A2), so this
    keeps a node's second moment independent of its in-degree.  Biases are zero
    unless ``bias_scale`` > 0 (then N(0, bias_scale^2), used by tests)."""
    rng = np.random.default_rng(seed)
    fan_in = [0] * len(g.nodes)
    for ei, e in enumerate(g.edges):
        kh, kw, cin, _ = edge_weight_shape(g, ei)
        fan_in[e.dst] += kh * kw * cin
    weights = []
    for ei, e in enumerate(g.edges):
        std = gain * np.sqrt(2.0 / fan_in[e.dst])
        w = rng.standard_normal(edge_weight_shape(g, ei), dtype=np.float32) * np.float32(std)
        weights.append(np.ascontiguousarray(w, dtype=np.float32))
    biases = []
    for n in g.nodes:
        if bias_scale > 0:
            b = rng.standard_normal(n.channels, dtype=np.float32) * np.float32(bias_scale)
        else:
            b = np.zeros(n.channels, dtype=np.float32)
        biases.append(b.astype(np.float32))
    return weights, biases


def _gauss_kernel(sigma: float):
    r = int(np.ceil(3 * sigma))
    x = np.arange(-r, r + 1, dtype=np.float64)
    k = np.exp(-0.5 * (x / sigma) ** 2)
    return k / k.sum()


def _blur2d(img: np.ndarray, sigma: float) -> np.ndarray:
    """Separable Gaussian blur with wrap-around borders, (H, W, C) array."""
    k = _gauss_kernel(sigma)
    r = len(k) // 2
    out = np.zeros_like(img)
    for i, kv in enumerate(k):
        out += kv * np.roll(img, i - r, axis=0)
    img2 = out
    out = np.zeros_like(img2)
    for i, kv in enumerate(k):
        out += kv * np.roll(img2, i - r, axis=1)
    return out


def make_inputs(g: Graph, seed: int = 0, recipe: str | None = None, frames: int | None = None):
    """Input frames x_in[v][t], t = 0..T, for every input node v, as float32
    arrays of shape (T+1, B, H, W, C).  Frame 0 is real data (the zero-th frame of
    the first rollout window holds the input); frames 1..T drive the T frame
    updates.

    recipes
      'uniform'    i.i.d. U[0,1) per pixel and frame (noisy-MNIST stand-in)
      'noisy_base' fixed N(0,1) image per sequence + fresh N(0, 0.5^2) noise per frame
      'occluded'   U[0,1) frames with one zeroed rectangle per frame and sample whose
                   area is U[0, 0.5] of the frame
      'video'      crop of a Gaussian-blurred (sigma = 2 px) N(0,1) canvas that moves
                   1 px per frame along a seeded random walk
    """
    T = g.frames if frames is None else frames
    if recipe is None:
        recipe = {"tiny_sr": "uniform", "cifar_sr": "noisy_base", "gtsrb_sr": "occluded",
                  "hires_sr": "video"}.get(g.name.split("/")[0], "uniform")
    rng = np.random.default_rng(seed + 1000003)
    out = {}
    for v in g.input_nodes():
        n = g.nodes[v]
        shape = (T + 1, g.batch, n.height, n.width, n.channels)
        if recipe == "uniform":
            x = rng.random(shape, dtype=np.float32)
        elif recipe == "noisy_base":
            base = rng.standard_normal(shape[1:], dtype=np.float32)
            x = base[None] + np.float32(0.5) * rng.standard_normal(shape, dtype=np.float32)
        elif recipe == "occluded":
            x = rng.random(shape, dtype=np.float32)
            H, W = n.height, n.width
            frac = rng.random((T + 1, g.batch)) * 0.5
            aspect = rng.uniform(0.5, 2.0, (T + 1, g.batch))
            cy = rng.random((T + 1, g.batch)) * H
            cx = rng.random((T + 1, g.batch)) * W
            for t in range(T + 1):
                for b in range(g.batch):
                    area = frac[t, b] * H * W
                    hh = np.sqrt(area * aspect[t, b])
                    ww = area / max(hh, 1e-9)
                    y0 = int(np.clip(np.floor(cy[t, b] - hh / 2), 0, H))
                    y1 = int(np.clip(np.ceil(cy[t, b] + hh / 2), 0, H))
                    x0 = int(np.clip(np.floor(cx[t, b] - ww / 2), 0, W))
                    x1 = int(np.clip(np.ceil(cx[t, b] + ww / 2), 0, W))
                    x[t, b, y0:y1, x0:x1, :] = 0.0
        elif recipe == "video":
            H, W = n.height, n.width
            x = np.empty(shape, dtype=np.float32)
            for b in range(g.batch):
                canvas = rng.standard_normal((H + 2 * (T + 1), W + 2 * (T + 1), n.channels))
                canvas = _blur2d(canvas, 2.0)
                canvas /= canvas.std()
                steps = rng.integers(0, 4, T + 1)
                y, xx = T + 1, T + 1
                for t in range(T + 1):
                    x[t, b] = canvas[y:y + H, xx:xx + W, :].astype(np.float32)
                    dy, dx = [(0, 1), (1, 0), (0, -1), (-1, 0)][int(steps[t])]
                    y, xx = y + dy, xx + dx
        else:
            raise ValueError(recipe)
        out[v] = np.ascontiguousarray(x, dtype=np.float32)
    return out


def make_case(g: Graph, seed: int = 0, bias_scale: float = 0.0, gain: float = 1.0,
              recipe: str | None = None, frames: int | None = None):
    """(weights, biases, inputs) for a graph, all float32."""
    w, b = make_weights(g, seed, bias_scale, gain)
    x = make_inputs(g, seed, recipe, frames)
    return w, b, x
