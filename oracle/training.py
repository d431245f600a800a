"""CPU oracle, part 3: one training window -- forward over an explicit rollout window of W frames,
the loss, and its gradients by backpropagation through the window (BPTT), in float64.

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import this package; the product path never does, and it shares no code with the GPU library.

What it computes.  The rollout window R_W of a network under a rollout pattern R (Sec. 3) is a
feed-forward graph over (frame, node) pairs: node v of frame i reads, over edge e = (u, v), node u
of frame i - R(e) (Eq. 2).  With the states of frame 0 given (zero for every node that has incoming
edges: training details of App. A2) and the input nodes given at all frames,

    a_v(i) = b_v + sum_{e=(u,v)} f_e(theta_e, x_u(i - R(e))),   x_v(i) = sigma_v(a_v(i)),   i = 1..W

and the loss is the mean over the W frames (and the batch) of the cross-entropy between
softmax(x_out(i)) and the labels (App. A2: the loss of a rolled-out network is the mean over the
single-frame prediction losses).  Because R_W is acyclic (a valid pattern), the gradient is the
ordinary reverse sweep over it: frames W..1, and inside a frame the update steps of the inference
tableau in reverse (Eq. 5), so that every (frame, node) has received the gradient of all its readers
before it is processed.  Weights are shared by the W copies of an edge: their gradients add up.

Pins (tests/test_oracle_training.py): central finite differences of the loss for every weight and
bias of tiny graphs under the streaming, hybrid and sequential patterns; the same windows rebuilt
from torch's CPU operators and differentiated by torch.autograd; softmax cross-entropy against its
closed-form gradient; the adjoint identity <f_e(x), y> = <x, f_e^T(y)> of every edge kind; what
Sec. 4 fixes: a window shorter than the shortest input-to-output path gives the weights of edges
that leave an input no gradient at all under the streaming pattern; and the gradient with the
rectifier's derivative toggled at chosen elements (see Window.near_kink) against torch.autograd on a
window whose rectifiers carry that derivative; dropout masks: finite differences and torch.autograd with
the same masks, masks of ones change nothing, a zero mask cuts a node off.  rmsprop_step: closed form of the first step, a constant
gradient's limit, and torch.optim.RMSprop over several steps.
"""
from __future__ import annotations

import numpy as np

from . import rollout as ro

ACT_IDENTITY = 0
ACT_RELU = 1


# ----------------------------------------------------------------------------
# edge transformations: adjoints
# ----------------------------------------------------------------------------

def _patches(x, kh, kw, stride, pad):
    """P[b,ho,wo,i,j,ci] = x[b, ho*s+i-p, wo*s+j-p, ci] (zero outside), as in rollout.conv2d_nhwc."""
    B, H, W, Cin = x.shape
    Ho = ro.conv_out_size(H, kh, stride, pad)
    Wo = ro.conv_out_size(W, kw, stride, pad)
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    P = np.empty((B, Ho, Wo, kh, kw, Cin), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            P[:, :, :, i, j, :] = xp[:, i:i + (Ho - 1) * stride + 1:stride, j:j + (Wo - 1) * stride + 1:stride, :]
    return P


def conv2d_backward(x, theta, stride, pad, dy):
    """Gradients of y = conv2d_nhwc(x, theta, stride, pad) given dL/dy:
       dtheta[i,j,ci,co] = sum_{b,ho,wo} x[b, ho*s+i-p, wo*s+j-p, ci] * dy[b,ho,wo,co]
       dx[b,h,w,ci]      = sum_{i,j,co : h = ho*s+i-p, w = wo*s+j-p} theta[i,j,ci,co] * dy[b,ho,wo,co]."""
    B, H, W, Cin = x.shape
    kh, kw, _, Cout = theta.shape
    Ho, Wo = dy.shape[1], dy.shape[2]
    P = _patches(x, kh, kw, stride, pad)
    dY = dy.reshape(B * Ho * Wo, Cout)
    dtheta = (P.reshape(B * Ho * Wo, kh * kw * Cin).T @ dY).reshape(kh, kw, Cin, Cout)
    dP = (dY @ theta.reshape(kh * kw * Cin, Cout).astype(np.float64).T).reshape(B, Ho, Wo, kh, kw, Cin)
    dxp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            dxp[:, i:i + (Ho - 1) * stride + 1:stride, j:j + (Wo - 1) * stride + 1:stride, :] += dP[:, :, :, i, j, :]
    return dxp[:, pad:pad + H, pad:pad + W, :], dtheta


def upsample_backward(dy, up):
    """Adjoint of nearest up-sampling: every source pixel collects its up x up block."""
    if up == 1:
        return dy
    B, H, W, C = dy.shape
    return dy.reshape(B, H // up, up, W // up, up, C).sum(axis=(2, 4))


def edge_backward(edge, theta, x, dy):
    """(dx, dtheta) of y_e = f_e(theta_e, x) (App. A1.2) given dL/dy_e."""
    theta = np.asarray(theta, dtype=np.float64)
    if edge.kind == "conv":
        return conv2d_backward(x, theta, edge.stride, edge.pad, upsample_backward(dy, edge.up))
    if edge.kind == "dense":
        B = x.shape[0]
        K = x.shape[1] * x.shape[2] * x.shape[3]
        d = dy.reshape(B, -1)
        dtheta = (x.reshape(B, K).T @ d).reshape(theta.shape)
        dx = (d @ theta.reshape(K, -1).T).reshape(x.shape)
        return dx, dtheta
    if edge.kind == "gap_dense":
        B, H, W, C = x.shape
        d = dy.reshape(B, -1)
        mean = x.mean(axis=(1, 2))
        dtheta = (mean.T @ d).reshape(theta.shape)
        dmean = d @ theta.reshape(theta.shape[2], theta.shape[3]).T
        dx = np.broadcast_to(dmean[:, None, None, :] / (H * W), x.shape).copy()
        return dx, dtheta
    raise ValueError(f"unknown edge kind {edge.kind!r}")


# ----------------------------------------------------------------------------
# loss
# ----------------------------------------------------------------------------

def softmax_cross_entropy(logits, labels):
    """Mean over the batch of -log softmax(logits)[label]; logits (B, C) or (B,1,1,C).  Returns
    (loss, dloss/dlogits) with the gradient shaped like `logits`."""
    z = np.asarray(logits, dtype=np.float64)
    shape = z.shape
    z = z.reshape(shape[0], -1)
    B = z.shape[0]
    zmax = z.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=1))
    loss = float((lse - z[np.arange(B), labels]).mean())
    p = np.exp(z - lse[:, None])
    p[np.arange(B), labels] -= 1.0
    return loss, (p / B).reshape(shape)


# ----------------------------------------------------------------------------
# the window
# ----------------------------------------------------------------------------

class Window:
    """Forward and backward sweep over the rollout window of size W."""

    def __init__(self, graph, weights, biases):
        ro.check_graph(graph)
        self.g = graph
        self.theta = [np.asarray(w, dtype=np.float64) for w in weights]
        self.bias = [np.asarray(b, dtype=np.float64) for b in biases]
        self.schedule = ro.frame_schedule(graph)
        self.inputs = self.schedule[0]
        self.src_edges = [[ei for ei, e in enumerate(graph.edges) if e.dst == v] for v in range(len(graph.nodes))]

    def forward(self, inputs, W, init=None, masks=None):
        """inputs[v]: (W+1,B,H,W,C) for every input node.  Returns X with X[i][v] the state of node v at
        frame i = 0..W (frame 0: `init[v]` or zeros for nodes with incoming edges).  The pre-activations
        a_v(i) are kept in self.A.
        masks (dropout, App. A2 training details): {v: (W+1,B,H,W,C)} multipliers of the node's state,
        x_v(i) = m_v(i) * sigma_v(a_v(i)); the caller draws them (0 with the dropout rate, 1/(1 - rate)
        otherwise, afresh for every frame and node: the paper does not say more than the rates).  Frame 0
        of a mask is not used."""
        g = self.g
        X = [[None] * len(g.nodes) for _ in range(W + 1)]
        A = [[None] * len(g.nodes) for _ in range(W + 1)]
        for v, n in enumerate(g.nodes):
            if v in self.inputs:
                for i in range(W + 1):
                    X[i][v] = np.asarray(inputs[v][i], dtype=np.float64)
            else:
                X[0][v] = (np.zeros((g.batch, n.height, n.width, n.channels)) if init is None
                           else np.asarray(init[v], dtype=np.float64))
        for i in range(1, W + 1):
            for level in self.schedule[1:]:
                for v in level:
                    n = g.nodes[v]
                    a = np.zeros((g.batch, n.height, n.width, n.channels)) + self.bias[v]
                    for ei in self.src_edges[v]:
                        e = g.edges[ei]
                        a = a + ro.edge_transform(e, self.theta[ei], X[i - e.bridge][e.src])
                    A[i][v] = a
                    X[i][v] = ro.activation(n.act, a)
                    if masks is not None and masks.get(v) is not None:
                        X[i][v] = X[i][v] * np.asarray(masks[v][i], dtype=np.float64)
        self.X, self.A, self.W, self.masks = X, A, W, masks
        return X

    def near_kink(self, tau_rel):
        """Elements of rectifier nodes whose pre-activation lies within tau_rel * max|x_v| of zero, as
        (frame, node, flat index) triples.  There the rectifier's derivative is not defined by the
        arithmetic of a finite-precision forward pass: a pre-activation that is +1e-8 in one summation
        order is -1e-8 in another, and either decision is a correct one."""
        out = []
        for v, n in enumerate(self.g.nodes):
            if v in self.inputs or n.act != ACT_RELU:
                continue
            scale = max(float(np.abs(self.X[i][v]).max()) for i in range(1, self.W + 1))
            for i in range(1, self.W + 1):
                for k in np.flatnonzero(np.abs(self.A[i][v]).ravel() <= tau_rel * scale):
                    out.append((i, v, int(k)))
        return out

    def loss(self, labels, out_node=None):
        """Mean over the frames 1..W of the batch-mean cross-entropy at the output node (App. A2)."""
        out = self.g.out_node if out_node is None else out_node
        return float(np.mean([softmax_cross_entropy(self.X[i][out], labels)[0] for i in range(1, self.W + 1)]))

    def backward(self, labels, out_node=None, flips=()):
        """Gradients of `loss` with respect to every weight and bias (and, as a by-product, to the input
        frames 1..W): returns (dtheta list, dbias list, dinputs {v: (W+1,B,H,W,C)}).
        flips: (frame, node, flat index) triples at which the rectifier's derivative is taken as the
        other one of {0, 1} (see near_kink); the forward values stay as they are."""
        g, X, W = self.g, self.X, self.W
        toggled = {}
        for (fi, fv, fk) in set(flips):
            toggled.setdefault((fi, fv), []).append(fk)
        out = g.out_node if out_node is None else out_node
        dtheta = [np.zeros_like(t) for t in self.theta]
        dbias = [np.zeros_like(b) for b in self.bias]
        # gradient with respect to the state of (frame, node); frame 0 is given, it receives none that is used
        dX = [[np.zeros_like(X[i][v]) for v in range(len(g.nodes))] for i in range(W + 1)]
        for i in range(W, 0, -1):
            dX[i][out] = dX[i][out] + softmax_cross_entropy(X[i][out], labels)[1] / W
            for level in reversed(self.schedule[1:]):
                for v in level:
                    n = g.nodes[v]
                    # x = sigma(a): for the rectifier a > 0 exactly where x > 0
                    if n.act == ACT_RELU:
                        mask = X[i][v] > 0
                        if (i, v) in toggled:
                            mask = mask.copy()
                            flat = mask.reshape(-1)
                            flat[toggled[(i, v)]] = ~flat[toggled[(i, v)]]
                        da = dX[i][v] * mask
                    else:
                        da = dX[i][v]
                    if self.masks is not None and self.masks.get(v) is not None:
                        da = da * np.asarray(self.masks[v][i], dtype=np.float64)      # x = m * sigma(a)
                    dbias[v] += da.sum(axis=(0, 1, 2))
                    for ei in self.src_edges[v]:
                        e = g.edges[ei]
                        dx, dth = edge_backward(e, self.theta[ei], X[i - e.bridge][e.src], da)
                        dtheta[ei] += dth
                        dX[i - e.bridge][e.src] += dx
        dinputs = {v: np.stack([dX[i][v] for i in range(W + 1)]) for v in self.inputs}
        return dtheta, dbias, dinputs


def window_gradients(graph, weights, biases, inputs, labels, W, out_node=None, masks=None):
    """(loss, dtheta, dbias) of one training window from the zero initial state."""
    win = Window(graph, weights, biases)
    win.forward(inputs, W, masks=masks)
    loss = win.loss(labels, out_node)
    dtheta, dbias, _ = win.backward(labels, out_node)
    return loss, dtheta, dbias


# ----------------------------------------------------------------------------
# optimiser
# ----------------------------------------------------------------------------

def rmsprop_step(theta, mean_square, grad, lr, rho=0.9, eps=1e-7):
    """One RMSprop update (the optimiser of App. A2, training details; Tieleman & Hinton 2012):
         a     <- rho * a + (1 - rho) * g^2
         theta <- theta - lr * g / (sqrt(a) + eps)
    with a the running mean of the squared gradient (zero before the first step).  The paper gives the
    initial learning rate (1e-4) and its decay (1e-6 per update: lr_t = lr / (1 + decay * t), the
    caller's business); rho and eps are not stated: the defaults of the authors' framework are taken.
    Returns (theta, a) as new float64 arrays."""
    g = np.asarray(grad, dtype=np.float64)
    a = rho * np.asarray(mean_square, dtype=np.float64) + (1.0 - rho) * g * g
    return np.asarray(theta, dtype=np.float64) - lr * g / (np.sqrt(a) + eps), a
