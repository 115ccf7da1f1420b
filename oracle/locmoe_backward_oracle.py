"""CPU oracle for the backward pass of the LocMoE MoE-layer path (arXiv 2401.13920).

TEST INFRASTRUCTURE ONLY: only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg
may import this file; the product path never does, and this file imports nothing from it.

What is differentiated is the training objective of Section 3.2.2 (the equation after Eq. 6):
    L_task = L_cross + L_aux + L_loc,
as far as it depends on this layer: L_cross reaches the layer through dy = dL_cross/dy (an input
here), L_aux is Eq. 5 and L_loc is Eq. 6.  Everything is the chain rule applied to the forward
definitions (Eq. 1-6), in float64, one function per forward step, in reverse order.

Readings where the paper is silent:
* The routing decision (Eq. 2's argmax), the capacity drop and f_i of Eq. 5 are piecewise constant in x:
  they carry no gradient (the usual treatment of Eq. 5 in the work the paper cites for it).
* Eq. 6's current distribution D_c is differentiated through its smooth stand-in P (the mean router
  probability), i.e. the gradient is that of mu * KL(P || D_l); with D_c = f the gradient is zero
  almost everywhere and the loss could not act on the router at all.
* ReLU'(0) = 0.
* The GrAP weight of Eq. 4 is fixed by construction: the gate has no trainable parameter, so the
  gradients are dx, dW_in and dW_out.
* If some D_l[i] = 0 the forward KL is infinite and the gradient is not finite.

Every function is pinned in tests/test_backward_oracle_pins.py by central finite differences of the
(already pinned) forward oracle and by PyTorch's reverse-mode differentiation of the same forward written
with library ops; none is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

from oracle import locmoe_oracle as fwd


def gelu_grad(v: np.ndarray) -> np.ndarray:
    """d/dv [v Phi(v)] = Phi(v) + v phi(v), Phi/phi the standard normal CDF/density (Eq. 1's GeLU)."""
    v = np.asarray(v, dtype=np.float64)
    Phi = 0.5 * (1.0 + fwd._sp.erf(v / math.sqrt(2.0)))
    phi = np.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)
    return Phi + v * phi


def combine_backward(dy: np.ndarray, out: np.ndarray, slot: np.ndarray, w: np.ndarray):
    """y_m = w_m out[slot_m] (Eq. 1 under top-1): dout[slot_m] = w_m dy_m and dw_m = <dy_m, out[slot_m]>
    for a kept token; a dropped token contributes nothing (dw_m = 0).  Returns dout [K,d], dw [T]."""
    dy = np.asarray(dy, dtype=np.float64)
    dout = np.zeros_like(np.asarray(out, dtype=np.float64))
    dw = np.zeros(len(slot), dtype=np.float64)
    for m in range(len(slot)):
        s = int(slot[m])
        if s >= 0:
            dout[s] = w[m] * dy[m]
            dw[m] = float(np.dot(dy[m], out[s]))
    return dout, dw


def ffn_rows_backward(S, W_in, W_out, dO):
    """One expert on its rows, O = GeLU(S W_in^T) W_out^T (Eq. 1's orientation):
    dH = dO W_out, dZ = dH * GeLU'(Z), dS = dZ W_in, dW_out = dO^T H, dW_in = dZ^T S.
    Returns dS, dW_in, dW_out, Z, dZ."""
    S = np.asarray(S, dtype=np.float64)
    W_in = np.asarray(W_in, dtype=np.float64)
    W_out = np.asarray(W_out, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    Z = S @ W_in.T
    H = fwd.gelu(Z)
    dH = dO @ W_out
    dZ = dH * gelu_grad(Z)
    return dZ @ W_in, dZ.T @ S, dO.T @ H, Z, dZ


def expert_ffn_backward(send, dout, seg_off, buf_expert, weights):
    """Segment by segment; returns dsend [K,d] and {expert: (dW_in, dW_out)} for experts with rows
    (an expert without rows has zero weight gradients)."""
    K = int(seg_off[-1])
    dsend = np.zeros((K, send.shape[1]), dtype=np.float64)
    grads = {}
    for r, e in enumerate(buf_expert):
        a, b = int(seg_off[r]), int(seg_off[r + 1])
        if b > a:
            W_in, W_out = weights(int(e))
            dS, dWi, dWo, _, _ = ffn_rows_backward(send[a:b], W_in, W_out, dout[a:b])
            dsend[a:b] = dS
            grads[int(e)] = (dWi, dWo)
    return dsend, grads


def loss_coefficients(cnt, Psum, T, home, e2n, N, alpha, mu):
    """dL/dp[m,i] from the two batch losses, the same for every token m:
    Eq. 5 with f fixed: alpha n f_i / T;  Eq. 6 through P: mu (ln(P_i / D_l[i]) + 1) / T."""
    E = len(cnt)
    f = np.asarray(cnt, dtype=np.float64) / T
    coef = alpha * E * f / T
    if home is not None and mu != 0.0:
        P = np.asarray(Psum, dtype=np.float64) / T
        e2n = np.asarray(e2n)
        Tnode = np.bincount(home, minlength=N).astype(np.float64)
        per_node = np.bincount(e2n, minlength=N).astype(np.float64)
        Dl = Tnode[e2n] / (T * per_node[e2n])
        with np.errstate(divide="ignore"):
            coef = coef + mu * (np.log(P / Dl) + 1.0) / T
    return coef


def route_backward(g32, eps, relu, eid, dw, coef):
    """Through Eq. 3 and the ReLU below it: with s = g + eps, G = ReLU(s), p = softmax(G), w_m = p[m, e*_m]:
    dp[m,i] = [i = e*_m] dw_m + coef_i;  dG = p * (dp - <p, dp>);  dg = dG where s > 0 (or everywhere
    without the ReLU).  s, G are the float32 values the forward decided on; p is float64 from them.
    Returns dg [T,E]."""
    _, _, p, _ = fwd.route(g32, eps, relu)
    g32 = np.asarray(g32, dtype=np.float32)
    s = g32 if eps is None else (g32 + np.asarray(eps, dtype=np.float32)[None, :]).astype(np.float32)
    T, E = p.shape
    dp = np.tile(np.asarray(coef, dtype=np.float64)[None, :], (T, 1))
    dp[np.arange(T), eid] += np.asarray(dw, dtype=np.float64)
    inner = np.sum(p * dp, axis=1, keepdims=True)
    dG = p * (dp - inner)
    if relu:
        dG = np.where(s > np.float32(0.0), dG, 0.0)
    return dG


def gate_backward(dg: np.ndarray, d: int) -> np.ndarray:
    """Eq. 4: g[m,i] is the mean of block i, so every feature of block i receives dg[m,i] * E/d."""
    T, E = dg.shape
    blk = d // E
    return np.repeat(np.asarray(dg, dtype=np.float64), blk, axis=1) * (E / d)


def dispatch_backward(dsend: np.ndarray, slot: np.ndarray) -> np.ndarray:
    """send[slot_m] = x_m: the gradient row goes back to its token; a dropped token gets zeros."""
    T = len(slot)
    dx = np.zeros((T, dsend.shape[1]), dtype=np.float64)
    for m in range(T):
        if slot[m] >= 0:
            dx[m] = dsend[slot[m]]
    return dx


def moe_layer_backward(x, home, e2n, E, N, C, weights, dy, eps=None, relu=True, alpha=0.01, mu=0.01):
    """Forward (the forward oracle, every intermediate), then the steps above in reverse order.
    Returns the forward dict extended by dout, dw, dsend, dg, dx and grads {expert: (dW_in, dW_out)}."""
    f = fwd.moe_layer(x, home, e2n, E, N, C, weights, eps, relu, alpha, mu)
    T, d = np.asarray(x).shape
    dout, dw = combine_backward(dy, f["out"], f["slot"], f["w"])
    dsend, grads = expert_ffn_backward(f["send"], dout, f["seg_off"], f["buf_expert"], weights)
    coef = loss_coefficients(f["stats"]["cnt"], f["stats"]["Psum"], T, home, e2n, N, alpha, mu)
    dg = route_backward(f["g32"], eps, relu, f["eid"], dw, coef)
    dx = dispatch_backward(dsend, f["slot"]) + gate_backward(dg, d)
    f.update(dout=dout, dw=dw, dsend=dsend, coef=coef, dg=dg, dx=dx, grads=grads)
    return f
