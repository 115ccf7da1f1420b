"""Pins for the backward oracle: it must agree with what does not depend on it.

* central finite differences of an objective assembled from the forward oracle's (already pinned)
  functions, the routing decisions held at their base values: every coordinate of x and sampled weight
  entries, with and without the ReLU, with dropped tokens, with and without the locality term;
* PyTorch's reverse-mode differentiation of the same forward written with library ops (float64);
* closed forms: GeLU'(0) = 1/2, GeLU' -> 1 / 0 in the tails, its only zero near -0.7518; a single expert
  (E = 1: w = 1, nothing to route) reduces to the gradient of a plain two-layer MLP.
"""
import math

import numpy as np
import pytest
from scipy import special as sp

from oracle import locmoe_backward_oracle as bwd
from oracle import locmoe_oracle as orc


def make_case(seed, T, d, E, N, h, C, relu=True, with_eps=True, exact=False):
    rng = np.random.default_rng(seed)
    if exact:
        # multiples of 1/64 in a power-of-two block: the gating values are exact in float32 and float64 alike
        x = rng.integers(-64, 192, size=(T, d)).astype(np.float64) / 64.0
        eps = rng.integers(-8, 8, size=E).astype(np.float64) / 8.0 if with_eps else None
    else:
        x = rng.standard_normal((T, d)) + 0.6
        eps = rng.uniform(-0.6, 0.4, size=E) if with_eps else None
    home = rng.integers(0, N, size=T).astype(np.int32)
    home[:N] = np.arange(N)                                  # every node has tokens: D_l > 0
    e2n = (np.arange(E) * N // E).astype(np.int32)
    W = {e: (rng.standard_normal((h, d)) * 0.3, rng.standard_normal((d, h)) * 0.3) for e in range(E)}
    dy = rng.standard_normal((T, d))
    return dict(x=x, eps=eps, home=home, e2n=e2n, W=W, dy=dy, T=T, d=d, E=E, N=N, h=h, C=C, relu=relu)


def objective(c, x, W, base, alpha, mu, use_home):
    """dy.y + L_aux + mu KL(P || D_l) from forward-oracle functions, decisions (eid, slots) held fixed."""
    g = orc.gate(x, c["E"])
    s = g if c["eps"] is None else g + c["eps"][None, :]
    G = np.maximum(s, 0.0) if c["relu"] else s
    p = sp.softmax(G, axis=1)
    w = p[np.arange(c["T"]), base["eid"]]
    K = int(base["seg_off"][-1])
    send = orc.dispatch(x, base["slot"], K)
    out = orc.expert_ffn(send, base["seg_off"], base["buf_expert"], lambda e: W[e])
    y = orc.combine(out, base["slot"], w)
    st = orc.route_stats(base["eid"], p, c["home"] if use_home else None, c["e2n"], c["N"], alpha, mu)
    return float(np.sum(c["dy"] * y)) + st["L_aux"] + mu * st["KL_soft"]


def run_oracle(c, alpha, mu, use_home):
    return bwd.moe_layer_backward(c["x"], c["home"] if use_home else None, c["e2n"], c["E"], c["N"], c["C"],
                                  lambda e: c["W"][e], c["dy"], c["eps"], c["relu"], alpha, mu)


@pytest.mark.parametrize("relu,with_eps,use_home,C", [(True, True, True, 2), (False, True, True, 3),
                                                      (True, False, False, 100), (True, True, True, 1)])
def test_finite_differences_of_the_forward_oracle(relu, with_eps, use_home, C):
    alpha, mu = 0.7, 0.9                                     # large enough for the loss terms to matter
    c = make_case(11, T=7, d=8, E=4, N=2, h=5, C=C, relu=relu, with_eps=with_eps)
    r = run_oracle(c, alpha, mu, use_home)
    if C <= 2:
        assert (r["slot"] < 0).any()                         # the small capacities drop tokens
    if relu and with_eps:
        s = r["g32"] + c["eps"].astype(np.float32)[None, :]
        assert (s <= 0).any() and (s > 0).any()              # both sides of the ReLU occur
    hstep = 1e-6
    scale = np.abs(r["dx"]).max()
    for m in range(c["T"]):
        for j in range(c["d"]):
            xp = c["x"].copy(); xp[m, j] += hstep
            xm = c["x"].copy(); xm[m, j] -= hstep
            fd = (objective(c, xp, c["W"], r, alpha, mu, use_home)
                  - objective(c, xm, c["W"], r, alpha, mu, use_home)) / (2 * hstep)
            assert abs(fd - r["dx"][m, j]) <= 2e-6 * scale, (m, j, fd, r["dx"][m, j])
    rng = np.random.default_rng(5)
    for e, (dWi, dWo) in r["grads"].items():
        for which, G in ((0, dWi), (1, dWo)):
            for _ in range(6):
                a, b = rng.integers(0, G.shape[0]), rng.integers(0, G.shape[1])
                Wp = {k: (v[0].copy(), v[1].copy()) for k, v in c["W"].items()}
                Wm = {k: (v[0].copy(), v[1].copy()) for k, v in c["W"].items()}
                Wp[e][which][a, b] += hstep
                Wm[e][which][a, b] -= hstep
                fd = (objective(c, c["x"], Wp, r, alpha, mu, use_home)
                      - objective(c, c["x"], Wm, r, alpha, mu, use_home)) / (2 * hstep)
                assert abs(fd - G[a, b]) <= 2e-6 * max(1.0, np.abs(G).max()), (e, which, a, b)
    # experts without kept rows have no entry (zero gradient): the objective does not move with them
    for e in set(range(c["E"])) - set(r["grads"]):
        Wp = {k: (v[0] + 0.1, v[1] - 0.1) if k == e else v for k, v in c["W"].items()}
        assert objective(c, c["x"], Wp, r, alpha, mu, use_home) == objective(c, c["x"], c["W"], r, alpha, mu, use_home)


@pytest.mark.parametrize("relu,use_home", [(True, True), (False, False)])
def test_against_reverse_mode_differentiation(relu, use_home):
    import torch
    alpha, mu = 0.3, 0.4
    c = make_case(3, T=96, d=32, E=8, N=4, h=12, C=9, relu=relu, exact=True)
    r = run_oracle(c, alpha, mu, use_home)
    assert (r["slot"] < 0).any()
    T, d, E = c["T"], c["d"], c["E"]
    x = torch.tensor(c["x"], dtype=torch.float64, requires_grad=True)
    Wi = {e: torch.tensor(c["W"][e][0], requires_grad=True) for e in range(E)}
    Wo = {e: torch.tensor(c["W"][e][1], requires_grad=True) for e in range(E)}
    g = x.reshape(T, E, d // E).mean(dim=2)
    s = g + torch.tensor(c["eps"])[None, :]
    G = torch.relu(s) if relu else s
    p = torch.softmax(G, dim=1)
    eid = torch.tensor(r["eid"], dtype=torch.int64)
    assert torch.equal(torch.argmax(G, dim=1), eid)
    w = p.gather(1, eid[:, None])[:, 0]
    J = torch.zeros((), dtype=torch.float64)
    dy = torch.tensor(c["dy"])
    for m in range(T):
        if r["slot"][m] >= 0:
            e = int(r["eid"][m])
            J = J + w[m] * torch.dot(dy[m], Wo[e] @ torch.nn.functional.gelu(Wi[e] @ x[m]))
    f = torch.tensor(np.bincount(r["eid"], minlength=E) / T)
    P = p.mean(dim=0)
    J = J + alpha * E * torch.sum(f * P)
    if use_home:
        J = J + mu * torch.sum(P * torch.log(P / torch.tensor(r["stats"]["D_l"])))
    J.backward()
    assert np.allclose(x.grad.numpy(), r["dx"], rtol=1e-9, atol=1e-11 * np.abs(r["dx"]).max())
    for e in range(E):
        if e in r["grads"]:
            assert np.allclose(Wi[e].grad.numpy(), r["grads"][e][0], rtol=1e-9, atol=1e-12)
            assert np.allclose(Wo[e].grad.numpy(), r["grads"][e][1], rtol=1e-9, atol=1e-12)
        else:
            assert Wi[e].grad is None or not Wi[e].grad.any()


def test_gelu_grad_closed_forms():
    assert bwd.gelu_grad(np.array([0.0]))[0] == 0.5
    assert abs(bwd.gelu_grad(np.array([9.0]))[0] - 1.0) < 1e-15
    assert abs(bwd.gelu_grad(np.array([-9.0]))[0]) < 1e-15
    # the derivative vanishes where Phi(v) = -v phi(v): the minimum of GeLU, near -0.75179
    assert bwd.gelu_grad(np.array([-0.7520]))[0] < 0.0 < bwd.gelu_grad(np.array([-0.7516]))[0]
    v = np.linspace(-6, 6, 241)
    hstep = 1e-6
    fd = (orc.gelu(v + hstep) - orc.gelu(v - hstep)) / (2 * hstep)
    assert np.max(np.abs(fd - bwd.gelu_grad(v))) < 1e-9
    # GeLU'(v) + GeLU'(-v) = 1 (Phi(v) + Phi(-v) = 1, v phi(v) odd)
    assert np.max(np.abs(bwd.gelu_grad(v) + bwd.gelu_grad(-v) - 1.0)) < 1e-15


def test_single_expert_is_a_plain_mlp():
    c = make_case(8, T=9, d=6, E=1, N=1, h=4, C=100, with_eps=False)
    r = run_oracle(c, 0.0, 0.0, False)
    Wi, Wo = c["W"][0]
    Z = c["x"] @ Wi.T
    Phi = 0.5 * (1 + sp.erf(Z / math.sqrt(2)))
    dH = c["dy"] @ Wo
    dZ = dH * (Phi + Z * np.exp(-Z * Z / 2) / math.sqrt(2 * math.pi))
    assert np.all(r["w"] == 1.0)
    # softmax over one expert is constant: no gradient reaches the gate
    assert not r["dg"].any()
    assert np.allclose(r["dx"], dZ @ Wi, rtol=1e-12, atol=1e-14)
    assert np.allclose(r["grads"][0][0], dZ.T @ c["x"], rtol=1e-12, atol=1e-14)
    assert np.allclose(r["grads"][0][1], c["dy"].T @ (Z * Phi), rtol=1e-12, atol=1e-14)


def test_steps_are_adjoints_of_the_forward_steps():
    """<forward(u), v> = <u, backward(v)> for the linear steps (gate, dispatch) on random vectors."""
    rng = np.random.default_rng(2)
    T, d, E = 13, 24, 6
    u = rng.standard_normal((T, d)); v = rng.standard_normal((T, E))
    assert abs(np.sum(orc.gate(u, E) * v) - np.sum(u * bwd.gate_backward(v, d))) < 1e-12
    slot = np.array([2, -1, 0, 3, -1, 1, 4, -1, -1, 5, -1, -1, 6], np.int32)
    vs = rng.standard_normal((7, d))
    assert abs(np.sum(orc.dispatch(u, slot, 7) * vs) - np.sum(u * bwd.dispatch_backward(vs, slot))) < 1e-12
