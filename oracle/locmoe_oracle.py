"""CPU oracle for the LocMoE MoE-layer forward path (arXiv 2401.13920).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct NumPy
implementation written from the paper.  Only the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it; the product path (the HIP library
and its Python binding) never does, and this file imports nothing from it.

Every function is a plain definition, in float64 unless stated:

* gating value          Section 3.2.1, Eq. 4 (GrAP weight) and the text after Eq. 3
* top-1 / expert score  Eq. 2, Eq. 3
* auxiliary loss        Eq. 5
* locality loss         Eq. 6
* capacity              Section 3.2.3: empirical capacity, Lemma 3, Theorem 1
* expert FFN / combine  Eq. 1
* token-to-gate angles  Section 3.2.3 (the assumption that defines delta_{i,j}), Section 4.1
* comparison routers    Section 3.2.1 (the dense layer that GrAP replaces, the switch router's gate), Section 2 and
                        Section 4 (hash routing without learnable parameters)

Readings where the paper is silent are spelled out at each function.  Every
function here is pinned by the CPU tests against closed forms, brute force or
values the paper prints; none is "parity unpinned".
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np
from scipy import special as _sp

# --------------------------------------------------------------------------
# Capacity: Lemma 3 and Theorem 1
# --------------------------------------------------------------------------

def p_delta(d: int, delta: float) -> float:
    """Lemma 3: probability that a uniformly distributed unit vector in R^d has
    |cos| >= delta to a fixed direction:  1 - I_{delta^2}(1/2, (d-1)/2)."""
    return 1.0 - float(_sp.betainc(0.5, 0.5 * (d - 1), delta * delta))


def ec_min(E: int, d: int, delta: float, form: str = "erfc") -> float:
    """Theorem 1, the three right-hand sides of the capacity lower bound (in tokens):
    'exact' 1/(n p_delta);  'erfc' 1/(n erfc(sqrt(y)));  'exp' exp(y)/n,
    with y = delta^2 d / (2 - delta^2)."""
    y = delta * delta * d / (2.0 - delta * delta)
    if form == "exact":
        p = p_delta(d, delta)
        return math.inf if p <= 0.0 else 1.0 / (E * p)
    if form == "erfc":
        c = math.erfc(math.sqrt(y))
        return math.inf if c <= 0.0 else 1.0 / (E * c)
    if form == "exp":
        return math.exp(y) / E if y < 700.0 else math.inf
    raise ValueError(form)


def capacity(T: int, E: int, d: int, cf: float, delta: float) -> int:
    """Rows per expert.  The empirical capacity ceil(b_s c_f / (ep n)) of Section 3.2.3
    becomes ceil(c_f T / E) on one device's share of T tokens; it is floored by the
    Theorem 1 bound (erfc form, the one both sides evaluate with libm) and clamped to
    [1, T].  c_f = 0 selects the bound alone.  The ceiling is the plain one of the printed formula, taken of
    the exact rational value with c_f read as the decimal number it is written as (1.1 is 11/10)."""
    emp = math.ceil(Fraction(repr(float(cf))) * T / E) if cf > 0.0 else 0
    b = ec_min(E, d, delta, "erfc")
    bound = T if math.isinf(b) or b >= T else math.ceil(b)
    return int(min(max(emp, bound, 1), T))


# --------------------------------------------------------------------------
# GrAP gate
# --------------------------------------------------------------------------

def grap_weight(E: int, d: int) -> np.ndarray:
    """Eq. 4: omega[i, j] = n/d for j in block i (i d/n <= j < (i+1) d/n), else 0."""
    if d % E:
        raise ValueError("d must be a multiple of the number of experts")
    W = np.zeros((E, d), dtype=np.float64)
    blk = d // E
    for i in range(E):
        W[i, i * blk:(i + 1) * blk] = E / d
    return W


def gate(x: np.ndarray, E: int) -> np.ndarray:
    """Raw gating value omega_i . x_m = mean of the i-th contiguous block of d/n features
    (grouped average pooling).  float64 [T, E]."""
    T, d = x.shape
    if d % E:
        raise ValueError("d must be a multiple of the number of experts")
    return np.asarray(x, dtype=np.float64).reshape(T, E, d // E).mean(axis=2)


def gate_dense(x: np.ndarray, E: int) -> np.ndarray:
    """The same value as the dense layer it stands for: x @ omega^T."""
    return np.asarray(x, dtype=np.float64) @ grap_weight(E, x.shape[1]).T


# --------------------------------------------------------------------------
# Route: Eq. 2, Eq. 3
# --------------------------------------------------------------------------

def route(g32: np.ndarray, eps: np.ndarray | None = None, relu: bool = True):
    """G = ReLU(g + eps) evaluated in float32 (the precision the decision is taken in on
    both sides); e* = lowest index attaining max_i G (softmax is monotone, so this is
    Eq. 2's argmax); p = softmax(G) in float64; w = p[e*] (Eq. 3).
    Returns eid int32 [T], w float64 [T], p float64 [T,E], G float32 [T,E]."""
    g32 = np.asarray(g32, dtype=np.float32)
    G = g32 if eps is None else (g32 + np.asarray(eps, dtype=np.float32)[None, :]).astype(np.float32)
    if relu:
        G = np.maximum(G, np.float32(0.0))
    eid = np.argmax(G, axis=1).astype(np.int32)          # first occurrence of the max
    G64 = G.astype(np.float64)
    z = np.exp(G64 - G64.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    w = p[np.arange(G.shape[0]), eid]
    return eid, w, p, G


def route_stats(eid, p, home, e2n, N, alpha=0.01, mu=0.01):
    """Eq. 5 and Eq. 6 (forward values).
    f_i = fraction of tokens whose argmax is i (before any capacity drop),
    P_i = mean router probability, L_aux = alpha n sum f_i P_i.
    Locality: D_l is the fully localized distribution - every token spread evenly over
    the experts placed on its home node; D_c is the current assignment distribution f
    (KL_hard) or its differentiable stand-in P (KL_soft); L_loc = mu KL(D_c || D_l),
    with 0 ln 0 = 0.  Returns a dict."""
    T, E = p.shape
    cnt = np.bincount(eid, minlength=E).astype(np.int64)
    Psum = p.sum(axis=0)
    f = cnt / T
    P = Psum / T
    out = {"cnt": cnt, "Psum": Psum, "L_aux": alpha * E * float(np.dot(f, P))}
    if home is None:
        out.update(KL_hard=0.0, KL_soft=0.0, L_loc=0.0, locality_frac=0.0)
        return out
    e2n = np.asarray(e2n)
    Tnode = np.bincount(home, minlength=N).astype(np.float64)
    per_node = np.bincount(e2n, minlength=N).astype(np.float64)   # experts on each node
    Dl = Tnode[e2n] / (T * per_node[e2n])

    def kl(Dc):
        s = 0.0
        for i in range(E):
            if Dc[i] > 0.0:
                if Dl[i] <= 0.0:
                    return math.inf
                s += Dc[i] * math.log(Dc[i] / Dl[i])
        return s

    out["KL_hard"] = kl(f)
    out["KL_soft"] = kl(P)
    out["L_loc"] = mu * out["KL_hard"]
    out["locality_frac"] = float(np.mean(e2n[eid] == home))
    out["D_l"] = Dl
    return out


# --------------------------------------------------------------------------
# Slot assignment + dispatch layout
# --------------------------------------------------------------------------

def buffer_order(e2n: np.ndarray) -> np.ndarray:
    """Experts in send-buffer order: by destination node, then by expert id."""
    E = len(e2n)
    return np.array(sorted(range(E), key=lambda e: (int(e2n[e]), e)), dtype=np.int32)


def slots(eid: np.ndarray, E: int, C: int, e2n: np.ndarray, N: int):
    """First-come-first-kept by token index (the GShard convention the capacity paragraph
    of Section 3.2.3 builds on): pos[m] = number of earlier tokens with the same expert;
    token kept iff pos < C.  Kept rows are packed expert by expert in buffer order
    (node-major), each expert's rows in token order.
    Returns dict(pos, slot, kept, seg_off, node_off, row_token, buf_expert, cnt)."""
    T = len(eid)
    pos = np.empty(T, dtype=np.int32)
    counter = [0] * E
    for m in range(T):
        e = int(eid[m])
        pos[m] = counter[e]
        counter[e] += 1
    cnt = np.array(counter, dtype=np.int32)
    kept = np.minimum(cnt, C).astype(np.int32)
    order = buffer_order(e2n)
    seg_off = np.zeros(E + 1, dtype=np.int32)
    rank_of = np.empty(E, dtype=np.int32)
    for r, e in enumerate(order):
        rank_of[e] = r
        seg_off[r + 1] = seg_off[r] + kept[e]
    node_off = np.zeros(N + 1, dtype=np.int32)
    for nu in range(N):
        node_off[nu + 1] = node_off[nu] + sum(int(kept[e]) for e in range(E) if e2n[e] == nu)
    K = int(seg_off[E])
    slot = np.full(T, -1, dtype=np.int32)
    row_token = np.full(K, -1, dtype=np.int32)
    for m in range(T):
        if pos[m] < C:
            s = int(seg_off[rank_of[eid[m]]]) + int(pos[m])
            slot[m] = s
            row_token[s] = m
    return dict(pos=pos, slot=slot, kept=kept, seg_off=seg_off, node_off=node_off,
                row_token=row_token, buf_expert=order, cnt=cnt)


def pos_bruteforce(eid: np.ndarray) -> np.ndarray:
    """pos[m] = #{m' < m : eid[m'] = eid[m]} by the definition, O(T^2)."""
    T = len(eid)
    return np.array([sum(1 for q in range(m) if eid[q] == eid[m]) for m in range(T)], dtype=np.int32)


def dispatch(x: np.ndarray, slot: np.ndarray, K: int) -> np.ndarray:
    """send[slot[m]] = x[m] for kept tokens (exact copy)."""
    send = np.zeros((K, x.shape[1]), dtype=x.dtype)
    for m in range(len(slot)):
        if slot[m] >= 0:
            send[slot[m]] = x[m]
    return send


# --------------------------------------------------------------------------
# Expert FFN and combine: Eq. 1
# --------------------------------------------------------------------------

def gelu(v: np.ndarray) -> np.ndarray:
    """GeLU as the paper words it: input times the standard Gaussian CDF."""
    v = np.asarray(v, dtype=np.float64)
    return v * 0.5 * (1.0 + _sp.erf(v / math.sqrt(2.0)))


def ffn_rows(S: np.ndarray, W_in: np.ndarray, W_out: np.ndarray) -> np.ndarray:
    """One expert on its rows: W_out . GeLU(W_in . x) with Eq. 1's orientation, W_in [h,d]
    and W_out [d,h]; the rows of S are the x vectors.  No biases, no intermediate rounding."""
    H = gelu(np.asarray(S, dtype=np.float64) @ np.asarray(W_in, dtype=np.float64).T)
    return H @ np.asarray(W_out, dtype=np.float64).T


def ffn_rows_loops(S, W_in, W_out) -> np.ndarray:
    """Triple-loop twin of :func:`ffn_rows` for tiny shapes."""
    R, d = S.shape
    h = W_in.shape[0]
    O = np.zeros((R, W_out.shape[0]), dtype=np.float64)
    for r in range(R):
        hid = [0.0] * h
        for j in range(h):
            a = 0.0
            for k in range(d):
                a += float(W_in[j, k]) * float(S[r, k])
            hid[j] = a * 0.5 * (1.0 + math.erf(a / math.sqrt(2.0)))
        for c in range(W_out.shape[0]):
            a = 0.0
            for j in range(h):
                a += float(W_out[c, j]) * hid[j]
            O[r, c] = a
    return O


def expert_ffn(send: np.ndarray, seg_off: np.ndarray, buf_expert: np.ndarray, weights) -> np.ndarray:
    """out[K,d]; ``weights(e)`` returns (W_in[e], W_out[e]) so that large configs can
    stream one expert at a time."""
    K = int(seg_off[-1])
    out = np.zeros((K, send.shape[1]), dtype=np.float64)
    for r, e in enumerate(buf_expert):
        a, b = int(seg_off[r]), int(seg_off[r + 1])
        if b > a:
            W_in, W_out = weights(int(e))
            out[a:b] = ffn_rows(send[a:b], W_in, W_out)
    return out


def combine(out: np.ndarray, slot: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Eq. 1 under top-1: y_m = R_{m,i*} . expert_{i*}(x_m); a dropped token gets zeros."""
    T = len(slot)
    y = np.zeros((T, out.shape[1]), dtype=np.float64)
    for m in range(T):
        if slot[m] >= 0:
            y[m] = w[m] * out[slot[m]]
    return y


def moe_layer(x, home, e2n, E, N, C, weights, eps=None, relu=True, alpha=0.01, mu=0.01):
    """The whole forward path in the paper's order; returns every intermediate."""
    g = gate(x, E)
    g32 = g.astype(np.float32)
    eid, w, p, _ = route(g32, eps, relu)
    stats = route_stats(eid, p, home, e2n, N, alpha, mu)
    sl = slots(eid, E, C, e2n, N)
    K = int(sl["seg_off"][-1])
    send = dispatch(x, sl["slot"], K)
    out = expert_ffn(send, sl["seg_off"], sl["buf_expert"], weights)
    y = combine(out, sl["slot"], w)
    return dict(g=g, g32=g32, eid=eid, w=w, p=p, stats=stats, send=send, out=out, y=y, **sl)


# --------------------------------------------------------------------------
# Angles between tokens and gating weights (Section 3.2.3, Section 4.1)
# --------------------------------------------------------------------------
def token_gate_cosines(x: np.ndarray, E: int) -> np.ndarray:
    """delta_{i,j} of Section 3.2.3: the cosine of the angle between token j and gating weight
    omega_i (Eq. 4), as the plain normalised dot product, for every token and expert: [T, E].
    A zero token has no angle; its cosines are set to 0."""
    x = np.asarray(x, dtype=np.float64)
    W = grap_weight(E, x.shape[1])
    dots = x @ W.T
    nx = np.sqrt(np.sum(x * x, axis=1))
    nw = np.sqrt(np.sum(W * W, axis=1))
    safe = np.where(nx > 0.0, nx, 1.0)
    return np.where(nx[:, None] > 0.0, dots / (safe[:, None] * nw[None, :]), 0.0)


def angle_stats(x: np.ndarray, eid: np.ndarray, E: int, shift: int, nbins: int):
    """The measurement behind Section 4.1 ("Analysis for Expert Capacity"): for the tokens routed to
    each expert i, the histogram of their cosine to omega_i and of their cosine to another expert
    (expert (i + shift) mod E here), and the smallest cosine to omega_i among them.  The paper reads
    its delta off such histograms; delta_hat below is the literal reading of the assumption in
    Section 3.2.3 (every routed token satisfies delta_{i,j} >= delta): the smallest routed cosine.

    Bins split [-1, 1] evenly; bin b = floor((c + 1) / 2 * nbins), clamped to [0, nbins - 1].
    Returns c_self [T], c_other [T], hist_self [E, nbins], hist_other [E, nbins], cmin [E] (2.0 for an
    expert without tokens: no cosine reaches it) and delta_hat (2.0 when there are no tokens)."""
    cos = token_gate_cosines(x, E)
    eid = np.asarray(eid, dtype=np.int64)
    T = cos.shape[0]
    rows = np.arange(T)
    c_self = cos[rows, eid]
    c_other = cos[rows, (eid + shift) % E]

    def bins(c):
        return np.clip(np.floor((c + 1.0) * 0.5 * nbins).astype(np.int64), 0, nbins - 1)

    hist_self = np.zeros((E, nbins), dtype=np.int64)
    hist_other = np.zeros((E, nbins), dtype=np.int64)
    np.add.at(hist_self, (eid, bins(c_self)), 1)
    np.add.at(hist_other, (eid, bins(c_other)), 1)
    cmin = np.full(E, 2.0)
    np.minimum.at(cmin, eid, c_self)
    delta_hat = float(cmin.min()) if T > 0 else 2.0
    return c_self, c_other, hist_self, hist_other, cmin, delta_hat



# --------------------------------------------------------------------------
# Comparison routers (Section 2, Section 3.2.1, Section 4)
# --------------------------------------------------------------------------

def gate_dense_learned(x: np.ndarray, Wg: np.ndarray) -> np.ndarray:
    """The gate as the dense layer Section 3.2.1 says it usually is, with a learned weight omega [n, d]:
    g[m, i] = omega_i . x_m (raw value, like :func:`gate`; bias and ReLU belong to :func:`route`).  This is the
    gate of the switch router the paper compares with; GrAP is the special case omega = Eq. 4's weight."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(Wg, dtype=np.float64).T


def mix32(v: np.ndarray) -> np.ndarray:
    """The 32-bit finalizer of MurmurHash3 (a published, public-domain integer mixer; a bijection of the 32-bit
    integers): xor-shift 16, times 0x85EBCA6B, xor-shift 13, times 0xC2B2AE35, xor-shift 16, all modulo 2^32."""
    v = np.asarray(v, dtype=np.uint64) & np.uint64(0xFFFFFFFF)
    v ^= v >> np.uint64(16)
    v = (v * np.uint64(0x85EBCA6B)) & np.uint64(0xFFFFFFFF)
    v ^= v >> np.uint64(13)
    v = (v * np.uint64(0xC2B2AE35)) & np.uint64(0xFFFFFFFF)
    v ^= v >> np.uint64(16)
    return v.astype(np.uint32)


def route_hash(keys: np.ndarray, E: int, seed: int = 0):
    """Hash routing as Section 2 and Section 4 describe the hash router: the expert is a fixed, parameter-free,
    (near-)uniform function of the token's key (its vocabulary id, or its position when no ids are given), and no
    feature of the token is computed.  Reading (the paper names no hash function): expert = mix32(key + seed *
    0x9E3779B9 mod 2^32) mod n.  There is no gating score, so the expert's output enters Eq. 1 with weight 1.
    Returns eid int32 [T], w float64 [T] (ones), cnt int64 [n]."""
    k = (np.asarray(keys, dtype=np.int64) + ((int(seed) * 0x9E3779B9) & 0xFFFFFFFF)) & 0xFFFFFFFF
    eid = (mix32(k).astype(np.uint64) % np.uint64(E)).astype(np.int32)
    return eid, np.ones(len(eid), dtype=np.float64), np.bincount(eid, minlength=E)
