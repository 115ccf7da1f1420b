"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars:
  * routing assignments, positions, slots, kept/segment/node offsets, row_token, dropped set and
    the send buffer rows: bit-exact, given the oracle's float32 gating values;
  * gating values: relative L2 <= 1e-5 and |diff| <= 1e-5 * (E/d) * sum_j |x_j| per element;
  * scores w, Psum and the loss scalars: 1e-5 relative;
  * FFN output and y: relative L2 <= 1e-2 against the float64 oracle (which rounds nothing; the
    budget covers bf16 rounding of H, out and y);
  * cosines between tokens and gating weights, and their per-expert minimum: |diff| <= 1e-5; histogram
    rows: totals exact, and every cumulative count between the oracle's for cosines moved by -1e-5 and
    by +1e-5 (equal to the oracle's histogram wherever no cosine lies that close to a bin edge).
"""
import sys
import time

import numpy as np
import pytest

from oracle import locmoe_oracle as orc
from paper_2401_13920_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2401_13920_amd import harness, locmoe as lm
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lm.lib()
    return torch, lm, harness


def rel_l2(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


def i32(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def check_gate(env, c, x, x_dev, desc, g_dev):
    torch, lm, hz = env
    lm.locmoe_gate(desc, x_dev, g_dev)
    torch.cuda.synchronize()
    g = g_dev.cpu().numpy()
    ref = orc.gate(x, c.E)
    assert rel_l2(g, ref) <= 1e-5
    blk = c.d // c.E
    bound = 1e-5 * np.abs(x.astype(np.float64)).reshape(len(x), c.E, blk).sum(axis=2) / blk
    assert np.all(np.abs(g - ref) <= bound + 1e-30)
    return ref.astype(np.float32)


def check_route(env, c, desc, b, g32, eps, home, e2n, relu, alpha, mu):
    torch, lm, hz = env
    g_dev = torch.from_numpy(g32).cuda()
    eps_dev = None if eps is None else torch.from_numpy(eps.astype(np.float32)).cuda()
    home_dev = None if home is None else i32(torch, home)
    e2n_dev = None if e2n is None else i32(torch, e2n)
    lm.locmoe_route(desc, g_dev, eps_dev, home_dev, e2n_dev, b.eid, b.w, b.cnt, b.Psum, b.stats, b.ws, b.ws_bytes)
    torch.cuda.synchronize()
    eid, w, p, _ = orc.route(g32, eps, relu)
    e2n_full = e2n if e2n is not None else np.arange(c.E) // (c.E // c.N)
    st = orc.route_stats(eid, p, home, e2n_full, c.N, alpha, mu)
    assert np.array_equal(b.eid.cpu().numpy(), eid)                      # bit-exact assignments
    assert np.allclose(b.w.cpu().numpy(), w, rtol=1e-5, atol=0)
    assert np.array_equal(b.cnt.cpu().numpy(), st["cnt"])
    assert np.allclose(b.Psum.cpu().numpy(), st["Psum"], rtol=1e-5, atol=1e-7)
    s = b.stats.cpu().numpy()
    for k, name in enumerate(["L_aux", "KL_hard", "KL_soft", "L_loc", "locality_frac"]):
        assert s[k] == pytest.approx(st[name], rel=1e-5, abs=2e-7), name
    assert s[5] == st["cnt"].max() and s[6] == int((st["cnt"] == 0).sum())
    return eid, w


def check_dispatch(env, c, desc, b, x, x_dev, eid, e2n, C):
    torch, lm, hz = env
    e2n_dev = None if e2n is None else i32(torch, e2n)
    e2n_full = e2n if e2n is not None else np.arange(c.E) // (c.E // c.N)
    b.send.zero_()
    lm.locmoe_dispatch(desc, x_dev, i32(torch, eid), e2n_dev, b.pos, b.slot, b.kept, b.seg_off, b.node_off,
                       b.buf_expert, b.row_token, b.send, b.ws, b.ws_bytes)
    torch.cuda.synchronize()
    s = orc.slots(eid, c.E, C, np.asarray(e2n_full), c.N)
    K = int(s["seg_off"][-1])
    for name in ("pos", "slot", "kept", "seg_off", "node_off", "buf_expert"):
        assert np.array_equal(getattr(b, name).cpu().numpy(), s[name]), name
    assert np.array_equal(b.row_token.cpu().numpy()[:K], s["row_token"])
    send = hz.to_host_f32(b.send[:K])
    assert np.array_equal(send, x[s["row_token"]])                          # bit copies of the rows
    return s, K


COS_TOL = 1e-5


def check_angles(env, c, x, x_dev, desc, eid, shift, nbins, want_cos=True):
    """locmoe_gate_sq + locmoe_angle_stats against the oracle's cosines, histograms and minima."""
    torch, lm, hz = env
    T, E = len(x), c.E
    g_dev = torch.empty(T, E, dtype=torch.float32, device="cuda")
    g2_dev = torch.empty_like(g_dev)
    q_dev = torch.empty_like(g_dev)
    lm.locmoe_gate(desc, x_dev, g_dev)
    lm.locmoe_gate_sq(desc, x_dev, g2_dev, q_dev)
    torch.cuda.synchronize()
    assert torch.equal(g_dev, g2_dev)                       # the same gating arithmetic with or without q
    blk = c.d // E
    q_def = (x.astype(np.float64).reshape(T, E, blk) ** 2).sum(axis=2)
    assert np.all(np.abs(q_dev.cpu().numpy() - q_def) <= 1e-5 * q_def + 1e-37)
    cs_dev = torch.full((T,), 7.0, dtype=torch.float32, device="cuda") if want_cos else None
    co_dev = torch.full((T,), 7.0, dtype=torch.float32, device="cuda") if want_cos else None
    hs_dev = torch.full((E, nbins), -3, dtype=torch.int32, device="cuda")
    ho_dev = torch.full((E, nbins), -3, dtype=torch.int32, device="cuda")
    cmin_dev = torch.full((E,), -9.0, dtype=torch.float32, device="cuda")
    st_dev = torch.full((4,), -9.0, dtype=torch.float32, device="cuda")
    lm.locmoe_angle_stats(desc, g_dev, q_dev, i32(torch, eid), shift, nbins, cs_dev, co_dev, hs_dev, ho_dev,
                          cmin_dev, st_dev)
    torch.cuda.synchronize()
    c_self, c_other, hist_self, hist_other, cmin, delta_hat = orc.angle_stats(x, eid, E, shift, nbins)
    if want_cos:
        assert np.all(np.abs(cs_dev.cpu().numpy() - c_self) <= COS_TOL)
        assert np.all(np.abs(co_dev.cpu().numpy() - c_other) <= COS_TOL)

    def cumulative(cv):
        b = np.clip(np.floor((cv + 1.0) / 2.0 * nbins), 0, nbins - 1).astype(np.int64)
        h = np.zeros((E, nbins), np.int64)
        np.add.at(h, (np.asarray(eid, np.int64), b), 1)
        return np.cumsum(h, axis=1)

    for got_dev, ref_hist, cv in ((hs_dev, hist_self, c_self), (ho_dev, hist_other, c_other)):
        got = got_dev.cpu().numpy().astype(np.int64)
        assert got.min() >= 0
        assert np.array_equal(got.sum(axis=1), np.bincount(eid, minlength=E))
        cum = np.cumsum(got, axis=1)
        # a cosine moved up by the tolerance lands in the same or a higher bin: fewer tokens at or below b
        assert np.all(cumulative(cv + COS_TOL) <= cum) and np.all(cum <= cumulative(cv - COS_TOL))
        scaled = (cv + 1.0) / 2.0 * nbins
        if np.all(np.abs(scaled - np.round(scaled)) > COS_TOL * nbins):
            assert np.array_equal(got, ref_hist)
    got_min = cmin_dev.cpu().numpy()
    empty = np.bincount(eid, minlength=E) == 0
    assert np.all(got_min[empty] == 2.0) and np.all(cmin[empty] == 2.0)
    assert np.all(np.abs(got_min[~empty] - cmin[~empty]) <= COS_TOL)
    st = st_dev.cpu().numpy()
    assert abs(st[0] - delta_hat) <= COS_TOL and st[1] == int((~empty).sum()) and st[2] == 0 and st[3] == 0
    return delta_hat


def packed_desc(lm, desc):
    """A copy of the descriptor that selects the packed-weight kernels, or None if the shape cannot."""
    if lm.locmoe_packed_weights_bytes(desc) == 0 or desc.x_dtype != lm.LOCMOE_BF16:
        return None
    import copy
    d2 = copy.copy(desc)
    d2.w_packed = 1
    return d2


def pack(env, desc, W_in_dev, W_out_dev):
    torch, lm, hz = env
    n = lm.locmoe_packed_weights_bytes(desc)
    assert n == W_in_dev.numel() * 2
    Wi = torch.empty_like(W_in_dev); Wo = torch.empty_like(W_out_dev)
    lm.locmoe_pack_weights(desc, W_in_dev, W_out_dev, Wi, Wo)
    torch.cuda.synchronize()
    # the documented layout, checked on a few 16-byte chunks: chunk p of block (e, nt, kt) holds row p/4,
    # k-chunk (p%4) ^ ((row/2)%4)
    rng = np.random.default_rng(5)
    for W, Wp in ((W_in_dev, Wi), (W_out_dev, Wo)):
        E, N, K = W.shape
        flat = Wp.view(-1)
        for _ in range(64):
            e, nt, kt, p = (int(rng.integers(0, E)), int(rng.integers(0, N // 256)), int(rng.integers(0, K // 32)),
                            int(rng.integers(0, 1024)))
            row = p // 4
            kc = (p % 4) ^ ((row // 2) % 4)
            off = (((e * (N // 256) + nt) * (K // 32) + kt) * 1024 + p) * 8
            assert torch.equal(flat[off:off + 8], W[e, nt * 256 + row, kt * 32 + kc * 8: kt * 32 + kc * 8 + 8])
    return Wi, Wo


def poison(*tensors):
    """NaN in every element: a row the kernels skip cannot pass for a result."""
    for t in tensors:
        t.fill_(float("nan"))


def assert_rows_written(t, K, name):
    """Rows [0,K) hold results (no sentinel left), rows >= K were not touched."""
    import torch
    assert not bool(torch.isnan(t[:K]).any()), f"{name}: a row below K was not written"
    assert bool(torch.isnan(t[K:]).all()), f"{name}: a row at or above K was written"


def check_ffn(env, c, desc, b, x, s, K, W_in_dev, W_out_dev, weights):
    """FFN on the oracle's send buffer, every element of H's widest segment row and of out against the oracle,
    for the row-major kernels and (where the shape allows) the packed-weight kernels."""
    torch, lm, hz = env
    b.send[:K].copy_(hz.to_device(x[s["row_token"]], c.dtype))
    b.seg_off.copy_(i32(torch, s["seg_off"])); b.buf_expert.copy_(i32(torch, s["buf_expert"]))
    ref = orc.expert_ffn(x[s["row_token"]], s["seg_off"], s["buf_expert"], weights)

    def compare(out_t, H_t):
        assert_rows_written(out_t, K, "out"); assert_rows_written(H_t, K, "H")
        got = hz.to_host_f32(out_t[:K])
        assert rel_l2(got, ref) <= 1e-2
        if K:
            rows = np.linalg.norm(got - ref, axis=1) / (np.linalg.norm(ref, axis=1) + 1e-30)
            assert rows.max() <= 3e-2                                    # no single row is off
            # the intermediate H = GeLU(W_in x), element by element: bf16 rounding + the erfc formula
            r = int(np.argmax(np.diff(s["seg_off"])))
            e = int(s["buf_expert"][r]); a = int(s["seg_off"][r])
            xb = wl.round_to_storage(x[s["row_token"][a]], "bf16").astype(np.float64)
            href = orc.gelu(weights(e)[0].astype(np.float64) @ xb)
            hgot = hz.to_host_f32(H_t[a])
            assert np.all(np.abs(hgot - href) <= 2.0 ** -7 * np.abs(href) + 2e-6)

    poison(b.out, b.H)
    lm.locmoe_expert_ffn(desc, b.send, b.seg_off, b.buf_expert, W_in_dev, W_out_dev, b.H, b.out)
    torch.cuda.synchronize()
    compare(b.out, b.H)
    dp = packed_desc(lm, desc)
    if dp is not None:                                                   # same inputs through the packed-weight kernels
        Wi, Wo = pack(env, desc, W_in_dev, W_out_dev)
        poison(b.out, b.H)
        lm.locmoe_expert_ffn(dp, b.send, b.seg_off, b.buf_expert, Wi, Wo, b.H, b.out)       # fixed tile assignment
        torch.cuda.synchronize()
        compare(b.out, b.H)
        poison(b.out, b.H)
        lm.locmoe_expert_ffn_ws(dp, b.send, b.seg_off, b.buf_expert, Wi, Wo, b.H, b.out, b.ffn_ws,
                                lm.LOCMOE_FFN_WS_BYTES)                                      # tiles claimed from ws
        torch.cuda.synchronize()
        compare(b.out, b.H)
        assert int(b.ffn_ws.max()) == 0
    return ref


def check_combine(env, c, desc, b, out_ref, slot, w):
    """Combine alone on a given out buffer: the only rounding is the final store."""
    torch, lm, hz = env
    K = out_ref.shape[0]
    out_st = wl.round_to_storage(out_ref.astype(np.float32), c.dtype)
    if K:
        b.out[:K].copy_(hz.to_device(out_st, c.dtype))
    w32 = w.astype(np.float32)
    lm.locmoe_combine(desc, b.out, i32(torch, slot), torch.from_numpy(w32).cuda(), b.y)
    torch.cuda.synchronize()
    y = hz.to_host_f32(b.y)
    ref = orc.combine(out_st.astype(np.float64), slot, w32.astype(np.float64))
    assert np.all(y[slot < 0] == 0)
    tol = 2.0 ** -8 if c.dtype == "bf16" else 2.0 ** -23
    assert np.all(np.abs(y - ref) <= tol * np.abs(ref) + 1e-37)


def run_full(env, c, C, *, T=None, eps=None, relu=True, e2n=None, use_home=True, alpha=wl.ALPHA, mu=wl.MU):
    """Every step against the oracle, element by element, then the chained path end to end."""
    torch, lm, hz = env
    say(f"[case] cfg={c.cfg} T={T or c.T} d={c.d} E={c.E} N={c.N} h={c.h} C={C} dtype={c.dtype} relu={relu} "
        f"eps={'y' if eps is not None else 'n'} e2n={'custom' if e2n is not None else 'default'}")
    x, home = wl.hidden_states(c, T)
    T = len(x)
    if not use_home:
        home = None
    desc = lm.make_desc(T, c.d, c.E, c.N, c.h, C, c.dtype, relu, alpha, mu)
    b = lm.alloc_buffers(desc)
    x_dev = hz.to_device(x, c.dtype)
    g32 = check_gate(env, c, x, x_dev, desc, b.g)
    eid, w = check_route(env, c, desc, b, g32, eps, home, e2n, relu, alpha, mu)
    s, K = check_dispatch(env, c, desc, b, x, x_dev, eid, e2n, C)
    ws = {e: wl.expert_weights(c, e) for e in range(c.E)}
    W_in = torch.stack([hz.to_device(ws[e][0], "bf16") for e in range(c.E)])
    W_out = torch.stack([hz.to_device(ws[e][1], "bf16") for e in range(c.E)])
    out_ref = check_ffn(env, c, desc, b, x, s, K, W_in, W_out, lambda e: ws[e])
    check_combine(env, c, desc, b, out_ref, s["slot"], w)
    # end to end on the GPU's own intermediates
    b2 = lm.alloc_buffers(desc)
    poison(b2.y, b2.out, b2.H)
    eps_dev = None if eps is None else torch.from_numpy(eps.astype(np.float32)).cuda()
    lm.forward(desc, x_dev, None if home is None else i32(torch, home), None if e2n is None else i32(torch, e2n),
               W_in, W_out, b2, eps=eps_dev)
    torch.cuda.synchronize()
    eid_gpu = b2.eid.cpu().numpy()
    nflip = int((eid_gpu != eid).sum())
    say(f"        K={K} dropped={T - K} eid flips vs oracle (near ties only)={nflip}")
    y_ref = orc.combine(out_ref, s["slot"], w)
    y = hz.to_host_f32(b2.y)
    assert not np.isnan(y).any()                                           # every row of y is written
    if nflip == 0:
        assert np.array_equal(b2.slot.cpu().numpy(), s["slot"])
        assert rel_l2(y, y_ref) <= 1e-2
    else:
        # a flip is legitimate only where the two best float64 scores agree to fp32 rounding
        g64 = orc.gate(x, c.E)
        for m in np.nonzero(eid_gpu != eid)[0]:
            assert abs(g64[m, eid_gpu[m]] - g64[m, eid[m]]) <= 1e-5 * np.abs(x[m]).mean()
        # every other token kept on both sides still gets its expert's row times its score, whatever slot it has
        same = (eid_gpu == eid) & (b2.slot.cpu().numpy() >= 0) & (s["slot"] >= 0)
        assert rel_l2(y[same], y_ref[same]) <= 1e-2
    return b2


# ------------------------------------------------------------------------------------------
def test_config1_fp32(env):
    c = wl.CONFIGS[1]
    run_full(env, c, c.C)
    run_full(env, c, 1)                       # the paper's measured delta: bound < 1 token


def test_config2_bf16(env):
    c = wl.CONFIGS[2]
    run_full(env, c, c.C)


def test_small_odd_shapes(env):
    c = wl.small_config()                     # T=96 d=48 E=6 N=3 h=40: nothing is a tile multiple
    run_full(env, c, 9)
    run_full(env, c, 200)                     # capacity above every count: nothing dropped
    run_full(env, wl.small_config(dtype="f32"), 5)
    e2n = np.array([2, 0, 1, 1, 0, 2], np.int32)
    eps = np.array([0.3, -0.2, 0.0, 0.5, -1.0, 0.1], np.float32)
    run_full(env, c, 9, eps=eps, e2n=e2n)
    run_full(env, c, 9, relu=False, use_home=False)
    run_full(env, wl.small_config(T=1, E=3, N=1, d=24, h=8), 1)
    run_full(env, wl.small_config(T=5, E=1, N=1, d=8, h=8), 2)


def test_ragged_token_counts_and_wide_experts(env):
    # T not a multiple of any block size; E=128 with 40-wide blocks (5 chunks: the LDS gate path)
    run_full(env, wl.small_config(T=2500, d=5120, E=128, N=16, h=64, clusters=9), 7)
    # E=200 > 64 lanes: several experts per lane in the router; 8-wide blocks
    run_full(env, wl.small_config(T=1111, d=1600, E=200, N=8, h=16, clusters=9), 3)
    # 12-wide blocks: not a whole number of 16-byte chunks -> scalar gate path
    run_full(env, wl.small_config(T=300, d=96, E=8, N=2, h=24), 20)
    run_full(env, wl.small_config(T=300, d=96, E=8, N=2, h=24, dtype="f32"), 20)


def test_expert_count_limits(env):
    # the largest expert count the ABI allows: 16 experts per lane in the router, 1-wide GrAP blocks
    run_full(env, wl.small_config(T=700, d=1024, E=1024, N=32, h=8, clusters=7), 2)
    # one node, every expert local; capacity of a single row
    run_full(env, wl.small_config(T=257, d=64, E=64, N=1, h=16, clusters=3), 1)
    # more nodes than the default map could give evenly is rejected on the host; a free-form map works
    e2n = (np.arange(12) * 5 % 7).astype(np.int32)
    run_full(env, wl.small_config(T=513, d=96, E=12, N=7, h=24, clusters=4), 11, e2n=e2n)


def test_tuned_gemm_tiles_with_ragged_segments(env):
    # d, h multiples of the tuned tile; capacity spans several 256-row tiles with ragged tails
    run_full(env, wl.small_config(T=4096, d=256, E=4, N=2, h=512, clusters=3), 700)
    run_full(env, wl.small_config(T=3000, d=512, E=8, N=2, h=256, clusters=4, dtype="bf16"), 300)
    # many segments for few tiles: empty segments, one- and two-tile segments in one persistent launch
    run_full(env, wl.small_config(T=6000, d=256, E=64, N=8, h=512, clusters=5), 300)
    # the largest expert count of the persistent kernel (64 segments per XCD queue), mostly tiny or empty segments
    run_full(env, wl.small_config(T=5000, d=512, E=512, N=8, h=256, clusters=6), 40)
    # above it, and an expert count that is no multiple of 8: one tile per work-group
    run_full(env, wl.small_config(T=3000, d=1024, E=1024, N=32, h=256, clusters=7), 8)
    run_full(env, wl.small_config(T=2000, d=768, E=12, N=4, h=256, clusters=3), 400)
    # the shortest K the packed layout allows (four double steps) with three m-tiles per segment
    run_full(env, wl.small_config(T=3000, d=256, E=8, N=2, h=256, clusters=2), 700)
    # a long contraction (h = 8192) behind wide rows (d = 4096): more tiles on every XCD than it has work-groups
    run_full(env, wl.small_config(T=6000, d=4096, E=8, N=2, h=8192, clusters=2), 700)


def angles_case(env, c, shift, nbins, T=None, zero_rows=(), want_cos=True):
    torch, lm, hz = env
    x, _ = wl.hidden_states(c, T)
    x = x.copy()
    for m in zero_rows:
        x[m] = 0.0                                            # a token without a direction
    say(f"[angles] cfg={c.cfg} T={len(x)} d={c.d} E={c.E} dtype={c.dtype} shift={shift} nbins={nbins}")
    desc = lm.make_desc(len(x), c.d, c.E, c.N, c.h, 1, c.dtype)
    eid = orc.route(orc.gate(x, c.E).astype(np.float32))[0]
    dh = check_angles(env, c, x, hz.to_device(x, c.dtype), desc, eid, shift, nbins, want_cos)
    say(f"         delta_hat={dh:.5f}")


def test_angles_between_tokens_and_gating_weights(env):
    """Section 4.1's measurement (cosine histograms per expert, smallest routed cosine) on the paper-shaped
    configurations and on every gate kernel variant."""
    angles_case(env, wl.CONFIGS[1], 1, 64)
    angles_case(env, wl.CONFIGS[2], 3, 100)
    angles_case(env, wl.small_config(), 1, 7, zero_rows=(0, 50))
    angles_case(env, wl.small_config(dtype="f32"), -1, 1)
    angles_case(env, wl.small_config(T=5, E=1, N=1, d=8, h=8), 1, 4)                  # the other expert is itself
    angles_case(env, wl.small_config(T=2500, d=5120, E=128, N=16, h=64, clusters=9), 64, 33, zero_rows=(2499,))
    angles_case(env, wl.small_config(T=300, d=96, E=8, N=2, h=24), 9, 16)            # scalar gate path
    angles_case(env, wl.small_config(T=300, d=96, E=8, N=2, h=24, dtype="f32"), 2, 16, want_cos=False)
    angles_case(env, wl.small_config(T=700, d=1024, E=1024, N=32, h=8, clusters=7), 1, 8)
    angles_case(env, wl.small_config(T=1111, d=1600, E=200, N=8, h=16, clusters=9), 199, 4096)


def test_whole_path_bitwise_repeatable(env):
    """No atomics whose order could matter anywhere on the path: y is bit-identical from run to run, for the
    row-major and the packed-weight kernels."""
    torch, lm, hz = env
    c = wl.small_config(T=3000, d=512, E=8, N=2, h=256, clusters=4)
    x, home = wl.hidden_states(c)
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, 300, c.dtype)
    ws = [wl.expert_weights(c, e) for e in range(c.E)]
    W_in = torch.stack([hz.to_device(w[0], "bf16") for w in ws]); W_out = torch.stack([hz.to_device(w[1], "bf16") for w in ws])
    x_dev = hz.to_device(x, c.dtype); home_dev = i32(torch, home)
    for d_, wi, wo in ((desc, W_in, W_out), (packed_desc(lm, desc),) + pack(env, desc, W_in, W_out)):
        b = lm.alloc_buffers(d_)
        ref = None
        for _ in range(5):
            b.y.zero_(); b.H.zero_(); b.out.zero_()
            lm.forward(d_, x_dev, home_dev, None, wi, wo, b)
            torch.cuda.synchronize()
            cur = b.y.view(torch.int16).cpu().numpy().tobytes()
            ref = ref or cur
            assert cur == ref


def test_ffn_tile_claims_against_fixed_assignment_across_launches_and_streams(env):
    """The persistent grouped GEMM either takes its tiles in a fixed round-robin order (entry points without a
    workspace) or claims them from queue words in a caller workspace (*_ws).  Both must give the same bits (the
    fixed form is checked against the oracle first); a workspace must come back zeroed, so that many launches in
    a row can share one; launches that overlap on two streams use a workspace each."""
    torch, lm, hz = env
    # 8 experts = one segment per XCD, up to 2 x 32 tiles each for 32 work-groups: tiles are claimed dynamically
    c = wl.small_config(T=3000, d=512, E=8, N=2, h=8192, clusters=4)
    run_full(env, c, 300)
    x, home = wl.hidden_states(c)
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, 300, c.dtype)
    ws = [wl.expert_weights(c, e) for e in range(c.E)]
    W_in = torch.stack([hz.to_device(w[0], "bf16") for w in ws]); W_out = torch.stack([hz.to_device(w[1], "bf16") for w in ws])
    dp = packed_desc(lm, desc)
    Wi, Wo = pack(env, desc, W_in, W_out)
    b = lm.alloc_buffers(dp)
    lm.forward(dp, hz.to_device(x, c.dtype), i32(torch, home), None, Wi, Wo, b)
    torch.cuda.synchronize()
    K = int(b.seg_off[-1])
    bits = lambda t: t[:K].view(torch.int16).cpu().numpy().tobytes()
    poison(b.H, b.out)
    lm.locmoe_expert_ffn(dp, b.send, b.seg_off, b.buf_expert, Wi, Wo, b.H, b.out)          # fixed assignment
    torch.cuda.synchronize()
    ref, refH = bits(b.out), bits(b.H)
    nws = lm.LOCMOE_FFN_WS_BYTES
    for it in range(70):
        poison(b.H, b.out)
        lm.locmoe_expert_ffn_ws(dp, b.send, b.seg_off, b.buf_expert, Wi, Wo, b.H, b.out, b.ffn_ws, nws)
        torch.cuda.synchronize()
        assert bits(b.out) == ref and bits(b.H) == refH, it
        assert int(b.ffn_ws.max()) == 0, it                                                   # handed back zeroed
    # the two halves as separate calls, and the variant that keeps Z
    Z = torch.empty_like(b.H)
    poison(b.H, b.out, Z)
    lm.locmoe_expert_ffn_in_save_ws(dp, b.send, b.seg_off, b.buf_expert, Wi, b.H, Z, b.ffn_ws, nws)
    lm.locmoe_expert_ffn_out_ws(dp, b.H, b.seg_off, b.buf_expert, Wo, b.out, b.ffn_ws, nws)
    torch.cuda.synchronize()
    assert bits(b.out) == ref and bits(b.H) == refH and int(b.ffn_ws.max()) == 0
    assert_rows_written(Z, K, "Z")
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]   # default priority
    Hs = [torch.zeros_like(b.H) for _ in streams]; outs = [torch.zeros_like(b.out) for _ in streams]
    wss = [torch.zeros(nws, dtype=torch.uint8, device="cuda") for _ in streams]
    torch.cuda.synchronize()
    for rep in range(3):
        for st, H, out, w_ in zip(streams, Hs, outs, wss):
            lm.locmoe_expert_ffn_ws(dp, b.send, b.seg_off, b.buf_expert, Wi, Wo, H, out, w_, nws, stream=st)
        torch.cuda.synchronize()
        for out in outs:
            assert bits(out) == ref, rep
            out.zero_()
        torch.cuda.synchronize()


def test_route_dispatch_deterministic(env):
    torch, lm, hz = env
    c = wl.CONFIGS[2]
    x, home = wl.hidden_states(c)
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, c.C, c.dtype)
    b = lm.alloc_buffers(desc)
    x_dev = hz.to_device(x, c.dtype); home_dev = i32(torch, home)
    first = None
    for it in range(10):
        lm.locmoe_gate(desc, x_dev, b.g)
        lm.locmoe_route(desc, b.g, None, home_dev, None, b.eid, b.w, b.cnt, b.Psum, b.stats, b.ws, b.ws_bytes)
        lm.locmoe_dispatch(desc, x_dev, b.eid, None, b.pos, b.slot, b.kept, b.seg_off, b.node_off, b.buf_expert,
                           b.row_token, b.send, b.ws, b.ws_bytes)
        torch.cuda.synchronize()
        K = int(b.seg_off[-1])
        cur = [t.cpu().numpy().tobytes() for t in (b.eid, b.w, b.Psum, b.stats, b.pos, b.slot, b.row_token[:K])]
        first = first or cur
        assert cur == first


# ------------------------------------------------------------------------------------------
# Full-size workloads: routing and dispatch element by element; FFN output and y on whole experts
# against the oracle and on every row against a second, independent kernel.
# ------------------------------------------------------------------------------------------
def experts_to_check(s):
    """Buffer ranks whose whole segments are compared with the oracle.  The persistent grouped GEMM ranks
    the segments by row count and deals them to eight tile queues (ranks 0..7 to queues 0..7, 8..15 to
    7..0, ...); one segment of every queue is taken, at a different depth of each queue, plus the
    fullest segment, the emptiest non-empty one, one that needs two row tiles with a short second one,
    and the first and last non-empty segments in buffer order.  (Only a way to choose samples: the
    comparison itself knows nothing of the kernel.)"""
    rows = np.diff(s["seg_off"])
    E = len(rows)
    order = sorted(range(E), key=lambda r: (-int(rows[r]), r))
    queues = [[] for _ in range(8)]
    for rank, r in enumerate(order):
        q = rank & 7
        queues[7 - q if (rank >> 3) & 1 else q].append(r)
    picked = []
    for q, members in enumerate(queues):
        live = [r for r in members if rows[r] > 0]
        if live:
            picked.append(live[(q * 3) % len(live)])
    nz = [r for r in range(E) if rows[r] > 0]
    if nz:
        picked += [max(nz, key=lambda r: rows[r]), min(nz, key=lambda r: rows[r]), nz[0], nz[-1]]
        two = [r for r in nz if rows[r] > 256]
        if two:
            picked.append(min(two, key=lambda r: rows[r]))
    return sorted(set(picked))


def run_big(env, c, C, with_ffn=True):
    torch, lm, hz = env
    say(f"[big] cfg={c.cfg} T={c.T} d={c.d} E={c.E} h={c.h} C={C}")
    t0 = time.time()
    x, home = wl.hidden_states(c)
    say(f"      inputs {time.time() - t0:.1f}s")
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, C, c.dtype)
    b = lm.alloc_buffers(desc)
    x_dev = hz.to_device(x, c.dtype)
    g32 = check_gate(env, c, x, x_dev, desc, b.g)
    eid, w = check_route(env, c, desc, b, g32, None, home, None, True, wl.ALPHA, wl.MU)
    s, K = check_dispatch(env, c, desc, b, x, x_dev, eid, None, C)
    say(f"      gate/route/dispatch ok, K={K} dropped={c.T - K} ({time.time() - t0:.1f}s)")
    if not with_ffn:
        rng = np.random.default_rng(1)
        out_ref = rng.standard_normal((K, c.d)).astype(np.float32)
        check_combine(env, c, desc, b, out_ref, s["slot"], w)
        return
    ranks = experts_to_check(s)
    cand = {int(s["buf_expert"][r]) for r in ranks}
    W_in, W_out, host_w = hz.upload_weights(c, keep=cand, progress=lambda a, n: say(f"      weights {a}/{n}"))
    say(f"      weights uploaded ({time.time() - t0:.1f}s)")
    # the oracle's output for every row of the chosen segments
    out_ref = {}
    for r in ranks:
        a, z = int(s["seg_off"][r]), int(s["seg_off"][r + 1])
        out_ref[r] = orc.ffn_rows(x[s["row_token"][a:z]], *host_w[int(s["buf_expert"][r])])
    nrows = sum(len(v) for v in out_ref.values())
    say(f"      oracle FFN on {len(ranks)} whole segments, {nrows} rows: ranks {ranks} ({time.time() - t0:.1f}s)")

    def whole_segments(out_t, H_t, what):
        assert_rows_written(out_t, K, what + " out"); assert_rows_written(H_t, K, what + " H")
        num = den = 0.0
        for r in ranks:
            a, z = int(s["seg_off"][r]), int(s["seg_off"][r + 1])
            got = hz.to_host_f32(out_t[a:z]).astype(np.float64)
            diff = np.linalg.norm(got - out_ref[r], axis=1)
            assert np.all(diff <= 3e-2 * np.linalg.norm(out_ref[r], axis=1) + 1e-30), (what, r)   # no single row is off
            assert rel_l2(got, out_ref[r]) <= 1e-2, (what, r)
            num += float((diff ** 2).sum()); den += float((out_ref[r] ** 2).sum())
        say(f"      {what}: {nrows} rows of {len(ranks)} segments rel-L2 {np.sqrt(num / den):.2e} ({time.time() - t0:.1f}s)")

    b.send[:K].copy_(hz.to_device(x[s["row_token"]], c.dtype))
    poison(b.out, b.H)
    lm.locmoe_expert_ffn(desc, b.send, b.seg_off, b.buf_expert, W_in, W_out, b.H, b.out)
    torch.cuda.synchronize()
    whole_segments(b.out, b.H, "row-major weights")
    out_rm = b.out[:K].float()
    # the benchmark's launch configuration: packed weights, direct-to-LDS persistent kernels
    dp = packed_desc(lm, desc)
    assert dp is not None
    W_in, W_out = pack(env, desc, W_in, W_out)
    desc = dp
    poison(b.out, b.H)
    lm.locmoe_expert_ffn(desc, b.send, b.seg_off, b.buf_expert, W_in, W_out, b.H, b.out)
    torch.cuda.synchronize()
    whole_segments(b.out, b.H, "packed weights, fixed tile assignment")
    out_fixed = b.out[:K].clone()
    poison(b.out, b.H)
    lm.locmoe_expert_ffn_ws(desc, b.send, b.seg_off, b.buf_expert, W_in, W_out, b.H, b.out, b.ffn_ws,
                            lm.LOCMOE_FFN_WS_BYTES)
    torch.cuda.synchronize()
    whole_segments(b.out, b.H, "packed weights, tiles claimed from the workspace")
    assert torch.equal(b.out[:K].view(torch.int16), out_fixed.view(torch.int16))          # the same bits either way
    assert int(b.ffn_ws.max()) == 0
    del out_fixed
    # every row of the buffer: two kernels that share neither tiling nor scheduling, each within the bar of the
    # oracle on the segments above, agree on all K rows (a tile skipped or claimed twice on any expert shows here)
    diff = (b.out[:K].float() - out_rm).norm(dim=1)
    ref_n = out_rm.norm(dim=1)
    assert bool((diff <= 3e-2 * ref_n + 1e-30).all())
    assert float(diff.norm() / ref_n.norm()) <= 1e-2
    del out_rm, diff, ref_n
    # end to end on the GPU's own intermediates, in sentinel-filled buffers
    b2 = lm.alloc_buffers(desc)
    poison(b2.y, b2.out, b2.H)
    lm.forward(desc, x_dev, i32(torch, home), None, W_in, W_out, b2)
    torch.cuda.synchronize()
    eid_gpu = b2.eid.cpu().numpy()
    slot_gpu = b2.slot.cpu().numpy()
    flips = np.nonzero(eid_gpu != eid)[0]
    say(f"      end-to-end eid flips vs oracle: {len(flips)}")
    g64 = orc.gate(x, c.E) if len(flips) else None
    for m in flips:
        assert abs(g64[m, eid_gpu[m]] - g64[m, eid[m]]) <= 1e-5 * np.abs(x[m]).mean()
    if len(flips) == 0:
        assert np.array_equal(slot_gpu, s["slot"])
    Kg = int(b2.seg_off[-1])
    assert_rows_written(b2.out, Kg, "end-to-end out"); assert_rows_written(b2.H, Kg, "end-to-end H")
    assert not bool(torch.isnan(b2.y).any())                                   # every row of y is written
    kept_dev = b2.slot >= 0
    assert float(b2.y[~kept_dev].abs().max()) == 0.0 if bool((~kept_dev).any()) else True      # dropped: exactly zero
    # Eq. 1 token by token on the chosen experts: y_m = w_m * expert(x_m) for every token they keep (tokens whose
    # expert flipped, or that a flip pushed across the capacity limit, are left out)
    w_gpu = b2.w.cpu().numpy()
    assert np.allclose(w_gpu, w, rtol=1e-5, atol=0) if len(flips) == 0 else True
    checked = 0
    for r in ranks:
        a, z = int(s["seg_off"][r]), int(s["seg_off"][r + 1])
        toks = s["row_token"][a:z]
        ok = (eid_gpu[toks] == eid[toks]) & (slot_gpu[toks] >= 0)
        y_rows = hz.to_host_f32(b2.y[torch.from_numpy(toks[ok].astype(np.int64)).cuda()])
        ref = w[toks[ok]][:, None] * out_ref[r][ok]
        assert rel_l2(y_rows, ref) <= 1e-2, r
        assert np.all(np.linalg.norm(y_rows - ref, axis=1) <= 3e-2 * np.linalg.norm(ref, axis=1) + 1e-30), r
        checked += int(ok.sum())
    say(f"      y on {checked} tokens of the chosen experts ok ({time.time() - t0:.1f}s)")
    # at any size: a kept token's row is its score times its out row, rounded once
    kept_idx = torch.nonzero(kept_dev).squeeze(1)
    prod = (b2.w[kept_idx][:, None] * b2.out[b2.slot[kept_idx].long()].float()).to(b2.y.dtype)
    assert torch.equal(b2.y[kept_idx], prod)


def test_config3_full_size_capacity_sweep(env):
    c = wl.CONFIGS[3]
    torch, lm, hz = env
    x, home = wl.hidden_states(c)
    x_dev = hz.to_device(x, c.dtype)
    g32 = orc.gate(x, c.E).astype(np.float32)
    eid, w, _, _ = orc.route(g32)
    for C in (c.C, 1024, 1280, 2048, 1):
        say(f"[big] cfg=3 dispatch sweep C={C}")
        desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, C, c.dtype)
        b = lm.alloc_buffers(desc)
        check_dispatch(env, c, desc, b, x, x_dev, eid, None, C)


def test_config3_full_size_paper_bound_capacity(env):
    """Capacity 512, the Theorem 1 bound at this configuration's delta: half of the tokens dropped."""
    c = wl.CONFIGS[3]
    run_big(env, c, c.C)


def test_config3_full_size_large_capacity(env):
    """Capacity 2 048 (116 of 32 768 tokens dropped): segments of up to 2 048 rows, eight row tiles per weight tile."""
    run_big(env, wl.CONFIGS[3], 2048)


def test_config4_full_size_headline(env):
    c = wl.CONFIGS[4]
    run_big(env, c, c.C)


def test_config5_full_size_routing_stress(env):
    """The largest configuration: adversarial routing (four hot experts), 128 experts = 16 segments per XCD queue
    of the persistent GEMM, d = 5120 (20 column tiles); whole segments as at config 4."""
    c = wl.CONFIGS[5]
    run_big(env, c, c.C, with_ffn=True)


def test_element_indices_past_two_to_the_31(env):
    """Maximum sizes: T*d and K*d lie beyond 2^31 elements (x, y and the send buffer beyond 2^32 bytes), so an
    address formed in 32 bits anywhere on the path shows as a wrong row.  The input is one seeded block of 32 768
    tokens repeated 17 times on the device; what depends on one token alone (gating values, expert, score) must
    repeat bit for bit, what depends on the whole sequence (counts, losses, positions, slots, the packed buffers)
    is compared with the oracle run on the repeated sequence, the FFN with the oracle on sampled rows of the
    chosen segments (first, last and random rows of each), Eq. 1's last step with its definition on every token."""
    import dataclasses
    torch, lm, hz = env
    cb = wl.small_config(T=32768, d=4096, E=64, N=8, h=256, clusters=64, zipf=0.3)
    R, C = 17, 24576
    c = dataclasses.replace(cb, T=R * cb.T)
    assert c.T * c.d > 2 ** 31
    say(f"[past 2^31] T={c.T} d={c.d} E={c.E} h={c.h} C={C}")
    t0 = time.time()
    xb, homeb = wl.hidden_states(cb)
    home = np.tile(homeb, R)
    x_dev = hz.to_device(xb, c.dtype).repeat(R, 1)
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, C, c.dtype)
    b = lm.alloc_buffers(desc)
    # gate: the first block against the oracle, every other block against the first
    poison(b.g)
    lm.locmoe_gate(desc, x_dev, b.g)
    torch.cuda.synchronize()
    gref = orc.gate(xb, c.E)
    g0 = b.g[:cb.T].cpu().numpy()
    blk = c.d // c.E
    assert rel_l2(g0, gref) <= 1e-5
    assert np.all(np.abs(g0 - gref) <= 1e-5 * np.abs(xb.astype(np.float64)).reshape(cb.T, c.E, blk).sum(axis=2) / blk + 1e-30)
    assert bool((b.g.view(R, cb.T, c.E) == b.g[:cb.T].unsqueeze(0)).all())
    g32 = np.tile(gref.astype(np.float32), (R, 1))
    eid, w = check_route(env, c, desc, b, g32, None, home, None, True, wl.ALPHA, wl.MU)
    assert np.array_equal(eid.reshape(R, cb.T), np.tile(eid[:cb.T], (R, 1)))
    # dispatch
    poison(b.send)
    lm.locmoe_dispatch(desc, x_dev, i32(torch, eid), None, b.pos, b.slot, b.kept, b.seg_off, b.node_off,
                       b.buf_expert, b.row_token, b.send, b.ws, b.ws_bytes)
    torch.cuda.synchronize()
    s = orc.slots(eid, c.E, C, np.arange(c.E) // (c.E // c.N), c.N)
    K = int(s["seg_off"][-1])
    assert K * c.d > 2 ** 31
    for name in ("pos", "slot", "kept", "seg_off", "node_off", "buf_expert"):
        assert np.array_equal(getattr(b, name).cpu().numpy(), s[name]), name
    assert np.array_equal(b.row_token.cpu().numpy()[:K], s["row_token"])
    assert torch.equal(b.send[:K].view(torch.int16), x_dev[b.row_token[:K].long()].view(torch.int16))
    assert bool(torch.isnan(b.send[K:]).all())
    say(f"      gate/route/dispatch ok, K={K} dropped={c.T - K} ({time.time() - t0:.1f}s)")
    # expert FFN: sampled rows of the chosen segments (always the first and the last rows of each)
    ranks = experts_to_check(s)
    cand = {int(s["buf_expert"][r]) for r in ranks}
    W_in, W_out, host_w = hz.upload_weights(c, keep=cand)
    rng = np.random.default_rng(11)
    rows_of, ref_of = {}, {}
    for r in ranks:
        a, z = int(s["seg_off"][r]), int(s["seg_off"][r + 1])
        pick = np.unique(np.concatenate([np.arange(a, min(a + 48, z)), np.arange(max(z - 48, a), z),
                                         rng.integers(a, z, size=160)]))
        rows_of[r] = pick
        ref_of[r] = orc.ffn_rows(xb[s["row_token"][pick] % cb.T], *host_w[int(s["buf_expert"][r])])

    def sampled(out_t, H_t, what):
        assert_rows_written(out_t, K, what + " out"); assert_rows_written(H_t, K, what + " H")
        for r in ranks:
            got = hz.to_host_f32(out_t[torch.from_numpy(rows_of[r]).cuda()]).astype(np.float64)
            diff = np.linalg.norm(got - ref_of[r], axis=1)
            assert np.all(diff <= 3e-2 * np.linalg.norm(ref_of[r], axis=1) + 1e-30), (what, r)
            assert rel_l2(got, ref_of[r]) <= 1e-2, (what, r)

    poison(b.out, b.H)
    lm.locmoe_expert_ffn(desc, b.send, b.seg_off, b.buf_expert, W_in, W_out, b.H, b.out)
    torch.cuda.synchronize()
    sampled(b.out, b.H, "row-major weights")
    out_rm = b.out[:K].clone()
    dp = packed_desc(lm, desc)
    assert dp is not None
    Wi, Wo = pack(env, desc, W_in, W_out)
    poison(b.out, b.H)
    lm.locmoe_expert_ffn_ws(dp, b.send, b.seg_off, b.buf_expert, Wi, Wo, b.H, b.out, b.ffn_ws, lm.LOCMOE_FFN_WS_BYTES)
    torch.cuda.synchronize()
    sampled(b.out, b.H, "packed weights")
    # every row: the two kernels, which share neither tiling nor scheduling, agree within the bar
    for a in range(0, K, 65536):
        z = min(K, a + 65536)
        ref = out_rm[a:z].float()
        diff = (b.out[a:z].float() - ref).norm(dim=1)
        assert bool((diff <= 3e-2 * ref.norm(dim=1) + 1e-30).all()), a
    del out_rm
    say(f"      FFN on {sum(len(v) for v in rows_of.values())} sampled rows of {len(ranks)} segments ok ({time.time() - t0:.1f}s)")
    # combine: a kept token's row is its score times its out row, rounded once; a dropped token's row is zero
    poison(b.y)
    lm.locmoe_combine(dp, b.out, b.slot, b.w, b.y)
    torch.cuda.synchronize()
    kept_dev = b.slot >= 0
    assert not bool(torch.isnan(b.y).any())
    if bool((~kept_dev).any()):
        assert float(b.y[~kept_dev].abs().max()) == 0.0
    for a in range(0, c.T, 131072):
        idx = torch.nonzero(kept_dev[a:a + 131072]).squeeze(1) + a
        prod = (b.w[idx][:, None] * b.out[b.slot[idx].long()].float()).to(b.y.dtype)
        assert torch.equal(b.y[idx], prod), a
    say(f"      combine ok ({time.time() - t0:.1f}s)")


def test_config4_full_size_angles(env):
    """The headline shape: every token's cosine, the histograms and delta_hat against the oracle."""
    angles_case(env, wl.CONFIGS[4], 1, 64)
