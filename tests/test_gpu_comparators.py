"""GPU parity of the comparison routers (Section 2, Section 3.2.1, Section 4) through the C ABI against the oracle:
the dense learned gate (the switch router's gate) and hash routing, alone and followed by the shared path.

Bars: dense gating values: relative L2 <= 1e-5 and |diff| <= 1e-5 * sum_j |omega_ij x_mj| per element (fp32
accumulation of exact bf16 products; the same form as the GrAP gate's bar); hash routing: eid, cnt, w bit-exact;
whatever follows (route on the oracle's gating values, dispatch, FFN, combine): the bars of the LocMoE path.
"""
import sys

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


def check_dense_gate(env, c, T=None, Wg=None):
    torch, lm, hz = env
    x, _ = wl.hidden_states(c, T)
    T = len(x)
    Wg = wl.dense_gate_weight(c) if Wg is None else Wg
    say(f"[dense gate] T={T} d={c.d} E={c.E} dtype={c.dtype}")
    desc = lm.make_desc(T, c.d, c.E, c.N, c.h, 1, c.dtype)
    g_dev = torch.full((T, c.E), float("nan"), dtype=torch.float32, device="cuda")
    lm.locmoe_gate_dense(desc, hz.to_device(x, c.dtype), hz.to_device(Wg, c.dtype), g_dev)
    torch.cuda.synchronize()
    g = g_dev.cpu().numpy()
    ref = orc.gate_dense_learned(x, Wg)
    assert not np.isnan(g).any()
    assert rel_l2(g, ref) <= 1e-5
    bound = 1e-5 * (np.abs(x.astype(np.float64)) @ np.abs(Wg.astype(np.float64)).T)
    assert np.all(np.abs(g - ref) <= bound + 1e-30)
    return x, Wg, g, ref


def test_dense_gate_matches_oracle_on_every_kernel_variant(env):
    check_dense_gate(env, wl.CONFIGS[1])                                              # fp32: generic kernel
    check_dense_gate(env, wl.CONFIGS[2])                                              # E=16: one 32-expert tile
    check_dense_gate(env, wl.small_config())                                          # d=48, E=6: generic, bf16
    check_dense_gate(env, wl.small_config(T=2500, d=5120, E=128, N=16, h=64, clusters=9))   # four tiles, ragged T
    check_dense_gate(env, wl.small_config(T=1000, d=1280, E=80, N=8, h=16, clusters=4))     # three tiles, E % 32 != 0
    check_dense_gate(env, wl.small_config(T=333, d=1600, E=200, N=8, h=16, clusters=4))     # two passes over experts
    check_dense_gate(env, wl.small_config(T=130, d=192, E=6, N=3, h=8))                     # E % 4 != 0: scalar stores
    check_dense_gate(env, wl.small_config(T=700, d=1024, E=1024, N=32, h=8, clusters=7))    # eight passes


def test_dense_gate_with_the_grap_weight_is_the_grap_gate(env):
    """Eq. 4's weight in the dense layer gives the gating values of locmoe_gate (Section 3.2.1)."""
    torch, lm, hz = env
    for c in (wl.CONFIGS[2], wl.small_config(T=500, d=1024, E=64, N=8, h=16)):
        W = wl.round_to_storage(orc.grap_weight(c.E, c.d).astype(np.float32), c.dtype)   # n/d is a power of two here
        assert np.array_equal(W, orc.grap_weight(c.E, c.d))
        x, _, g, _ = check_dense_gate(env, c, Wg=W)
        desc = lm.make_desc(len(x), c.d, c.E, c.N, c.h, 1, c.dtype)
        g2 = torch.empty(len(x), c.E, dtype=torch.float32, device="cuda")
        lm.locmoe_gate(desc, hz.to_device(x, c.dtype), g2)
        torch.cuda.synchronize()
        assert rel_l2(g, g2.cpu().numpy()) <= 1e-5


def test_switch_router_path_at_config4_full_size(env):
    """The switch comparator at the headline shape: dense gate on the GPU against the oracle (every element), then
    route on the oracle's float32 gating values (bit-exact assignments, Eq. 5) and the dispatch."""
    torch, lm, hz = env
    c = wl.CONFIGS[4]
    x, Wg, g, ref = check_dense_gate(env, c)
    g32 = ref.astype(np.float32)
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, c.C, c.dtype)
    b = lm.alloc_buffers(desc)
    lm.locmoe_route(desc, torch.from_numpy(g32).cuda(), None, None, None, b.eid, b.w, b.cnt, b.Psum, b.stats, b.ws,
                    b.ws_bytes)
    torch.cuda.synchronize()
    eid, w, p, _ = orc.route(g32)
    st = orc.route_stats(eid, p, None, wl.expert_to_node(c), c.N, wl.ALPHA, wl.MU)
    assert np.array_equal(b.eid.cpu().numpy(), eid) and np.array_equal(b.cnt.cpu().numpy(), st["cnt"])
    assert np.allclose(b.w.cpu().numpy(), w, rtol=1e-5, atol=0)
    assert float(b.stats[0]) == pytest.approx(st["L_aux"], rel=1e-5)
    # flips between the GPU's own gating values and the oracle's: near ties only
    eid_gpu = orc.route(g)[0]
    flips = np.nonzero(eid_gpu != eid)[0]
    say(f"      switch router: max count {st['cnt'].max()}, empty experts {(st['cnt'] == 0).sum()}, eid flips {len(flips)}")
    scale = (np.abs(x.astype(np.float64)) @ np.abs(Wg.astype(np.float64)).T)
    for m in flips:
        assert abs(ref[m, eid_gpu[m]] - ref[m, eid[m]]) <= 2e-5 * scale[m].max()
    s = orc.slots(eid, c.E, c.C, wl.expert_to_node(c), c.N)
    lm.locmoe_dispatch(desc, hz.to_device(x, c.dtype), b.eid, None, b.pos, b.slot, b.kept, b.seg_off, b.node_off,
                       b.buf_expert, b.row_token, b.send, b.ws, b.ws_bytes)
    torch.cuda.synchronize()
    for name in ("pos", "slot", "kept", "seg_off"):
        assert np.array_equal(getattr(b, name).cpu().numpy(), s[name]), name


def check_hash(env, c, keys, seed, T=None):
    torch, lm, hz = env
    T = c.T if T is None else T
    desc = lm.make_desc(T, c.d, c.E, c.N, c.h, 1, c.dtype)
    eid_dev = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    w_dev = torch.full((T,), float("nan"), dtype=torch.float32, device="cuda")
    cnt_dev = torch.full((c.E,), -5, dtype=torch.int32, device="cuda")
    lm.locmoe_route_hash(desc, None if keys is None else i32(torch, keys), seed, eid_dev, w_dev, cnt_dev)
    torch.cuda.synchronize()
    eid, w, cnt = orc.route_hash(np.arange(T) if keys is None else keys, c.E, seed)
    assert np.array_equal(eid_dev.cpu().numpy(), eid)
    assert np.array_equal(cnt_dev.cpu().numpy(), cnt)
    assert np.array_equal(w_dev.cpu().numpy(), w.astype(np.float32))
    return eid, cnt


def test_hash_router_bit_exact(env):
    for c in (wl.CONFIGS[1], wl.CONFIGS[4], wl.CONFIGS[5], wl.small_config(T=2500, d=48, E=6),
              wl.small_config(T=7, d=1024, E=1024, N=32, h=8), wl.small_config(T=100000, d=8, E=1, N=1, h=8)):
        say(f"[hash] T={c.T} E={c.E}")
        check_hash(env, c, None, 0)
        check_hash(env, c, None, 12345)
        keys = wl.token_keys(c)
        eid, cnt = check_hash(env, c, keys, 7)
        check_hash(env, c, (keys.astype(np.int64) - 25000).astype(np.int32), 0xFFFFFFFF)        # negative ids, largest seed
    c = wl.CONFIGS[4]
    eid, cnt = check_hash(env, c, None, 3)
    say(f"      config 4 by position: max count {cnt.max()}, min {cnt.min()} (mean {c.T / c.E:.0f})")


def test_hash_router_end_to_end(env):
    """Hash routing followed by the shared dispatch, expert FFN and combine, against the oracle's layer with the same
    assignment and unit scores."""
    torch, lm, hz = env
    c = wl.small_config(T=3000, d=512, E=8, N=2, h=256, clusters=4)
    x, _ = wl.hidden_states(c)
    keys = wl.token_keys(c)
    C = 300
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, C, c.dtype)
    b = lm.alloc_buffers(desc)
    ws = {e: wl.expert_weights(c, e) for e in range(c.E)}
    W_in = torch.stack([hz.to_device(ws[e][0], "bf16") for e in range(c.E)])
    W_out = torch.stack([hz.to_device(ws[e][1], "bf16") for e in range(c.E)])
    x_dev = hz.to_device(x, c.dtype)
    for t in (b.y, b.out, b.H):
        t.fill_(float("nan"))
    lm.locmoe_route_hash(desc, i32(torch, keys), 11, b.eid, b.w, b.cnt)
    lm.locmoe_dispatch(desc, x_dev, b.eid, None, b.pos, b.slot, b.kept, b.seg_off, b.node_off, b.buf_expert,
                       b.row_token, b.send, b.ws, b.ws_bytes)
    lm.locmoe_expert_ffn(desc, b.send, b.seg_off, b.buf_expert, W_in, W_out, b.H, b.out)
    lm.locmoe_combine(desc, b.out, b.slot, b.w, b.y)
    torch.cuda.synchronize()
    eid, w, _ = orc.route_hash(keys, c.E, 11)
    s = orc.slots(eid, c.E, C, wl.expert_to_node(c), c.N)
    K = int(s["seg_off"][-1])
    assert np.array_equal(b.slot.cpu().numpy(), s["slot"])
    out = orc.expert_ffn(orc.dispatch(x, s["slot"], K), s["seg_off"], s["buf_expert"], lambda e: ws[e])
    y_ref = orc.combine(out, s["slot"], w)
    y = hz.to_host_f32(b.y)
    assert not np.isnan(y).any() and np.all(y[s["slot"] < 0] == 0)
    assert rel_l2(y, y_ref) <= 1e-2
