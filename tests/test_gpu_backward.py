"""GPU parity of the backward path (through the C ABI) against the backward oracle, step by step on the
oracle's own intermediates (rounded to what the step reads) and end to end on the GPU's.

Bars:
  * dout, dsend, dZ, dx, dW_in, dW_out (bf16 results of fp32 sums): relative L2 <= 1e-2 against the float64
    oracle, as for the forward FFN; fp32 storage (dout, dsend, dx of an fp32 layer): 1e-2 as well where a
    bf16 intermediate (Z, dZ, H) lies on the way, 1e-5 where none does;
  * dw: |diff| <= 1e-5 * sum_j |dy_j out_j| (fp32 dot product in a fixed order);
  * coef: 1e-5 relative;  dg: |diff| <= 2e-5 * max_i |dp[m,i]| per row (fp32 softmax, p <= 1);
  * transposed weights: bit-exact;  experts without rows: dW exactly zero.
"""
import sys

import numpy as np
import pytest

from oracle import locmoe_backward_oracle as bwd
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


def bf16_round(a):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.asarray(a, np.float32)))


def store_round(a, dtype):
    return wl.round_to_storage(np.asarray(a, np.float32), dtype)


def run_backward_case(env, c, C, *, T=None, eps=None, relu=True, e2n=None, use_home=True, alpha=0.3, mu=0.2):
    torch, lm, hz = env
    x, home = wl.hidden_states(c, T)
    T = len(x)
    dy = wl.upstream_grad(c, T)
    if not use_home:
        home = None
    say(f"[bwd] cfg={c.cfg} T={T} d={c.d} E={c.E} N={c.N} h={c.h} C={C} dtype={c.dtype} relu={relu} "
        f"eps={'y' if eps is not None else 'n'} home={'y' if use_home else 'n'}")
    e2n_full = np.asarray(e2n if e2n is not None else np.arange(c.E) // (c.E // c.N))
    ws = {e: wl.expert_weights(c, e) for e in range(c.E)}
    ref = bwd.moe_layer_backward(x, home, e2n_full, c.E, c.N, C, lambda e: ws[e], dy, eps, relu, alpha, mu)
    K = int(ref["seg_off"][-1])
    desc = lm.make_desc(T, c.d, c.E, c.N, c.h, C, c.dtype, relu, alpha, mu)
    b = lm.alloc_buffers(desc)
    gb = lm.alloc_grad_buffers(desc)
    x_dev, dy_dev = hz.to_device(x, c.dtype), hz.to_device(dy, c.dtype)
    home_dev = None if home is None else i32(torch, home)
    e2n_dev = None if e2n is None else i32(torch, e2n)
    eps_dev = None if eps is None else torch.from_numpy(eps.astype(np.float32)).cuda()
    W_in = torch.stack([hz.to_device(ws[e][0], "bf16") for e in range(c.E)])
    W_out = torch.stack([hz.to_device(ws[e][1], "bf16") for e in range(c.E)])

    # --- transposed weights: bit-exact
    W_in_t, W_out_t = torch.empty_like(W_out), torch.empty_like(W_in)
    lm.locmoe_transpose_weights(desc, W_in, W_out, W_in_t, W_out_t)
    torch.cuda.synchronize()
    assert torch.equal(W_in_t, W_in.transpose(1, 2).contiguous())
    assert torch.equal(W_out_t, W_out.transpose(1, 2).contiguous())

    slot_dev, seg_dev, be_dev = i32(torch, ref["slot"]), i32(torch, ref["seg_off"]), i32(torch, ref["buf_expert"])
    rows = c.E * C

    def rows_dev(a, dtype):
        t = torch.zeros(rows, a.shape[1], dtype=hz.torch_dtype(dtype), device="cuda")
        t[:K] = hz.to_device(a, dtype)
        return t

    # --- combine backward on the oracle's out and w
    out_st = store_round(ref["out"], c.dtype)
    w32 = ref["w"].astype(np.float32)
    lm.locmoe_combine_bwd(desc, dy_dev, rows_dev(out_st, c.dtype), slot_dev, torch.from_numpy(w32).cuda(), gb.dout,
                          gb.dw)
    torch.cuda.synchronize()
    dout_ref, dw_ref = bwd.combine_backward(dy, out_st, ref["slot"], w32)
    assert rel_l2(hz.to_host_f32(gb.dout[:K]), dout_ref) <= (1e-2 if c.dtype == "bf16" else 1e-6)
    kept = ref["slot"] >= 0
    bound = np.zeros(T)
    bound[kept] = np.abs(dy[kept].astype(np.float64) * out_st[ref["slot"][kept]]).sum(axis=1)
    got_dw = gb.dw.cpu().numpy()
    assert np.all(np.abs(got_dw - dw_ref) <= 1e-5 * bound + 1e-30)
    assert np.all(got_dw[~kept] == 0.0)

    # --- forward GEMM that keeps Z: H is what the plain entry point gives, Z the pre-activation
    send_dev = rows_dev(ref["send"], c.dtype)
    H_plain = torch.empty_like(b.H)
    lm.locmoe_expert_ffn_in(desc, send_dev, seg_dev, be_dev, W_in, H_plain)
    lm.locmoe_expert_ffn_in_save(desc, send_dev, seg_dev, be_dev, W_in, b.H, gb.Z)
    torch.cuda.synchronize()
    assert torch.equal(b.H[:K], H_plain[:K])
    Z_ref = np.zeros((K, c.h))
    for r, e in enumerate(ref["buf_expert"]):
        a, z = int(ref["seg_off"][r]), int(ref["seg_off"][r + 1])
        if z > a:
            Z_ref[a:z] = ref["send"][a:z].astype(np.float64) @ ws[int(e)][0].astype(np.float64).T
    if K:
        assert rel_l2(hz.to_host_f32(gb.Z[:K]), Z_ref) <= 1e-2

    # --- data gradients on the oracle's dout (rounded to storage) and Z (rounded to bf16)
    dout_st = store_round(ref["dout"], c.dtype)
    Z_b = bf16_round(Z_ref)
    lm.locmoe_expert_ffn_dgrad(desc, rows_dev(dout_st, c.dtype), rows_dev(Z_b, "bf16"), seg_dev, be_dev, W_out_t,
                               W_in_t, gb.dZ, gb.dsend)
    torch.cuda.synchronize()
    dZ_ref = np.zeros((K, c.h)); dsend_ref = np.zeros((K, c.d))
    for r, e in enumerate(ref["buf_expert"]):
        a, z = int(ref["seg_off"][r]), int(ref["seg_off"][r + 1])
        if z > a:
            Wi, Wo = ws[int(e)]
            dZ_ref[a:z] = (dout_st[a:z].astype(np.float64) @ Wo.astype(np.float64)) * bwd.gelu_grad(Z_b[a:z])
            dsend_ref[a:z] = dZ_ref[a:z] @ Wi.astype(np.float64)
    if K:
        assert rel_l2(hz.to_host_f32(gb.dZ[:K]), dZ_ref) <= 1e-2
        assert rel_l2(hz.to_host_f32(gb.dsend[:K]), dsend_ref) <= 1e-2

    # --- weight gradients on the oracle's operands (rounded to what the kernel reads)
    H_b = bf16_round(orc.gelu(Z_ref))
    dZ_b = bf16_round(dZ_ref)
    lm.locmoe_expert_ffn_wgrad(desc, send_dev, rows_dev(H_b, "bf16"), rows_dev(dout_st, c.dtype),
                               rows_dev(dZ_b, "bf16"), seg_dev, be_dev, gb.dW_in, gb.dW_out)
    torch.cuda.synchronize()
    for r, e in enumerate(ref["buf_expert"]):
        a, z = int(ref["seg_off"][r]), int(ref["seg_off"][r + 1])
        gi, go = hz.to_host_f32(gb.dW_in[int(e)]), hz.to_host_f32(gb.dW_out[int(e)])
        if z > a:
            assert rel_l2(gi, dZ_b[a:z].astype(np.float64).T @ ref["send"][a:z].astype(np.float64)) <= 1e-2
            assert rel_l2(go, dout_st[a:z].astype(np.float64).T @ H_b[a:z].astype(np.float64)) <= 1e-2
        else:
            assert not gi.any() and not go.any()

    # --- router backward on the oracle's g (float32), routing and dw
    g_dev = torch.from_numpy(ref["g32"]).cuda()
    cnt_dev = i32(torch, ref["stats"]["cnt"])
    Psum_dev = torch.from_numpy(ref["stats"]["Psum"].astype(np.float32)).cuda()
    dw32 = ref["dw"].astype(np.float32)
    lm.locmoe_route_bwd(desc, g_dev, eps_dev, home_dev, e2n_dev, i32(torch, ref["eid"]), cnt_dev, Psum_dev,
                        torch.from_numpy(dw32).cuda(), gb.coef, gb.dg)
    torch.cuda.synchronize()
    coef_ref = bwd.loss_coefficients(ref["stats"]["cnt"], ref["stats"]["Psum"].astype(np.float32), T, home, e2n_full,
                                     c.N, alpha, mu)
    assert np.allclose(gb.coef.cpu().numpy(), coef_ref, rtol=1e-5, atol=1e-12)
    dg_ref = bwd.route_backward(ref["g32"], eps, relu, ref["eid"], dw32, coef_ref)
    row_scale = np.abs(coef_ref).max() + np.abs(dw32)
    assert np.all(np.abs(gb.dg.cpu().numpy() - dg_ref) <= 2e-5 * row_scale[:, None] + 1e-30)

    # --- dispatch + gate backward on the oracle's dsend (rounded to storage) and dg (float32)
    dsend_st = store_round(ref["dsend"], c.dtype)
    dg32 = ref["dg"].astype(np.float32)
    lm.locmoe_dispatch_bwd(desc, rows_dev(dsend_st, c.dtype), slot_dev, torch.from_numpy(dg32).cuda(), gb.dx)
    torch.cuda.synchronize()
    dx_ref = bwd.dispatch_backward(dsend_st, ref["slot"]) + bwd.gate_backward(dg32, c.d)
    assert rel_l2(hz.to_host_f32(gb.dx), dx_ref) <= (1e-2 if c.dtype == "bf16" else 1e-6)

    # --- end to end on the GPU's own intermediates, against the float64 oracle
    b2, gb2 = lm.alloc_buffers(desc), lm.alloc_grad_buffers(desc)
    lm.forward_train(desc, x_dev, home_dev, e2n_dev, W_in, W_out, b2, gb2, eps=eps_dev)
    lm.backward(desc, dy_dev, home_dev, e2n_dev, W_in_t, W_out_t, b2, gb2, eps=eps_dev)
    torch.cuda.synchronize()
    assert np.array_equal(b2.eid.cpu().numpy(), ref["eid"])
    errs = {"dx": rel_l2(hz.to_host_f32(gb2.dx), ref["dx"])}
    gi = np.stack([ref["grads"][e][0] if e in ref["grads"] else np.zeros((c.h, c.d)) for e in range(c.E)])
    go = np.stack([ref["grads"][e][1] if e in ref["grads"] else np.zeros((c.d, c.h)) for e in range(c.E)])
    errs["dW_in"] = rel_l2(hz.to_host_f32(gb2.dW_in), gi)
    errs["dW_out"] = rel_l2(hz.to_host_f32(gb2.dW_out), go)
    say("      end to end rel-L2: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert v <= 1e-2, (k, v)
    return errs


def test_backward_config1_fp32(env):
    c = wl.CONFIGS[1]
    run_backward_case(env, c, c.C)


def test_backward_config2_bf16(env):
    c = wl.CONFIGS[2]
    run_backward_case(env, c, c.C)


def test_backward_small_odd_shapes(env):
    c = wl.small_config()                     # T=96 d=48 E=6 N=3 h=40: generic kernels everywhere
    run_backward_case(env, c, 9)
    run_backward_case(env, c, 200)
    run_backward_case(env, wl.small_config(dtype="f32"), 5)
    e2n = np.array([2, 0, 1, 1, 0, 2], np.int32)
    eps = np.array([0.3, -0.2, 0.0, 0.5, -1.0, 0.1], np.float32)
    run_backward_case(env, c, 9, eps=eps, e2n=e2n)
    run_backward_case(env, c, 9, relu=False, use_home=False)
    run_backward_case(env, wl.small_config(T=5, E=1, N=1, d=8, h=8), 2)
    run_backward_case(env, wl.small_config(T=300, d=96, E=8, N=2, h=24), 20)      # 12-wide GrAP blocks
    run_backward_case(env, wl.small_config(T=300, d=96, E=8, N=2, h=24, dtype="f32"), 20)


def test_backward_tuned_tiles_with_ragged_segments(env):
    # 256-multiples: the MFMA weight-gradient kernel; segments with ragged tails, empty experts
    run_backward_case(env, wl.small_config(T=3000, d=512, E=8, N=2, h=256, clusters=4), 300)
    run_backward_case(env, wl.small_config(T=2000, d=256, E=16, N=4, h=512, clusters=3), 70)
    run_backward_case(env, wl.small_config(T=1500, d=768, E=12, N=4, h=256, clusters=3), 33)


def run_backward_big(env, c, C, repeats=1):
    """A full-size shape in the benchmark's launch configuration (packed weights, persistent kernels):
    two whole experts against the oracle (their dout, dsend, dW_in, dW_out and the dx rows of their tokens),
    dropped tokens, and properties that hold at any size.  With repeats > 1 the tokens (and their upstream
    gradients) are c's, repeated that many times on the device: a way to reach token counts whose inputs would
    take minutes to draw; the oracle sees the repeated sequence like any other."""
    import dataclasses
    import time
    torch, lm, hz = env
    alpha, mu = wl.ALPHA, wl.MU
    t0 = time.time()
    xb, homeb = wl.hidden_states(c)
    dyb = wl.upstream_grad(c)
    Tb = c.T
    c = dataclasses.replace(c, T=repeats * Tb)
    T = c.T
    home = np.tile(homeb, repeats)

    class Rows:                      # row t of the repeated sequence
        def __init__(self, a):
            self.a = a

        def __getitem__(self, t):
            return self.a[np.asarray(t) % Tb]

    x, dy = Rows(xb), Rows(dyb)
    say(f"[bwd big] cfg={c.cfg} T={T} d={c.d} E={c.E} h={c.h} C={C}; inputs {time.time() - t0:.1f}s")
    e2n_full = np.arange(c.E) // (c.E // c.N)
    g32 = np.tile(orc.gate(xb, c.E).astype(np.float32), (repeats, 1))
    eid, w, p, _ = orc.route(g32)
    st = orc.route_stats(eid, p, home, e2n_full, c.N, alpha, mu)
    s = orc.slots(eid, c.E, C, e2n_full, c.N)
    K = int(s["seg_off"][-1])
    kept_cnt = s["kept"]
    order = np.argsort(kept_cnt)
    cand = [int(order[-1]), int(order[len(order) // 2])]          # the fullest expert and a median one
    if repeats > 1:                                               # ... and the one whose rows come last in the buffers
        last = max(r for r in range(c.E) if s["seg_off"][r + 1] > s["seg_off"][r])
        if int(s["buf_expert"][last]) not in cand:
            cand.append(int(s["buf_expert"][last]))
        assert int(s["seg_off"][last + 1]) * c.d > 2 ** 31
    W_in, W_out, host_w = hz.upload_weights(c, keep=set(cand), progress=lambda a, n: say(f"      weights {a}/{n}"))
    desc = lm.make_desc(T, c.d, c.E, c.N, c.h, C, c.dtype, True, alpha, mu)
    # packed transposes straight from the row-major weights, then the packed forward weights; the row-major copies
    # are released before the gradient buffers are allocated (config 5: 50 GiB per set of weights)
    W_in_tp, W_out_tp = torch.empty_like(W_out), torch.empty_like(W_in)
    lm.locmoe_pack_weights_t(desc, W_in, W_out, W_in_tp, W_out_tp)
    W_in_p, W_out_p = torch.empty_like(W_in), torch.empty_like(W_out)
    lm.locmoe_pack_weights(desc, W_in, W_out, W_in_p, W_out_p)
    torch.cuda.synchronize()
    del W_in, W_out
    torch.cuda.empty_cache()
    desc.w_packed = 1
    b, gb = lm.alloc_buffers(desc), lm.alloc_grad_buffers(desc)
    for t in (b.H, b.out, b.y, gb.Z, gb.dout, gb.dZ, gb.dsend, gb.dx, gb.dW_in, gb.dW_out, gb.dw, gb.dg):
        t.fill_(float("nan"))                 # a row or tile that a kernel skips cannot pass for a result
    x_dev, dy_dev, home_dev = hz.to_device(xb, c.dtype), hz.to_device(dyb, c.dtype), i32(torch, home)
    if repeats > 1:
        x_dev, dy_dev = x_dev.repeat(repeats, 1), dy_dev.repeat(repeats, 1)
    lm.forward_train(desc, x_dev, home_dev, None, W_in_p, W_out_p, b, gb)
    lm.backward(desc, dy_dev, home_dev, None, W_in_tp, W_out_tp, b, gb)
    torch.cuda.synchronize()
    for name in ("dx", "dW_in", "dW_out", "dw", "dg"):          # every element of these is written
        assert not bool(torch.isnan(getattr(gb, name)).any()), name
    for name in ("Z", "dout", "dZ", "dsend"):                   # rows below K written, the rest untouched
        t = getattr(gb, name)
        assert not bool(torch.isnan(t[:K]).any()), name
        assert bool(torch.isnan(t[K:]).all()), name
    say(f"      GPU forward + backward done ({time.time() - t0:.1f}s)")
    assert np.array_equal(b.eid.cpu().numpy(), eid)
    assert np.array_equal(b.slot.cpu().numpy(), s["slot"])
    coef = bwd.loss_coefficients(st["cnt"], st["Psum"], T, home, e2n_full, c.N, alpha, mu)
    assert np.allclose(gb.coef.cpu().numpy(), coef, rtol=1e-4, atol=1e-12)
    rank_of = {int(e): r for r, e in enumerate(s["buf_expert"])}
    for e in cand:
        a, z = int(s["seg_off"][rank_of[e]]), int(s["seg_off"][rank_of[e] + 1])
        toks = s["row_token"][a:z]
        Wi, Wo = host_w[e]
        S = x[toks]
        out_rows = orc.ffn_rows(S, Wi, Wo)
        dO = w[toks][:, None] * dy[toks].astype(np.float64)
        dS, dWi, dWo, _, _ = bwd.ffn_rows_backward(S, Wi, Wo, dO)
        errs = dict(dout=rel_l2(hz.to_host_f32(gb.dout[a:z]), dO), dsend=rel_l2(hz.to_host_f32(gb.dsend[a:z]), dS),
                    dW_in=rel_l2(hz.to_host_f32(gb.dW_in[e]), dWi), dW_out=rel_l2(hz.to_host_f32(gb.dW_out[e]), dWo))
        dw = np.einsum("ij,ij->i", dy[toks].astype(np.float64), out_rows)
        dg = bwd.route_backward(g32[toks], None, True, eid[toks], dw, coef)
        dx_ref = dS + bwd.gate_backward(dg, c.d)
        errs["dx"] = rel_l2(hz.to_host_f32(gb.dx[torch.from_numpy(toks.astype(np.int64)).cuda()]), dx_ref)
        errs["dw"] = rel_l2(gb.dw.cpu().numpy()[toks], dw)
        say(f"      expert {e} ({z - a} rows): " + " ".join(f"{k}={v:.2e}" for k, v in errs.items())
            + f" ({time.time() - t0:.1f}s)")
        for k, v in errs.items():
            assert v <= 1e-2, (e, k, v)
    # dropped tokens: no expert term, dw = 0, only the losses reach the gate
    dropped = np.nonzero(s["slot"] < 0)[0][:256]
    if len(dropped):
        assert not gb.dw.cpu().numpy()[dropped].any()
        dg = bwd.route_backward(g32[dropped], None, True, eid[dropped], np.zeros(len(dropped)), coef)
        got = hz.to_host_f32(gb.dx[torch.from_numpy(dropped.astype(np.int64)).cuda()])
        ref_dx = bwd.gate_backward(dg, c.d)
        assert np.all(np.abs(got - ref_dx) <= 2.0 ** -8 * np.abs(ref_dx) + 2e-5 * np.abs(coef).max() * c.E / c.d)
    # any size: each row of dg sums to zero where no ReLU gate is closed (softmax Jacobian annihilates constants)
    g_all = b.g.cpu().numpy()
    open_rows = np.nonzero((g_all > 0).all(axis=1))[0][:4096]
    dg_rows = gb.dg.cpu().numpy()[open_rows]
    assert np.all(np.abs(dg_rows.sum(axis=1)) <= 1e-5 * np.abs(dg_rows).sum(axis=1) + 1e-12)
    # an expert's weight gradient is zero exactly when it kept no rows
    kept_dev = b.kept.cpu().numpy()
    for grad in (gb.dW_in, gb.dW_out):      # expert by expert: the tensors are tens of GiB at the largest shape
        nz = np.array([bool((grad[e] != 0).any()) for e in range(c.E)])
        assert np.array_equal(nz, kept_dev > 0)


def test_backward_bitwise_repeatable(env):
    """Every backward result element is written once by one lane and every sum runs in a fixed order:
    dx, dW_in and dW_out are bit-identical from run to run, for the row-major and the packed-weight kernels."""
    torch, lm, hz = env
    c = wl.small_config(T=3000, d=512, E=8, N=2, h=256, clusters=4)
    x, home = wl.hidden_states(c)
    dy = wl.upstream_grad(c)
    ws = {e: wl.expert_weights(c, e) for e in range(c.E)}
    W_in = torch.stack([hz.to_device(ws[e][0], "bf16") for e in range(c.E)])
    W_out = torch.stack([hz.to_device(ws[e][1], "bf16") for e in range(c.E)])
    x_dev, dy_dev, home_dev = hz.to_device(x, c.dtype), hz.to_device(dy, c.dtype), i32(torch, home)
    for packed in (False, True):
        desc = lm.make_desc(len(x), c.d, c.E, c.N, c.h, 300, c.dtype, True, 0.3, 0.2)
        W_in_t, W_out_t = torch.empty_like(W_out), torch.empty_like(W_in)
        lm.locmoe_transpose_weights(desc, W_in, W_out, W_in_t, W_out_t)
        Wi, Wo = W_in, W_out
        if packed:
            Wi, Wo = torch.empty_like(W_in), torch.empty_like(W_out)
            lm.locmoe_pack_weights(desc, W_in, W_out, Wi, Wo)
            Wit, Wot = torch.empty_like(W_in_t), torch.empty_like(W_out_t)
            lm.locmoe_pack_weights(desc, W_out_t, W_in_t, Wot, Wit)
            # the one-pass form gives the same bits
            Wit1, Wot1 = torch.zeros_like(Wit), torch.zeros_like(Wot)
            lm.locmoe_pack_weights_t(desc, W_in, W_out, Wit1, Wot1)
            torch.cuda.synchronize()
            assert torch.equal(Wit1.view(torch.int16), Wit.view(torch.int16))
            assert torch.equal(Wot1.view(torch.int16), Wot.view(torch.int16))
            W_in_t, W_out_t = Wit, Wot
            desc.w_packed = 1
        runs = []
        for _ in range(3):
            b, gb = lm.alloc_buffers(desc), lm.alloc_grad_buffers(desc)
            lm.forward_train(desc, x_dev, home_dev, None, Wi, Wo, b, gb)
            lm.backward(desc, dy_dev, home_dev, None, W_in_t, W_out_t, b, gb)
            torch.cuda.synchronize()
            runs.append((gb.dx.clone(), gb.dW_in.clone(), gb.dW_out.clone(), gb.dg.clone()))
        for r in runs[1:]:
            for a, b_ in zip(runs[0], r):
                assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32),
                                   b_.view(torch.int16) if b_.dtype == torch.bfloat16 else b_.view(torch.int32))
        if packed:
            # the packed-weight kernels against the row-major ones: same arithmetic order per output? not promised;
            # the bar between them is the oracle's
            assert rel_l2(hz.to_host_f32(runs[0][0]), hz.to_host_f32(first_dx)) <= 1e-2
        else:
            first_dx = runs[0][0]


def test_backward_expert_count_limits(env):
    # the largest expert count the ABI allows (1-wide GrAP blocks, 16 experts per lane in the router backward)
    run_backward_case(env, wl.small_config(T=700, d=1024, E=1024, N=32, h=8, clusters=7), 2)
    # one node, capacity of a single row: almost every token is dropped and only the losses reach the gate
    run_backward_case(env, wl.small_config(T=257, d=64, E=64, N=1, h=16, clusters=3), 1)
    # a free-form expert-to-node map with more nodes than experts per node, E no multiple of 8
    e2n = (np.arange(12) * 5 % 7).astype(np.int32)
    run_backward_case(env, wl.small_config(T=513, d=96, E=12, N=7, h=24, clusters=4), 11, e2n=e2n)
    # 200 experts (several per lane group, E/4 units not a power of two), wide experts with LDS gate path
    run_backward_case(env, wl.small_config(T=1111, d=1600, E=200, N=8, h=16, clusters=9), 3)


def test_backward_config4_full_size(env):
    c = wl.CONFIGS[4]
    run_backward_big(env, c, c.C)


def test_backward_config5_full_size(env):
    """The largest configuration (128 experts, four of them hot, d = 5120): 16 segments per tile queue in the data
    gradients, 20 x 80 output tiles per expert in the weight gradients."""
    c = wl.CONFIGS[5]
    run_backward_big(env, c, c.C)


def test_backward_element_indices_past_two_to_the_31(env):
    """Maximum sizes: T*d and K*d beyond 2^31 elements (dy, dx, dout, dsend beyond 2^32 bytes): a block of 32 768
    tokens repeated 17 times, experts of up to 24 576 rows (96 row tiles per expert in the grouped GEMMs)."""
    cb = wl.small_config(T=32768, d=4096, E=64, N=8, h=256, clusters=64, zipf=0.3)
    assert 17 * cb.T * cb.d > 2 ** 31
    run_backward_big(env, cb, 24576, repeats=17)


def test_backward_config3_full_size_large_capacity(env):
    """Capacity 2 048 (almost nothing dropped): segments of up to 2 048 rows (many m-tiles per weight tile in the data
    gradients, a hundred steps per tile in the weight gradients), very uneven."""
    run_backward_big(env, wl.CONFIGS[3], 2048)
