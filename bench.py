#!/usr/bin/env python3
"""MoE-layer forward throughput of the LocMoE hot path on one MI355X.

A step = one pass of the whole path (gate -> route -> dispatch -> expert FFN -> combine) over
one batch of seeded synthetic tokens, all inputs resident in HBM.  Workload = the headline
config (T=65536, d=4096 bf16, E=64 in 8 nodes, h=16384, capacity from the Theorem 1 bound).
Prints ONE JSON line with the metric, the roofline of the dominant kernel and the CPU oracle
baseline.  `--config N` selects another of the five configs (diagnostics only).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the two grouped-GEMM kernels at the bench workload come from the tracked rocprofv3 summary
# below (--pmc FETCH_SIZE and WRITE_SIZE, KiB per dispatch).  FETCH_SIZE is scaled by 2.0, the factor the same counter
# needs for a plain 1 GiB copy in the same run; WRITE_SIZE needs none.  The summary records a hash of the kernel
# sources it was taken with: when the sources have changed since, `traffic` is reported as null.
PROFILE = os.path.join(ROOT, "profiles", "bench_config4_kernels_and_hbm_counters.txt")
KERNEL_SOURCES = ("ffn.hip", "common.h", "gelu_coef.h")
FETCH_FACTOR, WRITE_FACTOR = 2.0, 1.0


def kernel_sources_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2401_13920_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def profiled_traffic():
    """{'ffn_in': (fetch KiB, write KiB), 'ffn_out': ...} from the tracked summary, and why not if it cannot be used."""
    import re
    try:
        text = open(PROFILE).read()
    except OSError:
        return None, "no profile summary in the tree"
    m = re.search(r"^# kernel sources sha256/16 .*: ([0-9a-f]{16})", text, re.M)
    if not m:
        return None, "the profile summary does not record the kernel sources it was taken with"
    if m.group(1) != kernel_sources_hash():
        return None, "the profile summary is older than the kernel sources"
    out = {}
    for key, tag in (("ffn_out", "<0>"), ("ffn_in", "<1>")):
        mm = re.search(r"ffn_gemm_dma_persistent" + re.escape(tag) + r".*FETCH_SIZE=\s*([0-9.]+)\s+WRITE_SIZE=\s*([0-9.]+)", text)
        if not mm:
            return None, "the profile summary has no counters for the grouped GEMM"
        out[key] = (float(mm.group(1)), float(mm.group(2)))
    return out, None


HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(c, C, x, home, W_in_dev, W_out_dev, budget_rows=4096):
    """The oracle as it stands, timed on the host: gate, route, losses, slots, dispatch and combine
    at full size; the FFN on the first buffer segments (about `budget_rows` rows) and scaled to
    all kept rows."""
    import numpy as np
    from oracle import locmoe_oracle as orc
    from paper_2401_13920_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    e2n = wl.expert_to_node(c)
    t = {}
    t0 = time.perf_counter(); g = orc.gate(x, c.E); g32 = g.astype(np.float32); t["gate"] = time.perf_counter() - t0
    t0 = time.perf_counter(); eid, w, p, _ = orc.route(g32); orc.route_stats(eid, p, home, e2n, c.N)
    t["route"] = time.perf_counter() - t0
    t0 = time.perf_counter(); s = orc.slots(eid, c.E, C, e2n, c.N); K = int(s["seg_off"][-1])
    send = orc.dispatch(x, s["slot"], K); t["dispatch"] = time.perf_counter() - t0
    # FFN on leading segments
    rows = 0; nseg = 0
    while nseg < c.E and rows < budget_rows:
        rows = int(s["seg_off"][nseg + 1]); nseg += 1
    host_w = {}
    for r in range(nseg):
        e = int(s["buf_expert"][r])
        host_w[e] = (W_in_dev[e].float().cpu().numpy(), W_out_dev[e].float().cpu().numpy())
    t0 = time.perf_counter()
    seg = s["seg_off"][:nseg + 1]
    out_part = orc.expert_ffn(send[:rows], seg, s["buf_expert"][:nseg], lambda e: host_w[e])
    t_ffn_part = time.perf_counter() - t0
    t["ffn"] = t_ffn_part * (K / max(rows, 1))
    out = np.zeros((K, c.d), dtype=np.float64); out[:rows] = out_part
    t0 = time.perf_counter(); orc.combine(out, s["slot"], w); t["combine"] = time.perf_counter() - t0
    total = sum(t.values())
    return {
        "value": c.T / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"gate/route/losses/slots/dispatch/combine at full size (T={c.T}); FFN timed on the first "
                   f"{nseg} buffer segments ({rows} of K={K} rows, {t_ffn_part:.1f}s) and scaled by K/rows"),
        "seconds": {k: round(v, 3) for k, v in t.items()},
    }


def time_backward(lm, hz, wl, torch, np, c, desc, sets, W_in_rm, W_out_rm, W_in, W_out, stream, reps, K):
    """Times the backward path (not part of `value`): the forward that keeps Z, then the backward chain, call by
    call with HIP events on the launch stream.  The transposed (and packed) weights the data gradients read are
    laid out once, outside the timed calls, and their cost is reported separately (`weight_relayout_ms`): it is
    paid once per optimizer step, not per batch."""
    ev = lambda: torch.cuda.Event(enable_timing=True)
    gb = lm.alloc_grad_buffers(desc)
    dy = hz.to_device(wl.upstream_grad(c), c.dtype)
    W_in_t, W_out_t = torch.empty_like(W_out_rm), torch.empty_like(W_in_rm)
    e0, e1 = ev(), ev()
    e0.record(stream)
    if desc.w_packed:
        lm.locmoe_pack_weights_t(desc, W_in_rm, W_out_rm, W_in_t, W_out_t, stream)   # transposed and packed in one pass
    else:
        lm.locmoe_transpose_weights(desc, W_in_rm, W_out_rm, W_in_t, W_out_t, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    relayout = round(e0.elapsed_time(e1), 3)
    names = ["ffn_in_save", "combine_bwd", "dgrad", "wgrad", "route_bwd", "dispatch_bwd"]
    acc = {n: [] for n in names}
    total = []
    for k in range(reps):
        xs, hs, b = sets[k % len(sets)]
        lm.forward(desc, xs, hs, None, W_in, W_out, b, stream=stream)
        evs = [ev() for _ in range(len(names) + 1)]
        evs[0].record(stream)
        lm.locmoe_expert_ffn_in_save_ws(desc, b.send, b.seg_off, b.buf_expert, W_in, b.H, gb.Z, b.ffn_ws,
                                        lm.LOCMOE_FFN_WS_BYTES, stream); evs[1].record(stream)
        lm.locmoe_combine_bwd(desc, dy, b.out, b.slot, b.w, gb.dout, gb.dw, stream); evs[2].record(stream)
        lm.locmoe_expert_ffn_dgrad_ws(desc, gb.dout, gb.Z, b.seg_off, b.buf_expert, W_out_t, W_in_t, gb.dZ, gb.dsend,
                                      b.ffn_ws, lm.LOCMOE_FFN_WS_BYTES, stream); evs[3].record(stream)
        lm.locmoe_expert_ffn_wgrad(desc, b.send, b.H, gb.dout, gb.dZ, b.seg_off, b.buf_expert, gb.dW_in, gb.dW_out,
                                   stream); evs[4].record(stream)
        lm.locmoe_route_bwd(desc, b.g, None, hs, None, b.eid, b.cnt, b.Psum, gb.dw, gb.coef, gb.dg, stream)
        evs[5].record(stream)
        lm.locmoe_dispatch_bwd(desc, gb.dsend, b.slot, gb.dg, gb.dx, stream); evs[6].record(stream)
        torch.cuda.synchronize()
        for i, n in enumerate(names):
            acc[n].append(evs[i].elapsed_time(evs[i + 1]))
        total.append(evs[1].elapsed_time(evs[6]))
    out = {n: round(float(np.median(acc[n])), 4) for n in names}      # medians over the timed iterations
    flops = 2.0 * K * c.d * c.h
    bwd_ms = float(np.median(total))
    return {"ms": out, "backward_ms": round(bwd_ms, 4), "weight_relayout_ms": relayout,
            "dgrad_TFLOPs": round(2 * flops / (out["dgrad"] * 1e-3) / 1e12, 1),
            "wgrad_TFLOPs": round(2 * flops / (out["wgrad"] * 1e-3) / 1e12, 1),
            "wgrad_write_GBps": round(2.0 * c.E * c.d * c.h * 2 / (out["wgrad"] * 1e-3) / 1e9, 1),
            "roofline": {"bound": "mfma", "kernel": "wgrad_dma_kernel (two launches per step)" if desc.w_packed else "wgrad",
                         "achieved": round(2 * flops / (out["wgrad"] * 1e-3) / 1e12, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s",
                         "frac": round(2 * flops / (out["wgrad"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                         "flops_per_launch": flops, "bytes_written_per_launch": c.E * c.d * c.h * 2},
            "note": "backward_ms = combine_bwd .. dispatch_bwd for one batch; ffn_in_save replaces ffn_in in a training forward"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--sets", type=int, default=4, help="rotating input/buffer sets (defeats cache residency)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward-path timings (reported beside the step)")
    ap.add_argument("--no-full-capacity", action="store_true",
                    help="skip the extra FFN timing with every expert at capacity (it launches the same kernels on "
                         "another shape: leave it out when profiling per kernel)")
    ap.add_argument("--capacity", type=int, default=0, help="override C (0 = Theorem 1 bound at the config's delta)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2401_13920_amd import harness as hz, locmoe as lm, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    lm.lib()  # fails loudly if the HIP library is not built
    c = wl.CONFIGS[args.config]
    C = args.capacity or lm.locmoe_capacity(c.T, c.E, c.d, 0.0, c.delta)
    desc = lm.make_desc(c.T, c.d, c.E, c.N, c.h, C, c.dtype, True, wl.ALPHA, wl.MU)
    t0 = time.time()
    x, home = wl.hidden_states(c)
    log(f"[bench] config {c.cfg}: T={c.T} d={c.d} E={c.E} N={c.N} h={c.h} C={C}; inputs {time.time() - t0:.1f}s")
    W_in, W_out, _ = hz.upload_weights(c, progress=lambda a, n: log(f"[bench] weights {a}/{n}"))
    log(f"[bench] weights resident {time.time() - t0:.1f}s")
    W_in_rm, W_out_rm = W_in, W_out          # row-major copies stay for the CPU baseline
    if lm.locmoe_packed_weights_bytes(desc) and c.dtype == "bf16":
        # one-time re-tiling of the static weights (outside the timed region)
        W_in = torch.empty_like(W_in_rm); W_out = torch.empty_like(W_out_rm)
        lm.locmoe_pack_weights(desc, W_in_rm, W_out_rm, W_in, W_out)
        torch.cuda.synchronize()
        desc.w_packed = 1
        log(f"[bench] weights packed {time.time() - t0:.1f}s")
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    x0 = hz.to_device(x, c.dtype)
    # rotating sets: the same tokens rolled by a different offset (distinct memory, same statistics)
    sets = []
    for k in range(args.sets):
        sh = (k * 9973) % c.T
        xs = x0 if k == 0 else torch.roll(x0, sh, 0).contiguous()
        hs = i32(np.roll(home, sh))
        sets.append((xs, hs, lm.alloc_buffers(desc)))
    stream = torch.cuda.current_stream()
    # a plain copy of known size (1 GiB read + 1 GiB written): the calibration kernel for HBM byte counters
    calib = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    calib2 = calib.clone()
    del calib, calib2

    def step(k):
        xs, hs, b = sets[k % len(sets)]
        lm.forward(desc, xs, hs, None, W_in, W_out, b, stream=stream)

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    K = int(sets[0][2].seg_off[-1])

    # per-call durations with HIP events on the launch stream, over the same rotating sets
    names = ["gate", "route", "dispatch", "ffn_in", "ffn_out", "combine"]
    acc = {n: [] for n in names}
    reps = max(args.steps, 5)
    nws = lm.LOCMOE_FFN_WS_BYTES
    for k in range(reps):
        xs, hs, b = sets[k % len(sets)]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]
        ev[0].record(stream)
        lm.locmoe_gate(desc, xs, b.g, stream); ev[1].record(stream)
        lm.locmoe_route(desc, b.g, None, hs, None, b.eid, b.w, b.cnt, b.Psum, b.stats, b.ws, b.ws_bytes, stream)
        ev[2].record(stream)
        lm.locmoe_dispatch(desc, xs, b.eid, None, b.pos, b.slot, b.kept, b.seg_off, b.node_off, b.buf_expert,
                           b.row_token, b.send, b.ws, b.ws_bytes, stream); ev[3].record(stream)
        lm.locmoe_expert_ffn_in_ws(desc, b.send, b.seg_off, b.buf_expert, W_in, b.H, b.ffn_ws, nws, stream)
        ev[4].record(stream)
        lm.locmoe_expert_ffn_out_ws(desc, b.H, b.seg_off, b.buf_expert, W_out, b.out, b.ffn_ws, nws, stream)
        ev[5].record(stream)
        lm.locmoe_combine(desc, b.out, b.slot, b.w, b.y, stream); ev[6].record(stream)
        torch.cuda.synchronize()
        for i, n in enumerate(names):
            acc[n].append(ev[i].elapsed_time(ev[i + 1]))
    ms = {n: float(np.median(acc[n])) for n in names}          # median over the timed iterations
    s = 2 if c.dtype == "bf16" else 4
    alg_bytes = {
        "gate": c.T * c.d * s + c.T * c.E * 4,
        "route": c.T * c.E * 4 + 20 * c.T,
        "dispatch": 2 * K * c.d * s + 8 * c.T,
        "combine": K * c.d * s + c.T * c.d * s + 12 * c.T,
    }
    flops = 2.0 * K * c.d * c.h          # per GEMM launch
    steps_detail = {}
    for n in ("gate", "route", "dispatch", "combine"):
        gbs = alg_bytes[n] / (ms[n] * 1e-3) / 1e9
        steps_detail[n] = {"ms": round(ms[n], 4), "GB/s": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4)}
    for n in ("ffn_in", "ffn_out"):
        tf = flops / (ms[n] * 1e-3) / 1e12
        steps_detail[n] = {"ms": round(ms[n], 4), "TFLOP/s": round(tf, 1),
                           "mfma_frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}
    # the delta estimator of Section 4.1 (not part of the timed step): the gate pass that also writes the
    # block sums of squares, and the cosine histograms / smallest routed cosine
    nb = 64
    xs, hs, b = sets[0]
    q_dev = torch.empty_like(b.g)
    hist = torch.empty(2, c.E, nb, dtype=torch.int32, device="cuda")
    cmin = torch.empty(c.E, dtype=torch.float32, device="cuda")
    dstat = torch.empty(4, dtype=torch.float32, device="cuda")
    est = {"gate_sq": [], "angle_stats": []}
    for k in range(reps):
        xs, hs, b = sets[k % len(sets)]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record(stream)
        lm.locmoe_gate_sq(desc, xs, b.g, q_dev, stream); ev[1].record(stream)
        lm.locmoe_angle_stats(desc, b.g, q_dev, b.eid, 1, nb, None, None, hist[0], hist[1], cmin, dstat, stream)
        ev[2].record(stream)
        torch.cuda.synchronize()
        est["gate_sq"].append(ev[0].elapsed_time(ev[1])); est["angle_stats"].append(ev[1].elapsed_time(ev[2]))
    est_bytes = {"gate_sq": c.T * c.d * s + 2 * c.T * c.E * 4, "angle_stats": 2 * c.T * c.E * 4 + 4 * c.T}
    estimator = {"delta_hat": round(float(dstat[0]), 5), "nbins": nb}
    for n in est:
        t = float(np.median(est[n]))
        estimator[n] = {"ms": round(t, 4), "GB/s": round(est_bytes[n] / (t * 1e-3) / 1e9, 1)}
    # the routers the paper compares with (Section 2, Section 4; not part of the timed step): the dense learned gate
    # of the switch router in place of GrAP, and hash routing in place of gate + route
    Wg = hz.to_device(wl.dense_gate_weight(c), c.dtype)
    keys = i32(wl.token_keys(c))
    cmp_t = {"gate_dense": [], "route_hash": []}
    xs, hs, b = sets[0]
    g_dense = torch.empty_like(b.g); eid_h = torch.empty_like(b.eid); w_h = torch.empty_like(b.w)
    cnt_h = torch.empty_like(b.cnt)
    for k in range(reps):
        xs = sets[k % len(sets)][0]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record(stream)
        lm.locmoe_gate_dense(desc, xs, Wg, g_dense, stream); ev[1].record(stream)
        lm.locmoe_route_hash(desc, keys, 1, eid_h, w_h, cnt_h, stream); ev[2].record(stream)
        torch.cuda.synchronize()
        cmp_t["gate_dense"].append(ev[0].elapsed_time(ev[1])); cmp_t["route_hash"].append(ev[1].elapsed_time(ev[2]))
    t_gd, t_rh = float(np.median(cmp_t["gate_dense"])), float(np.median(cmp_t["route_hash"]))
    gd_bytes = c.T * c.d * s + c.E * c.d * s + c.T * c.E * 4
    comparators = {
        "gate_dense": {"ms": round(t_gd, 4), "GB/s": round(gd_bytes / (t_gd * 1e-3) / 1e9, 1),
                       "hbm_frac": round(gd_bytes / (t_gd * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "TFLOP/s": round(2.0 * c.T * c.d * c.E / (t_gd * 1e-3) / 1e12, 1),
                       "vs_grap_gate_ms": round(ms["gate"], 4)},
        "route_hash": {"ms": round(t_rh, 4), "GB/s": round(12 * c.T / (t_rh * 1e-3) / 1e9, 1),
                       "max_count": int(cnt_h.max()), "min_count": int(cnt_h.min())},
    }
    del Wg, keys, g_dense
    # the two GEMMs with every expert at capacity (K = E*C rows, the shape the roofline target of the FFN is
    # stated for): token rows stand in for the send buffer, so the operands have the statistics of real ones
    full = None
    if desc.w_packed and c.E * C <= c.T and not args.no_full_capacity:
        Kf = c.E * C
        seg_full = torch.arange(c.E + 1, dtype=torch.int32, device="cuda") * C
        be_full = torch.arange(c.E, dtype=torch.int32, device="cuda")
        send_full = sets[0][0][:Kf].contiguous()
        Hf = torch.empty(Kf, c.h, dtype=torch.bfloat16, device="cuda")
        of = torch.empty(Kf, c.d, dtype=send_full.dtype, device="cuda")
        accf = [[], []]
        ws_full = sets[0][2].ffn_ws
        for k in range(reps + 2):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            ev[0].record(stream)
            lm.locmoe_expert_ffn_in_ws(desc, send_full, seg_full, be_full, W_in, Hf, ws_full, nws, stream)
            ev[1].record(stream)
            lm.locmoe_expert_ffn_out_ws(desc, Hf, seg_full, be_full, W_out, of, ws_full, nws, stream)
            ev[2].record(stream)
            torch.cuda.synchronize()
            if k >= 2:
                accf[0].append(ev[0].elapsed_time(ev[1])); accf[1].append(ev[1].elapsed_time(ev[2]))
        ff = 2.0 * Kf * c.d * c.h
        t_in, t_out = float(np.median(accf[0])), float(np.median(accf[1]))
        full = {"K": Kf, "ffn_in_ms": round(t_in, 4), "ffn_out_ms": round(t_out, 4),
                "ffn_in_TFLOPs": round(ff / (t_in * 1e-3) / 1e12, 1),
                "ffn_out_TFLOPs": round(ff / (t_out * 1e-3) / 1e12, 1),
                "mfma_frac_both": round(2 * ff / ((t_in + t_out) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
        del send_full, Hf, of
    backward = None
    if not args.no_backward:
        backward = time_backward(lm, hz, wl, torch, np, c, desc, sets, W_in_rm, W_out_rm, W_in, W_out, stream, reps, K)
    dom = "ffn_in" if ms["ffn_in"] >= ms["ffn_out"] else "ffn_out"
    achieved = flops / (ms[dom] * 1e-3) / 1e12
    kname = "ffn_gemm_dma_persistent" if desc.w_packed else "ffn_gemm_256"
    traffic, traffic_note = None, "the tracked counters are for the config-4 bench workload with packed weights"
    if desc.w_packed and c.cfg == 4 and not args.capacity:
        kib, traffic_note = profiled_traffic()
        if kib:
            traffic = round((kib[dom][0] * FETCH_FACTOR + kib[dom][1] * WRITE_FACTOR) * 1024)
    roofline = {"bound": "mfma", "kernel": f"{kname} ({dom})", "achieved": round(achieved, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": traffic,
                "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE x2.0 + WRITE_SIZE, from profiles/)",
                "flops_per_launch": flops, "ms_per_launch": round(ms[dom], 4)}
    if traffic is None:
        roofline["traffic_note"] = traffic_note

    result = {
        "metric": "MoE-layer fwd tokens/sec (gate+dispatch+FFN+combine); dispatch GB/s vs HBM peak",
        "value": round(c.T / (dt / args.steps), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if c.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config{c.cfg}: T={c.T} d={c.d} E={c.E} nodes={c.N} h={c.h} C={C} "
                               f"(Theorem-1 bound at delta={c.delta}) top-1, K={K} kept rows, {c.T - K} dropped",
                   "rotating_sets": args.sets},
        "dispatch_GBps": steps_detail["dispatch"]["GB/s"],
        "dispatch_hbm_frac": steps_detail["dispatch"]["hbm_frac"],
        "per_step": steps_detail,
        "ffn_every_expert_at_capacity": full,
        "delta_estimator": estimator,
        "comparators": comparators,
        "backward": backward,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle (bounded sample)...")
        result["cpu_baseline"] = cpu_baseline(c, C, x, home, W_in_rm, W_out_rm)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
