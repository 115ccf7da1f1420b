"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, its scalar capacity formulas agree with the oracle (scipy's incomplete beta
vs the library's own continued fraction), and every argument error is caught before a launch."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from oracle import locmoe_oracle as orc
from paper_2401_13920_amd import locmoe as lm
from paper_2401_13920_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "locmoe.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(locmoe_[a-z_0-9]+)\s*\(", src)))


def test_library_loads_and_exports_declared_symbols():
    L = lm.lib()
    names = declared_symbols()
    assert set(names) == set(lm.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert lm.status_string(0) == "ok"
    seen = {lm.status_string(s) for s in range(-5, 1)}
    assert len(seen) == 6 and "unknown status" not in seen
    assert lm.status_string(-99) == "unknown status"


def test_p_delta_matches_oracle_and_closed_forms():
    for d, delta in [(3, 0.25), (2, 0.5), (128, 0.251), (1024, 0.1142), (4096, 0.065), (5120, 0.0603), (4096, 0.03),
                     (64, 0.0), (64, 1.0), (4096, 0.2)]:
        a, b = lm.locmoe_p_delta(d, delta), orc.p_delta(d, delta)
        assert a == pytest.approx(b, rel=1e-9, abs=2e-16)   # the literal 1 - I form cancels below 1e-16
    assert lm.locmoe_p_delta(3, 0.3) == pytest.approx(0.7, abs=1e-13)
    assert lm.locmoe_p_delta(2, 0.5) == pytest.approx(2 / math.pi * math.acos(0.5), abs=1e-13)


def test_capacity_min_and_capacity_match_oracle():
    forms = {0: "exact", 1: "erfc", 2: "exp"}
    for c in wl.CONFIGS.values():
        for delta in (c.delta, wl.PAPER_DELTA):
            for f, name in forms.items():
                assert lm.locmoe_capacity_min(c.E, c.d, delta, f) == pytest.approx(orc.ec_min(c.E, c.d, delta, name),
                                                                                   rel=1e-9)
            for cf in (0.0, 1.0, 1.25, 2.0):
                assert lm.locmoe_capacity(c.T, c.E, c.d, cf, delta) == orc.capacity(c.T, c.E, c.d, cf, delta)
        assert lm.locmoe_capacity(c.T, c.E, c.d, 0.0, c.delta) == c.C
    assert lm.locmoe_capacity(100, 8, 64, 0.0, 0.999) == 100
    # the empirical capacity is a plain ceiling of the exact product, the capacity factor read as a decimal; the
    # library forms it in integers from the shortest decimal of the double, the oracle in rational arithmetic
    assert lm.locmoe_capacity(100, 10, 4096, 1.1, 0.01) == 11
    assert lm.locmoe_capacity(32768, 32, 4096, math.nextafter(1.25, 2.0), 0.01) == 1281
    rng = np.random.default_rng(11)
    for _ in range(3000):
        T = int(rng.integers(1, 2 ** 31 - 1)) if rng.random() < 0.3 else int(rng.integers(1, 200000))
        E = int(rng.integers(1, 1025))
        cf = [round(float(rng.uniform(0.01, 4.0)), int(rng.integers(1, 6))), float(rng.uniform(1e-12, 2000.0)),
              float(np.nextafter(rng.integers(1, 9) / 4.0, 9.0)), 10.0 ** float(rng.integers(-12, 12))][int(rng.integers(0, 4))]
        if cf > 0:
            assert lm.locmoe_capacity(T, E, 4096, cf, 0.01) == orc.capacity(T, E, 4096, cf, 0.01), (T, E, cf)
    assert math.isinf(lm.locmoe_capacity_min(8, 4096, 0.9, 1))


def _status(fn, *a):
    try:
        fn(*a)
    except lm.LocMoEError as e:
        return e.status
    return 0


def test_scalar_argument_errors():
    L = lm.lib()
    out = C.c_double()
    assert L.locmoe_capacity_min(8, 128, 0.1, 1, None) == lm.LOCMOE_ERR_NULL
    assert L.locmoe_capacity_min(0, 128, 0.1, 1, C.byref(out)) == lm.LOCMOE_ERR_SHAPE
    assert L.locmoe_capacity_min(8, 128, 0.0, 1, C.byref(out)) == lm.LOCMOE_ERR_ARG
    assert L.locmoe_capacity_min(8, 128, 1.0, 1, C.byref(out)) == lm.LOCMOE_ERR_ARG
    assert L.locmoe_capacity_min(8, 128, float("nan"), 1, C.byref(out)) == lm.LOCMOE_ERR_ARG
    assert L.locmoe_capacity_min(8, 128, 0.1, 3, C.byref(out)) == lm.LOCMOE_ERR_ARG
    ci = C.c_int32()
    assert L.locmoe_capacity(0, 8, 128, 1.0, 0.1, C.byref(ci)) == lm.LOCMOE_ERR_SHAPE
    assert L.locmoe_capacity(64, 8, 128, -1.0, 0.1, C.byref(ci)) == lm.LOCMOE_ERR_ARG
    assert L.locmoe_capacity(64, 8, 128, 1.0, 0.1, None) == lm.LOCMOE_ERR_NULL
    assert L.locmoe_p_delta(1, 0.1, C.byref(out)) == lm.LOCMOE_ERR_SHAPE
    assert L.locmoe_p_delta(8, 1.5, C.byref(out)) == lm.LOCMOE_ERR_ARG


def bad_packed_desc(lm, good):
    return lm.make_desc(**dict(good, w_packed=True))   # shape not packable


def zero_c_desc(lm, good):
    return lm.make_desc(**dict(good, Cap=0))


def test_descriptor_validation_without_gpu():
    good = dict(T=64, d=64, E=8, N=2, h=32, Cap=4)
    assert lm.locmoe_workspace_bytes(lm.make_desc(**good)) > 0
    bad = [dict(good, T=0), dict(good, d=60), dict(good, d=68), dict(good, E=0), dict(good, E=2048, d=2048),
           dict(good, N=0), dict(good, N=16), dict(good, h=12), dict(good, Cap=0)]
    for kw in bad:
        assert lm.locmoe_workspace_bytes(lm.make_desc(**kw)) == 0, kw
    d = lm.make_desc(**good)
    d.x_dtype = 7
    assert lm.locmoe_workspace_bytes(d) == 0
    # device entry points validate before launching anything: fake non-NULL addresses are never touched
    p = 0x1000
    dsc = lm.make_desc(**dict(good, d=60))
    assert _status(lm.locmoe_gate, dsc, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    dsc = lm.make_desc(**good)
    assert _status(lm.locmoe_gate, dsc, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_gate_sq, dsc, p, p, None, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_gate_sq, lm.make_desc(**dict(good, d=60)), p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_angle_stats, dsc, p, p, None, 1, 8, None, None, p, p, p, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_angle_stats, dsc, p, p, p, 1, 8, None, None, p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_angle_stats, dsc, p, p, p, 1, 0, None, None, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_angle_stats, dsc, p, p, p, 1, 1 << 20, None, None, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_route, dsc, p, None, None, None, p, p, p, p, p, None, 0, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_route, dsc, p, None, None, None, p, p, p, p, p, p, 16, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_route, dsc, p, None, None, None, None, p, p, p, p, p, 1 << 20, 0) == lm.LOCMOE_ERR_NULL
    odd = lm.make_desc(**dict(good, N=3))          # default node map needs E % N == 0
    assert _status(lm.locmoe_route, odd, p, None, None, None, p, p, p, p, p, p, 1 << 20, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_dispatch, odd, p, p, None, p, p, p, p, p, p, p, p, p, 1 << 20, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_dispatch, dsc, p, p, None, p, p, p, p, p, p, p, p, None, 0, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_dispatch, dsc, p, None, None, p, p, p, p, p, p, p, p, p, 1 << 20, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_dispatch_static, odd, p, p, None, p, p, p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_dispatch_static, dsc, p, p, None, p, None, p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_NULL
    too_big = lm.make_desc(T=1024 * 257, d=1024, E=1024, N=32, h=8, Cap=4)   # 263 168 counts > the static scratch
    assert _status(lm.locmoe_dispatch_static, too_big, p, p, None, p, p, p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn, dsc, p, p, p, p, None, p, p, 0) == lm.LOCMOE_ERR_NULL
    n_ws = lm.LOCMOE_FFN_WS_BYTES
    assert _status(lm.locmoe_expert_ffn_ws, dsc, p, p, p, p, p, p, p, None, n_ws, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_ws, dsc, p, p, p, p, p, p, p, p, n_ws - 1, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_ws, dsc, p, p, p, p, p, p, p, p + 2, n_ws, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_ws, dsc, p, p, p, p, None, p, p, p, n_ws, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_in_ws, dsc, p, p, p, p, p, None, n_ws, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_in_ws, dsc, None, p, p, p, p, p, n_ws, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_out_ws, dsc, p, p, p, p, p, p, 0, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_out_ws, bad_packed_desc(lm, good), p, p, p, p, p, p, n_ws, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_expert_ffn_in_save_ws, dsc, p, p, p, p, p, None, p, n_ws, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_in_save_ws, dsc, p, p, p, p, p, p, None, n_ws, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_dgrad_ws, dsc, p, p, p, p, p, p, p, p, None, n_ws, 0) == lm.LOCMOE_ERR_WORKSPACE
    assert _status(lm.locmoe_expert_ffn_dgrad_ws, dsc, p, p, p, p, p, p, p, None, p, n_ws, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_gate_dense, dsc, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_gate_dense, lm.make_desc(**dict(good, d=60)), p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_route_hash, dsc, None, 3, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_route_hash, lm.make_desc(**dict(good, E=0)), None, 3, p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_combine, dsc, p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_combine_bwd, dsc, p, p, p, p, p, None, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_combine_bwd, zero_c_desc(lm, good), p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_route_bwd, dsc, p, None, None, None, p, p, p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_route_bwd, odd, p, None, None, None, p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_dispatch_bwd, dsc, p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_in_save, dsc, p, p, p, p, p, None, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_in_save, bad_packed_desc(lm, good), p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_transpose_weights, dsc, p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_pack_weights_t, dsc, p, p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_pack_weights_t, lm.make_desc(T=64, d=512, E=8, N=2, h=256, Cap=4), p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_dgrad, dsc, p, p, p, p, p, p, p, None, 0) == lm.LOCMOE_ERR_NULL
    assert _status(lm.locmoe_expert_ffn_dgrad, bad_packed_desc(lm, good), p, p, p, p, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_expert_ffn_wgrad, dsc, p, p, p, p, p, p, None, p, 0) == lm.LOCMOE_ERR_NULL
    # packed weights need 256-multiples of d and h and bf16 activations
    assert lm.locmoe_packed_weights_bytes(dsc) == 0
    big = lm.make_desc(T=64, d=512, E=8, N=2, h=256, Cap=4)
    assert lm.locmoe_packed_weights_bytes(big) == 8 * 512 * 256 * 2
    assert _status(lm.locmoe_pack_weights, dsc, p, p, p, p, 0) == lm.LOCMOE_ERR_SHAPE
    assert _status(lm.locmoe_pack_weights, big, p, None, p, p, 0) == lm.LOCMOE_ERR_NULL
    bad_packed = lm.make_desc(**dict(good, w_packed=True))
    assert _status(lm.locmoe_expert_ffn_in, bad_packed, p, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    assert _status(lm.locmoe_expert_ffn_out, bad_packed, p, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG
    zero_c = lm.make_desc(**dict(good, Cap=0))
    assert _status(lm.locmoe_combine, zero_c, p, p, p, p, 0) == lm.LOCMOE_ERR_ARG


def test_workspace_size_covers_both_users():
    for c in wl.CONFIGS.values():
        d = lm.make_desc(c.T, c.d, c.E, c.N, c.h, c.C, c.dtype)
        need_route = 512 * (c.E * 8 + c.N * 4 + 4)
        need_disp = -(-c.T // 1024) * c.E * 4
        assert lm.locmoe_workspace_bytes(d) >= max(need_route, need_disp)
