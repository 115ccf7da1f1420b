"""locmoe_dispatch_static (the dispatch for callers that cannot allocate device memory) against locmoe_dispatch,
through the C ABI: every output bit for bit, on two calls in a row, the second on a smaller input, so that whatever
the first call left in the library's static scratch must not leak into the second."""
import numpy as np
import pytest

from paper_2401_13920_amd import workloads as wl

pytestmark = pytest.mark.gpu

OUTPUTS = ("pos", "slot", "kept", "seg_off", "node_off", "buf_expert")


def both_ways(torch, lm, hz, c, C, T=None, e2n=None):
    x, _ = wl.hidden_states(c, T)
    T = len(x)
    print(f"[no-alloc] T={T} d={c.d} E={c.E} N={c.N} C={C} dtype={c.dtype}", flush=True)
    desc = lm.make_desc(T, c.d, c.E, c.N, c.h, C, c.dtype)
    x_dev = hz.to_device(x, c.dtype)
    # any assignment will do for a dispatch: the lowest index of the largest block mean, computed here with torch
    eid = x_dev.float().view(T, c.E, c.d // c.E).mean(dim=2).argmax(dim=1).to(torch.int32)
    e2n_dev = None if e2n is None else torch.from_numpy(np.ascontiguousarray(e2n, dtype=np.int32)).cuda()
    ref, got = lm.alloc_buffers(desc), lm.alloc_buffers(desc)
    for b in (ref, got):
        for name in OUTPUTS + ("row_token",):
            getattr(b, name).fill_(-7)
        b.send.fill_(float("nan"))
    lm.locmoe_dispatch(desc, x_dev, eid, e2n_dev, ref.pos, ref.slot, ref.kept, ref.seg_off, ref.node_off,
                       ref.buf_expert, ref.row_token, ref.send, ref.ws, ref.ws_bytes)
    lm.locmoe_dispatch_static(desc, x_dev, eid, e2n_dev, got.pos, got.slot, got.kept, got.seg_off, got.node_off,
                              got.buf_expert, got.row_token, got.send)
    torch.cuda.synchronize()
    K = int(ref.seg_off[-1])
    assert 0 < K <= T
    for name in OUTPUTS:
        assert torch.equal(getattr(got, name), getattr(ref, name)), name
    assert torch.equal(got.row_token[:K], ref.row_token[:K])
    bits = torch.int16 if c.dtype == "bf16" else torch.int32
    assert torch.equal(got.send[:K].view(bits), ref.send[:K].view(bits))
    assert torch.equal(got.send[:K].view(bits), x_dev[ref.row_token[:K].long()].view(bits))    # and both are the rows of x
    assert bool(torch.isnan(got.send[K:]).all())                                               # rows >= K untouched
    return K


def test_dispatch_static_matches_dispatch_twice_in_a_row():
    import torch
    from paper_2401_13920_amd import harness as hz, locmoe as lm
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lm.lib()
    # first call: several blocks of 1024 tokens, 128 experts; second call: fewer tokens, fewer experts, a free-form
    # expert-to-node map, fp32 rows
    big = wl.small_config(T=9000, d=1024, E=128, N=16, h=64, clusters=9)
    both_ways(torch, lm, hz, big, 40)
    small = wl.small_config(T=1500, d=96, E=12, N=7, h=24, clusters=4, dtype="f32")
    both_ways(torch, lm, hz, small, 11, e2n=(np.arange(12) * 5 % 7).astype(np.int32))
    # beyond the stated maximum of the static scratch: refused on the host, nothing launched
    over = lm.make_desc(1024 * 257, 1024, 1024, 32, 8, 4, "bf16")
    assert over.E * 257 > 262144
    with pytest.raises(lm.LocMoEError) as err:
        lm.locmoe_dispatch_static(over, 0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000,
                                  0x1000)
    assert err.value.status == lm.LOCMOE_ERR_WORKSPACE
