"""The library launches only kernels (no allocation, no memset, no host synchronisation), so a caller can record a
whole step into a HIP graph.  Each replay is checked bit for bit against the eager run, with eager work and
synchronisations between the replays."""
import sys

import numpy as np
import pytest

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


def bits(t):
    import torch
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


@pytest.mark.parametrize("packed", [False, True])
def test_training_step_recorded_into_a_graph(env, packed):
    import time
    torch, lm, hz = env
    c = wl.small_config(T=3000, d=512, E=8, N=2, h=256, clusters=4) if packed else wl.CONFIGS[1]
    C = 300 if packed else c.C
    x, home = wl.hidden_states(c)
    dy = wl.upstream_grad(c)
    ws = {e: wl.expert_weights(c, e) for e in range(c.E)}
    W_in = torch.stack([hz.to_device(ws[e][0], "bf16") for e in range(c.E)])
    W_out = torch.stack([hz.to_device(ws[e][1], "bf16") for e in range(c.E)])
    desc = lm.make_desc(len(x), c.d, c.E, c.N, c.h, C, c.dtype, True, 0.3, 0.2)
    W_in_t, W_out_t = torch.empty_like(W_out), torch.empty_like(W_in)
    if packed:
        Wi, Wo = torch.empty_like(W_in), torch.empty_like(W_out)
        lm.locmoe_pack_weights(desc, W_in, W_out, Wi, Wo)
        lm.locmoe_pack_weights_t(desc, W_in, W_out, W_in_t, W_out_t)
        W_in, W_out = Wi, Wo
        desc.w_packed = 1
    else:
        lm.locmoe_transpose_weights(desc, W_in, W_out, W_in_t, W_out_t)
    x_dev, dy_dev = hz.to_device(x, c.dtype), hz.to_device(dy, c.dtype)
    home_dev = torch.from_numpy(home.astype(np.int32)).cuda()
    b, gb = lm.alloc_buffers(desc), lm.alloc_grad_buffers(desc)

    def step():
        lm.forward_train(desc, x_dev, home_dev, None, W_in, W_out, b, gb)
        lm.backward(desc, dy_dev, home_dev, None, W_in_t, W_out_t, b, gb)

    outs = lambda: (b.y, b.stats, gb.dx, gb.dW_in, gb.dW_out)
    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in outs()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for t in outs():
            t.fill_(7 if t.dtype != torch.bfloat16 else 0.5)     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs(), eager):
            assert torch.equal(bits(got), bits(want)), rep
    # what the graph saves on a launch-bound step
    reps = 50
    torch.cuda.synchronize(); t0 = time.perf_counter()
    for _ in range(reps):
        step()
    torch.cuda.synchronize(); t_eager = (time.perf_counter() - t0) / reps
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize(); t_graph = (time.perf_counter() - t0) / reps
    say(f"[graph] packed={packed} T={len(x)}: eager {t_eager * 1e3:.3f} ms per step, graph replay {t_graph * 1e3:.3f} ms")
