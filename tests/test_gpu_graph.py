"""The library only enqueues kernels (no allocation, no synchronisation, no memset), so a
forward + backward can be captured into a HIP graph and replayed."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from helpers import bits, u8, f32, assert_gemm_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["dynamic", "delayed", "chained"])
def test_captured_step_replays_like_eager(mode):
    M, K, N = 512, 768, 256
    g = torch.Generator("cpu")
    g.manual_seed(3)
    batches = [(wl.randn_bf16((M, K), 1.0 + i, 0, generator=g), wl.randn_bf16((N, K), 0.02, 0, generator=g),
                wl.randn_bf16((M, N), 1e-3 * (i + 1), 0, generator=g)) for i in range(4)]
    desc = f8.linear_desc(M, K, N)
    ws = f8.new_workspace(1024, 1024)
    X, W, dY = (torch.empty_like(t, device="cuda") for t in batches[0])
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    saved = f8.Saved(M, K, N)
    state = f8.ScalingState(f8.DELAYED, 2) if mode == "delayed" else None
    a_y, a_dx = torch.empty(1, device="cuda"), torch.empty(1, device="cuda")

    def step():
        if mode == "dynamic":
            f8.linear_fwd(desc, X, W, Y, saved, ws)
            f8.linear_bwd(desc, dY, saved, dX, dW, ws)
        elif mode == "delayed":
            f8.linear_fwd_scaled(desc, state, X, W, Y, saved, ws)
            f8.linear_bwd_scaled(desc, state, dY, saved, dX, dW, ws)
        else:
            f8.linear_fwd_chained(desc, X, None, W, Y, a_y, saved, ws)
            f8.linear_bwd_chained(desc, dY, None, saved, dX, a_dx, dW, ws)

    def load(b):
        X.copy_(b[0]), W.copy_(b[1]), dY.copy_(b[2])

    def snapshot():
        torch.cuda.synchronize()
        out = [t.clone() for t in (Y, dX, dW, saved.x.q, saved.w.q, saved.dy.q, saved.x.scale, saved.dy.scale)]
        if mode == "delayed":
            out += [state.hist_x.clone(), state.scale_x.clone(), state.scale_dy.clone()]
        if mode == "chained":
            out += [a_y.clone(), a_dx.clone()]
        return out

    def seed_state():
        if mode == "delayed":
            for h in (state.hist_x, state.hist_w, state.hist_dy):
                h.zero_()
            state.scale_x.fill_(100.0), state.scale_w.fill_(4096.0), state.scale_dy.fill_(2.0 ** 16)

    # eager reference: the four batches in order
    seed_state()
    eager = []
    for b in batches:
        load(b)
        step()
        eager.append(snapshot())

    # capture once (on a side stream of default priority), then replay on every batch
    seed_state()
    load(batches[0])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        step()
    seed_state()                          # capturing does not run the kernels; start the state over
    for i, b in enumerate(batches):
        load(b)
        graph.replay()
        got = snapshot()
        scratch = torch.randn(1 << 20, device="cuda").sum().item()  # unrelated eager work and a sync between replays
        assert np.isfinite(scratch)
        for a, e in zip(got, eager[i]):
            assert torch.equal(a.view(torch.uint8), e.view(torch.uint8)), (mode, i)

    # and the last replay against the oracle
    if mode == "dynamic":
        rY, xq, wq = o.linear_fwd(bits(batches[-1][0]), bits(batches[-1][1]))
        rdX, rdW, dyq = o.linear_bwd(bits(batches[-1][2]), xq, wq)
        assert np.array_equal(u8(saved.x.q), xq.q) and f32(saved.dy.scale)[0] == dyq.scale[0]
        assert_gemm_close(bits(Y), rY), assert_gemm_close(bits(dX), rdX), assert_gemm_close(bits(dW), rdW)
