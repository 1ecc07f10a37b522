"""Host-side logic that needs no GPU: the workload tables, the seeded input recipe and the
benchmark's command line."""
import os
import subprocess
import sys

import numpy as np
import torch

from paper_2410_06511_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_workload_flops_and_shapes():
    total = lambda key: sum(l.flops for l in wl.WORKLOADS[key].linears)
    assert total("single") == 6 * 256 * 512 * 1024
    assert total("llama8b") == 10720238370816                 # 10.72 TFLOP per step
    assert total("llama8b_block") == 2 * total("llama8b")      # the same linears at M = 16384
    assert total("llama8b_fused") == total("llama8b_block")    # fusing along N keeps the work
    assert abs(total("llama405b_tp8") / 1e12 - 17.73) < 0.01                 # w1, w3, w2, wq
    for key, w in wl.WORKLOADS.items():
        for l in w.linears:
            assert l.M % 16 == 0 and l.K % 16 == 0 and l.N % 16 == 0
            if key != "single":
                assert l.M % 128 == 0 and l.K % 256 == 0 and l.N % 128 == 0   # the fast GEMM path
    # tensor-parallel degree 8 slices of the 70B / 405B hidden sizes
    assert [l.N for l in wl.WORKLOADS["llama70b_tp8"].linears] == [28672 // 8, 28672 // 8, 8192, 8192 // 8]
    assert [l.N for l in wl.WORKLOADS["llama405b_tp8"].linears] == [53248 // 8, 53248 // 8, 16384, 16384 // 8]


def test_seeded_inputs_are_reproducible_and_distinct():
    w = wl.WORKLOADS["llama70b_tp8"]
    a = wl.make_linear_inputs(w, 3, M=64)
    b = wl.make_linear_inputs(w, 3, M=64)
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
    c = wl.make_linear_inputs(w, 0, M=64)
    assert not torch.equal(a[2][:, :64].view(torch.int16), c[2][:, :64].view(torch.int16))
    assert wl.seed_for(3, 2, "w") == 3021 and wl.seed_for(5, 0, "dy") == 5002
    X, W, dY = a
    assert X.dtype == torch.bfloat16 and X.shape == (64, 8192) and W.shape == (1024, 8192) and dY.shape == (64, 1024)
    # the activation outliers of this workload: a few entries far outside N(0, 1)
    big = (X.float().abs() > 20).float().mean().item()
    assert 2e-4 < big < 2e-3
    assert abs(W.float().std().item() - 0.02) < 2e-3 and abs(dY.float().std().item() - 1e-3) < 1e-4


def test_small_config_draw_order():
    X, W, dY = wl.make_linear_inputs(wl.WORKLOADS["single"], 0)
    g = torch.Generator("cpu")
    g.manual_seed(0)
    x = torch.randn((256, 512), generator=g, dtype=torch.float32).to(torch.bfloat16)
    assert torch.equal(X.view(torch.int16), x.view(torch.int16))
    assert W.shape == (1024, 512) and dY.shape == (256, 1024)
    assert np.array_equal(wl.bits(X), x.view(torch.uint16).numpy())


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_reads_the_committed_traffic_summary():
    sys.path.insert(0, ROOT)
    import bench
    t, source = bench.committed_traffic()
    assert isinstance(t, int) and 1e8 < t < 5e9 and "revision" not in source.split("as of")[0]
    assert os.path.exists(os.path.join(ROOT, "profiles", bench.TRAFFIC_SUMMARY))


def test_linears_that_share_an_input_draw_the_same_tensor():
    """The 16384-token block: wq / wk / wv read one activation and w1 / w3 another, so their X is
    the owner's tensor bit for bit (and cast once); weights and output gradients stay distinct."""
    w = wl.WORKLOADS["llama8b_block"]
    names = [l.name for l in w.linears]
    assert [names[w.x_owner(i)] for i in range(7)] == ["wq", "wq", "wq", "wo", "w1", "w1", "w2"]
    x0, w0, _ = wl.make_linear_inputs(w, 0, M=32)
    x1, w1, _ = wl.make_linear_inputs(w, 1, M=32)
    x3, _, _ = wl.make_linear_inputs(w, 3, M=32)
    assert torch.equal(x0.view(torch.int16), x1.view(torch.int16)) and not torch.equal(x0.view(torch.int16), x3.view(torch.int16))
    assert w0.shape != w1.shape
    assert all(wl.WORKLOADS[k].shared_x == () for k in ("llama8b", "llama70b_tp8", "llama405b_tp8", "llama8b_fused"))
