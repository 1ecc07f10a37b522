"""How the path shards, checked on one GPU (no collectives): a weight that is stored in row
shards (as under FSDP) is quantised shard by shard with ONE global scale: each shard's amax, the
maximum of those (the 4-byte all-reduce a multi-GPU run would do), the scale, then each shard's
cast.  The codes equal those of the whole tensor quantised at once, and the oracle's."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from helpers import bits, u8, f32

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fmt", [f8.E4M3, f8.E5M2])
@pytest.mark.parametrize("N,K,shards", [(1024, 4096, 8), (3584, 1024, 7), (272, 336, 17)])
def test_shardwise_quantisation_equals_whole_tensor(N, K, shards, fmt):
    g = torch.Generator("cpu")
    g.manual_seed(N + shards)
    W = wl.randn_bf16((N, K), 0.02, 0, generator=g)
    W[N // 3, K // 2] = 0.75                      # one outlier, in one shard only
    Wd = W.cuda()
    rows = N // shards
    assert rows * shards == N and rows % 16 == 0
    ws = f8.new_workspace(N, K)
    # whole tensor
    amax, scale, inv = (torch.empty(1, device="cuda") for _ in range(3))
    q = torch.empty((N, K), dtype=torch.uint8, device="cuda")
    q_t = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    f8.amax_cast(Wd, f8.TENSORWISE, fmt, amax, scale, inv, q, q_t, ws)
    # shard by shard
    shard_amax = torch.empty(shards, device="cuda")
    for i in range(shards):
        f8.amax(Wd[i * rows:(i + 1) * rows], f8.TENSORWISE, shard_amax[i:i + 1], ws)
    global_amax = shard_amax.max().reshape(1)     # stands in for all-reduce(max) over the ranks
    g_scale, g_inv = torch.empty(1, device="cuda"), torch.empty(1, device="cuda")
    f8.scale(global_amax, fmt, g_scale, g_inv)
    qs = torch.empty((N, K), dtype=torch.uint8, device="cuda")
    qs_t = torch.empty((K, N), dtype=torch.uint8, device="cuda")
    for i in range(shards):
        sl = slice(i * rows, (i + 1) * rows)
        f8.cast(Wd[sl], g_scale, f8.TENSORWISE, fmt, qs[sl], qs_t[:, sl])
    torch.cuda.synchronize()
    assert torch.equal(global_amax, amax) and torch.equal(g_scale, scale) and torch.equal(g_inv, inv)
    assert torch.equal(qs, q) and torch.equal(qs_t, q_t)
    a, s, i_, codes = o.amax_cast(bits(W), o.TENSORWISE, fmt)
    assert f32(global_amax)[0] == a[0] and f32(g_scale)[0] == s[0]
    assert np.array_equal(u8(qs), codes) and np.array_equal(u8(qs_t), codes.T)
