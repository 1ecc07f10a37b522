"""A few passes of the attention forward and backward at the Llama 3.1 8B shape (one sequence of
8192 tokens, 32 query and 8 key/value heads of 128) on seeded inputs: the program that the
rocprofv3 counter summaries of the attention kernels are collected on.

    python3 -m paper_2410_06511_amd.attn_profile_workload [passes]
"""
import sys

import torch

from . import f8


def main(passes=3):
    B, S, Hq, Hkv, HD = 1, 8192, 32, 8, 128
    M = B * S
    g = torch.Generator("cpu")
    g.manual_seed(8192)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    qkv = torch.randn((M, (Hq + 2 * Hkv) * HD), generator=g).bfloat16().cuda()
    do = (torch.randn((M, Hq * HD), generator=g) * 0.01).bfloat16().cuda()
    q, k, v = qkv[:, :Hq * HD], qkv[:, Hq * HD:(Hq + Hkv) * HD], qkv[:, (Hq + Hkv) * HD:]
    vt, o = torch.empty((Hkv * HD, M), **bf), torch.empty((M, Hq * HD), **bf)
    qt, kt, dot = torch.empty((Hq * HD, M), **bf), torch.empty((Hkv * HD, M), **bf), torch.empty((Hq * HD, M), **bf)
    lse, delta = torch.empty((Hq, M), device="cuda"), torch.empty((Hq, M), device="cuda")
    dqkv = torch.zeros((M, (Hq + 2 * Hkv) * HD), **bf)
    dq, dk, dv = dqkv[:, :Hq * HD], dqkv[:, Hq * HD:(Hq + Hkv) * HD], dqkv[:, (Hq + Hkv) * HD:]
    ws = torch.empty(f8.sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, HD), dtype=torch.uint8, device="cuda")
    f8.transpose_bf16(v, vt)
    f8.transpose_bf16(q, qt)
    f8.transpose_bf16(k, kt)
    f8.transpose_bf16(do, dot)
    for _ in range(passes):
        f8.sdpa_fwd(q, k, vt, B, S, Hq, Hkv, HD, o, lse)
        f8.sdpa_bwd(q, qt, k, kt, v, o, do, dot, lse, B, S, Hq, Hkv, HD, dq, dk, dv, delta, ws)
    torch.cuda.synchronize()
    print("attention profile workload: %d passes done" % passes)


if __name__ == "__main__":
    main(int(sys.argv[1]) if len(sys.argv) > 1 else 3)
