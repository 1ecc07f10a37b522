"""One whole transformer block (paper_2410_06511_amd/block.py) stage by stage against the
oracles: every stage is fed the ORACLE's tensors of the stages before it and compared with the
oracle's tensors of this stage, so the wiring of the chain (which buffer feeds which call, pitches
of the q|k|v slices, the saved fp8 state handed from forward to backward) is what is under test;
the element-level accuracy of each operation has its own tests."""
import numpy as np
import pytest
import torch

import oracle as o
from oracle import block_oracle as bo
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from paper_2410_06511_amd.block import TransformerBlock
from helpers import bits, u8, qt_matches

pytestmark = pytest.mark.gpu


def gen(shape, seed, std=1.0):
    g = torch.Generator("cpu")
    g.manual_seed(seed)
    return wl.randn_bf16(shape, std, 0, generator=g)


def to_dev(b):
    return torch.from_numpy(np.ascontiguousarray(b).view(np.int16)).view(torch.bfloat16).cuda()


def close(got_bits, ref_bits, what):
    got, ref = (o.bf16_to_f32(np.asarray(b)).astype(np.float64) for b in (got_bits, ref_bits))
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref)
    assert err.max() <= 1e-2 * np.abs(ref).max() + 1e-30, (what, err.max(), np.abs(ref).max())
    assert err.mean() <= 1e-2 * np.abs(ref).mean() + 1e-30, (what, err.mean(), np.abs(ref).mean())


def oracle_block(x, w, dout, B, S, Hq, Hkv, hd, eps):
    """All tensors of the block, forward and backward, from the oracles (bf16 bits unless noted)."""
    r = {}
    M = B * S
    nq, nk = Hq * hd, Hkv * hd
    r["xn"], r["rstd1"], r["a_xn"] = o.rmsnorm(x, w["g1"], eps)
    r["qkv"], xq_qkv, wq_qkv = o.linear_fwd(r["xn"], w["Wqkv"])
    q, k, v = r["qkv"][:, :nq], r["qkv"][:, nq:nq + nk], r["qkv"][:, nq + nk:]
    r["qr"], r["kr"] = bo.rope(q, S, hd), bo.rope(k, S, hd)
    r["qt"], r["kt"], r["vt"] = bo.transpose(r["qr"]), bo.transpose(r["kr"]), bo.transpose(v)
    r["att"], lse = bo.sdpa(r["qr"], r["kr"], v, B, S, Hq, Hkv, hd)
    r["lse"] = np.ascontiguousarray(lse.transpose(1, 0, 2).reshape(Hq, M))
    r["a_att"] = o.amax(r["att"])
    r["yo"], xq_o, wq_o = o.linear_fwd(r["att"], w["Wo"])
    r["h1"] = bo.add(x, r["yo"])
    r["hn"], r["rstd2"], r["a_hn"] = o.rmsnorm(r["h1"], w["g2"], eps)
    r["ab"], xq_13, wq_13 = o.linear_fwd(r["hn"], w["W13"])
    r["hh"], r["a_hh"] = o.silu_mul(r["ab"])
    r["y2"], xq_2, wq_2 = o.linear_fwd(r["hh"], w["W2"])
    r["out"] = bo.add(r["h1"], r["y2"])
    r["codes"] = {"qkv": (xq_qkv, wq_qkv), "o": (xq_o, wq_o), "13": (xq_13, wq_13), "2": (xq_2, wq_2)}
    # backward
    r["dhh"], r["dW2"], _ = o.linear_bwd(dout, xq_2, wq_2)
    r["dab"], r["a_dab"] = o.silu_mul_bwd(r["ab"], r["dhh"])
    r["dhn"], r["dW13"], _ = o.linear_bwd(r["dab"], xq_13, wq_13)
    dnorm2, r["dg2"] = bo.rmsnorm_bwd(r["h1"], w["g2"], r["dhn"], eps)
    r["dh1"] = bo.add(dout, dnorm2)
    r["datt"], r["dWo"], _ = o.linear_bwd(r["dh1"], xq_o, wq_o)
    r["datt_t"] = bo.transpose(r["datt"])
    r["dqr"], r["dkr"], dv = bo.sdpa_bwd(r["qr"], r["kr"], v, r["datt"], B, S, Hq, Hkv, hd)
    dq, dk = bo.rope(r["dqr"], S, hd, inverse=True), bo.rope(r["dkr"], S, hd, inverse=True)
    r["dqkv"] = np.ascontiguousarray(np.concatenate([dq, dk, dv], axis=1))
    r["dxn"], r["dWqkv"], _ = o.linear_bwd(r["dqkv"], xq_qkv, wq_qkv)
    dnorm1, r["dg1"] = bo.rmsnorm_bwd(x, w["g1"], r["dxn"], eps)
    r["dx"] = bo.add(r["dh1"], dnorm1)
    return r


# what each stage writes (attribute names of TransformerBlock = keys of the oracle's dictionary)
WRITES = {
    "zero the amax cells": [],
    "rmsnorm 1": ["xn", "rstd1", "a_xn"], "linear wq|wk|wv fwd": ["qkv"], "rope q (+ transposed copy)": ["qr", "qt"],
    "rope k (+ transposed copy)": ["kr", "kt"], "transpose v": ["vt"], "attention fwd": ["att", "lse", "a_att"],
    "linear wo fwd": ["yo"], "residual 1": ["h1"], "rmsnorm 2": ["hn", "rstd2", "a_hn"], "linear w1|w3 fwd": ["ab"],
    "silu_mul": ["hh", "a_hh"], "linear w2 fwd": ["y2"], "residual 2": ["out"],
    "linear w2 bwd": ["dhh", "dW2"], "silu_mul bwd": ["dab", "a_dab"], "linear w1|w3 bwd": ["dhn", "dW13"],
    "rmsnorm 2 bwd + residual": ["dh1", "dg2"], "linear wo bwd": ["datt", "dWo"],
    "transpose dO": ["datt_t"], "attention bwd": ["dqr", "dkr"], "rope q bwd": [], "rope k bwd": [],
    "linear wq|wk|wv bwd": ["dxn", "dWqkv"], "rmsnorm 1 bwd + residual": ["dx", "dg1"],
}
EXACT = {"vt", "datt_t"}                      # copies of a tensor that the oracle's has replaced
TRANSPOSED_WITH = {"qt": "qr", "kt": "kr"}    # written by the same call as their untransposed twin
SAVED = {"linear wq|wk|wv fwd": ("s_qkv", "qkv"), "linear wo fwd": ("s_o", "o"), "linear w1|w3 fwd": ("s_13", "13"),
         "linear w2 fwd": ("s_2", "2")}


def compare_then_replace(blk, ref, names, stage):
    for n in names:
        t = getattr(blk, n)
        if t.dtype == torch.bfloat16:
            if n in EXACT:
                assert np.array_equal(bits(t), ref[n]), (stage, n)
            else:
                close(bits(t), ref[n], f"{stage}: {n}")
            if n in TRANSPOSED_WITH:
                assert np.array_equal(bits(t), bits(getattr(blk, TRANSPOSED_WITH[n])).T), (stage, n)
        else:
            got, want = t.cpu().numpy().astype(np.float64), np.asarray(ref[n], dtype=np.float64).reshape(t.shape)
            assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max() + 1e-30, (stage, n)
    for n in names:
        t = getattr(blk, n)
        if t.dtype == torch.bfloat16:
            t.copy_(to_dev(ref[n]))
        else:
            t.copy_(torch.from_numpy(np.asarray(ref[n], dtype=np.float32).reshape(t.shape)))


def test_transformer_block_stage_by_stage():
    B, S, Hq, Hkv, hd, H, eps = 2, 136, 4, 2, 128, 768, 1e-5
    D, M = Hq * hd, B * S
    x, dout = gen((M, D), 1), gen((M, D), 2, 1e-2)
    w = {"g1": gen((D,), 3, 0.3) + 1, "g2": gen((D,), 4, 0.3) + 1, "Wqkv": gen(((Hq + 2 * Hkv) * hd, D), 5, 0.04),
         "Wo": gen((D, D), 6, 0.04), "W13": gen((2 * H, D), 7, 0.04), "W2": gen((D, H), 8, 0.04)}
    w = {k: v.bfloat16() for k, v in w.items()}
    ref = oracle_block(bits(x), {k: bits(v) for k, v in w.items()}, bits(dout), B, S, Hq, Hkv, hd, eps)
    blk = TransformerBlock(B, S, D, H, Hq, Hkv, hd, eps)
    xd, dd, wd = x.cuda(), dout.cuda(), {k: v.cuda() for k, v in w.items()}
    for name, call, _, _ in blk.forward_stages(xd, wd) + blk.backward_stages(xd, wd, dd):
        call()
        torch.cuda.synchronize()
        if name == "rmsnorm 2 bwd + residual":
            # the amax handed to the output projection's backward is exactly that of the values written
            assert blk.a_bwd[0].item() == o.amax(bits(blk.dh1))[0]
            blk.a_bwd[0:1].copy_(torch.from_numpy(o.amax(ref["dh1"])))
        compare_then_replace(blk, ref, WRITES[name], name)
        if name in SAVED:
            # the fp8 state kept for the backward is the oracle's, bit for bit
            saved, key = getattr(blk, SAVED[name][0]), SAVED[name][1]
            xq, wq = ref["codes"][key]
            assert np.array_equal(u8(saved.x.q), xq.q) and np.array_equal(u8(saved.w.q), wq.q), name
            assert qt_matches(saved.x, xq.q.T), name
        if name == "attention bwd":
            # dv is written straight into its slice of dqkv; dq, dk get there through the inverse rope
            nq, nk = Hq * hd, Hkv * hd
            close(bits(blk.dqkv)[:, nq + nk:], ref["dqkv"][:, nq + nk:], "attention bwd: dv")
        if name == "rope k bwd":
            close(bits(blk.dqkv), ref["dqkv"], "dqkv assembled")
            # all three producers (inverse rope of dq and dk, the summed dv) have raised the amax cell
            assert blk.a_bwd[1].item() == o.amax(bits(blk.dqkv))[0]
            blk.dqkv.copy_(to_dev(ref["dqkv"]))
            blk.a_bwd[1:2].copy_(torch.from_numpy(o.amax(ref["dqkv"])))


def test_transformer_block_end_to_end_and_recompute():
    """The chain run straight through gives the same bits as stage by stage on its own tensors, and
    the backward after a recomputed forward (full activation checkpointing) gives the same bits
    as the backward after the kept forward."""
    B, S, Hq, Hkv, hd, H = 1, 272, 2, 1, 128, 512
    D, M = Hq * hd, B * S
    x, dout = gen((M, D), 11).cuda(), gen((M, D), 12, 1e-2).cuda()
    w = {"g1": (gen((D,), 13, 0.3) + 1).bfloat16().cuda(), "g2": (gen((D,), 14, 0.3) + 1).bfloat16().cuda(),
         "Wqkv": gen(((Hq + 2 * Hkv) * hd, D), 15, 0.05).cuda(), "Wo": gen((D, D), 16, 0.05).cuda(),
         "W13": gen((2 * H, D), 17, 0.05).cuda(), "W2": gen((D, H), 18, 0.05).cuda()}
    blk = TransformerBlock(B, S, D, H, Hq, Hkv, hd)
    out = blk.forward(x, w).clone()
    dx = blk.backward(x, w, dout).clone()
    grads = [t.clone() for t in (blk.dWqkv, blk.dWo, blk.dW13, blk.dW2, blk.dg1, blk.dg2)]
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(dx.float()).all()
    # scramble every activation, then backward with recomputation
    for n in ("xn", "qkv", "qr", "kr", "qt", "kt", "vt", "att", "yo", "h1", "hn", "ab", "hh", "y2", "out"):
        getattr(blk, n).fill_(7.0)
    dx2 = blk.backward(x, w, dout, recompute=True)
    torch.cuda.synchronize()
    assert torch.equal(dx.view(torch.int16), dx2.view(torch.int16))
    assert torch.equal(out.view(torch.int16), blk.out.view(torch.int16))
    for a, b in zip(grads, (blk.dWqkv, blk.dWo, blk.dW13, blk.dW2, blk.dg1, blk.dg2)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    # selective recomputation: the outputs of the products and of the attention are kept, the
    # cheap tensors are scrambled and come back
    for n in ("xn", "qr", "qt", "kr", "kt", "vt", "h1", "hn", "hh"):
        getattr(blk, n).fill_(-3.0)
    blk.rstd1.fill_(9.0), blk.rstd2.fill_(9.0)
    dx3 = blk.backward(x, w, dout, recompute="selective")
    torch.cuda.synchronize()
    assert torch.equal(dx.view(torch.int16), dx3.view(torch.int16))
    for a, b in zip(grads, (blk.dWqkv, blk.dWo, blk.dW13, blk.dW2, blk.dg1, blk.dg2)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_transformer_block_delayed_scaling_converges_to_dynamic():
    """Delayed scaling with a history of one step on a constant input: the scale a cast uses is
    then FMAX / amax of the same tensor one step earlier.  The first linear's input does not depend
    on any scale, so from the second step on its scale is the dynamic one; every later stage
    follows one step behind its producer.  After as many steps as there are stages the whole
    block, with the glue fused into the casts, gives the bits of the dynamic block."""
    B, S, Hq, Hkv, hd, H = 1, 272, 2, 1, 128, 512
    D, M = Hq * hd, B * S
    x, dout = gen((M, D), 21).cuda(), gen((M, D), 22, 1e-2).cuda()
    w = {"g1": (gen((D,), 23, 0.3) + 1).bfloat16().cuda(), "g2": (gen((D,), 24, 0.3) + 1).bfloat16().cuda(),
         "Wqkv": gen(((Hq + 2 * Hkv) * hd, D), 25, 0.05).cuda(), "Wo": gen((D, D), 26, 0.05).cuda(),
         "W13": gen((2 * H, D), 27, 0.05).cuda(), "W2": gen((D, H), 28, 0.05).cuda()}
    dyn = TransformerBlock(B, S, D, H, Hq, Hkv, hd)
    dyn.forward(x, w)
    dyn.backward(x, w, dout)
    dl = TransformerBlock(B, S, D, H, Hq, Hkv, hd, scaling="delayed", history_len=1)
    for _ in range(10):
        dl.forward(x, w)
        dl.backward(x, w, dout)
    torch.cuda.synchronize()
    for n in ("out", "dx", "dWqkv", "dWo", "dW13", "dW2", "dg1", "dg2", "att", "dqkv"):
        a, b = getattr(dyn, n), getattr(dl, n)
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), n
    # and the first step, whose scales are the initial ones (1.0), is not the dynamic result
    fresh = TransformerBlock(B, S, D, H, Hq, Hkv, hd, scaling="delayed", history_len=1)
    fresh.forward(x, w)
    torch.cuda.synchronize()
    assert not torch.equal(fresh.out.view(torch.int16), dyn.out.view(torch.int16))



def test_delayed_scaling_recomputed_forward_reproduces_the_first():
    """Activation checkpointing under delayed scaling: the forward that runs again inside the
    backward casts with the scales the first forward used and pushes nothing into the amax
    histories.  Over several steps with changing inputs, a block that recomputes gives the bits
    of one that does not: outputs, gradients, histories and next-step scales."""
    B, S, Hq, Hkv, hd, H = 1, 272, 2, 1, 128, 512
    D, M = Hq * hd, B * S
    w = {"g1": (gen((D,), 33, 0.3) + 1).bfloat16().cuda(), "g2": (gen((D,), 34, 0.3) + 1).bfloat16().cuda(),
         "Wqkv": gen(((Hq + 2 * Hkv) * hd, D), 35, 0.05).cuda(), "Wo": gen((D, D), 36, 0.05).cuda(),
         "W13": gen((2 * H, D), 37, 0.05).cuda(), "W2": gen((D, H), 38, 0.05).cuda()}
    steps = [(gen((M, D), 40 + i, 1.0 + 0.7 * i).cuda(), gen((M, D), 50 + i, 1e-2 * (1 + i)).cuda()) for i in range(4)]
    kept = TransformerBlock(B, S, D, H, Hq, Hkv, hd, scaling="delayed", history_len=3)
    redo = TransformerBlock(B, S, D, H, Hq, Hkv, hd, scaling="delayed", history_len=3)
    names = ("out", "dx", "dWqkv", "dWo", "dW13", "dW2", "dg1", "dg2")
    for x, dout in steps:
        kept.forward(x, w)
        kept.backward(x, w, dout)
        redo.forward(x, w)
        out_first = redo.out.clone()
        for n in ("xn", "qkv", "qr", "kr", "qt", "kt", "vt", "att", "yo", "h1", "hn", "ab", "y2", "out"):
            getattr(redo, n).fill_(7.0)      # every activation is gone: the backward has to rebuild them
        redo.backward(x, w, dout, recompute=True)
        torch.cuda.synchronize()
        assert torch.equal(redo.out.view(torch.int16), out_first.view(torch.int16))
        for n in names:
            assert torch.equal(getattr(kept, n).view(torch.uint8), getattr(redo, n).view(torch.uint8)), n
        for a, b in zip((kept.st_qkv, kept.st_o, kept.st_13, kept.st_2), (redo.st_qkv, redo.st_o, redo.st_13, redo.st_2)):
            for m in ("hist_x", "hist_w", "hist_dy", "scale_x", "scale_w", "scale_dy"):
                assert torch.equal(getattr(a, m), getattr(b, m)), m
