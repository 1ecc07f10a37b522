"""Call sequence of one Llama transformer block, forward and backward, on the C-ABI entry points
(Section 2.1: the TransformerBlock is the unit the paper wraps, shards and recomputes; Section
2.2.4: its linear layers run in Float8, everything between them in bf16).

Buffers and the order of calls only: every step runs in the library's kernels.

    x -> rmsnorm -> [wq|wk|wv] -> rope(q), rope(k) -> causal attention -> wo -> + x = h1
    h1 -> rmsnorm -> [w1|w3] -> silu(a) * b -> w2 -> + h1 = out

scaling="dynamic": the Float8 linears use dynamic tensorwise scaling; where a producer already
knows the amax of what it wrote (rmsnorm, the glue) the consumer's cast takes it instead of a pass
of its own.  scaling="delayed": every scale comes from the amax history of earlier steps, every
cast is a single pass, and the feed-forward glue is fused into the casts of its consumers (h and
dAB are never written).
"""
import torch

from . import f8


class TransformerBlock:
    def __init__(self, B, S, D, H, Hq, Hkv, hd=128, eps=1e-5, theta=500000.0, grad_format=f8.E4M3, device="cuda",
                 scaling="dynamic", history_len=16):
        assert D == Hq * hd and scaling in ("dynamic", "delayed")
        self.delayed, self.gfmt = scaling == "delayed", grad_format
        if self.delayed:
            self.st_qkv, self.st_o, self.st_13, self.st_2 = (f8.ScalingState(f8.DELAYED, history_len, device) for _ in range(4))
            self._replay = None   # static states on the saved scales, for recomputation (made on first use)
        self.B, self.S, self.D, self.H, self.Hq, self.Hkv, self.hd = B, S, D, H, Hq, Hkv, hd
        self.eps, self.theta = eps, theta
        M = self.M = B * S
        self.Nqkv = (Hq + 2 * Hkv) * hd
        bf = dict(dtype=torch.bfloat16, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        E = lambda *shape: torch.empty(shape, **bf)
        self.d_qkv = f8.linear_desc(M, D, self.Nqkv, False, grad_format)
        self.d_o = f8.linear_desc(M, D, D, False, grad_format)
        self.d_13 = f8.linear_desc(M, D, 2 * H, False, grad_format)
        self.d_2 = f8.linear_desc(M, H, D, False, grad_format)
        self.s_qkv, self.s_o = f8.Saved(M, D, self.Nqkv), f8.Saved(M, D, D)
        self.s_13, self.s_2 = f8.Saved(M, D, 2 * H), f8.Saved(M, H, D)
        big = max(M, D, 2 * H, self.Nqkv)
        self.ws = f8.new_workspace(big, big, device)
        # forward activations (all kept: the backward reads them)
        self.xn, self.rstd1, self.a_xn = E(M, D), torch.empty(M, **f32), torch.empty(1, **f32)
        self.qkv = E(M, self.Nqkv)
        self.qr, self.kr = E(M, Hq * hd), E(M, Hkv * hd)                 # rotated q, k
        self.qt, self.kt, self.vt = E(Hq * hd, M), E(Hkv * hd, M), E(Hkv * hd, M)
        self.att, self.lse, self.a_att = E(M, D), torch.empty((Hq, M), **f32), torch.empty(1, **f32)
        self.yo, self.h1 = E(M, D), E(M, D)
        self.hn, self.rstd2, self.a_hn = E(M, D), torch.empty(M, **f32), torch.empty(1, **f32)
        self.ab, self.hh, self.a_hh = E(M, 2 * H), E(M, H), torch.empty(1, **f32)
        self.y2, self.out = E(M, D), E(M, D)
        # backward
        self.dhh, self.dab, self.a_dab = E(M, H), E(M, 2 * H), torch.empty(1, **f32)
        self.dhn, self.dh1 = E(M, D), E(M, D)
        self.datt, self.datt_t = E(M, D), E(D, M)
        self.dqr, self.dkr, self.delta = E(M, Hq * hd), E(M, Hkv * hd), torch.empty((Hq, M), **f32)
        self.att_ws = torch.empty(max(16, f8.sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, hd)), dtype=torch.uint8, device=device)
        self.dqkv = E(M, self.Nqkv)
        self.a_bwd = torch.zeros(2, **f32)   # amax of dh1 and of dqkv, raised by the calls that write them
        self.dxn, self.dx = E(M, D), E(M, D)
        self.dg1, self.dg2 = torch.empty(D, **f32), torch.empty(D, **f32)
        self.dWqkv, self.dWo = E(self.Nqkv, D), E(D, D)
        self.dW13, self.dW2 = E(2 * H, D), E(D, H)

    def _slices(self, t):
        Hq, Hkv, hd = self.Hq, self.Hkv, self.hd
        return t[:, :Hq * hd], t[:, Hq * hd:(Hq + Hkv) * hd], t[:, (Hq + Hkv) * hd:]

    def forward_stages(self, x, w, stream=None, replay=False):
        """w: dict with g1, g2 [D], Wqkv [(Hq + 2 Hkv) hd, D], Wo [D, D], W13 [2 H, D], W2 [D, H] (bf16).
        Returns [(name, call, flops, algorithmic bytes)] in execution order.
        replay (delayed scaling only): the forward run AGAIN inside the backward.  It must
        reproduce the forward whose output fed the loss, so every cast uses the scale that forward
        used (kept next to the codes) and no amax history is touched; the glue is run unfused (h is
        written and cast with the saved scale: the same codes)."""
        s, M, D, H, B, S = self, self.M, self.D, self.H, self.B, self.S
        Hq, Hkv, hd = self.Hq, self.Hkv, self.hd
        q, k, v = self._slices(self.qkv)
        att_flops = 4 * B * S * S * Hq * hd // 2
        if self.delayed and replay:
            if self._replay is None:
                self._replay = tuple(f8.ReplayState(sv) for sv in (s.s_qkv, s.s_o, s.s_13, s.s_2))
            r_qkv, r_o, r_13, r_2 = self._replay
            return [
                ("rmsnorm 1", lambda: f8.rmsnorm(x, w["g1"], s.eps, s.xn, s.rstd1, None, None, stream), 0, 4 * M * D),
                ("linear wq|wk|wv fwd", lambda: f8.linear_fwd_scaled(s.d_qkv, r_qkv, s.xn, w["Wqkv"], s.qkv, s.s_qkv, s.ws, stream),
                 2 * M * D * s.Nqkv, 0),
                ("rope q (+ transposed copy)", lambda: f8.rope(q, S, Hq, hd, s.qr, s.qt, s.theta, False, stream), 0, 6 * M * Hq * hd),
                ("rope k (+ transposed copy)", lambda: f8.rope(k, S, Hkv, hd, s.kr, s.kt, s.theta, False, stream), 0, 6 * M * Hkv * hd),
                ("transpose v", lambda: f8.transpose_bf16(v, s.vt, stream), 0, 4 * M * Hkv * hd),
                ("attention fwd", lambda: f8.sdpa_fwd(s.qr, s.kr, s.vt, B, S, Hq, Hkv, hd, s.att, s.lse, stream), att_flops, 0),
                ("linear wo fwd", lambda: f8.linear_fwd_scaled(s.d_o, r_o, s.att, w["Wo"], s.yo, s.s_o, s.ws, stream), 2 * M * D * D, 0),
                ("residual 1", lambda: f8.add(x, s.yo, s.h1, stream), 0, 6 * M * D),
                ("rmsnorm 2", lambda: f8.rmsnorm(s.h1, w["g2"], s.eps, s.hn, s.rstd2, None, None, stream), 0, 4 * M * D),
                ("linear w1|w3 fwd", lambda: f8.linear_fwd_scaled(s.d_13, r_13, s.hn, w["W13"], s.ab, s.s_13, s.ws, stream),
                 2 * M * D * 2 * H, 0),
                ("silu_mul", lambda: f8.silu_mul(s.ab, s.hh, None, None, stream), 0, 6 * M * H),
                ("linear w2 fwd", lambda: f8.linear_fwd_scaled(s.d_2, r_2, s.hh, w["W2"], s.y2, s.s_2, s.ws, stream), 2 * M * H * D, 0),
                ("residual 2", lambda: f8.add(s.h1, s.y2, s.out, stream), 0, 6 * M * D),
            ]
        if self.delayed:
            return [
                ("rmsnorm 1", lambda: f8.rmsnorm(x, w["g1"], s.eps, s.xn, s.rstd1, None, None, stream), 0, 4 * M * D),
                ("linear wq|wk|wv fwd", lambda: f8.linear_fwd_scaled(s.d_qkv, s.st_qkv, s.xn, w["Wqkv"], s.qkv, s.s_qkv, s.ws, stream),
                 2 * M * D * s.Nqkv, 0),
                ("rope q (+ transposed copy)", lambda: f8.rope(q, S, Hq, hd, s.qr, s.qt, s.theta, False, stream), 0, 6 * M * Hq * hd),
                ("rope k (+ transposed copy)", lambda: f8.rope(k, S, Hkv, hd, s.kr, s.kt, s.theta, False, stream), 0, 6 * M * Hkv * hd),
                ("transpose v", lambda: f8.transpose_bf16(v, s.vt, stream), 0, 4 * M * Hkv * hd),
                ("attention fwd", lambda: f8.sdpa_fwd(s.qr, s.kr, s.vt, B, S, Hq, Hkv, hd, s.att, s.lse, stream), att_flops, 0),
                ("linear wo fwd", lambda: f8.linear_fwd_scaled(s.d_o, s.st_o, s.att, w["Wo"], s.yo, s.s_o, s.ws, stream), 2 * M * D * D, 0),
                ("residual 1", lambda: f8.add(x, s.yo, s.h1, stream), 0, 6 * M * D),
                ("rmsnorm 2", lambda: f8.rmsnorm(s.h1, w["g2"], s.eps, s.hn, s.rstd2, None, None, stream), 0, 4 * M * D),
                ("linear w1|w3 fwd", lambda: f8.linear_fwd_scaled(s.d_13, s.st_13, s.hn, w["W13"], s.ab, s.s_13, s.ws, stream),
                 2 * M * D * 2 * H, 0),
                ("silu_mul fused into the cast of h", lambda: f8.silu_mul_quantise_delayed(s.ab, f8.E4M3, s.st_2.hist_x, s.st_2.scale_x,
                                                                                          s.s_2.x, s.ws, stream), 0, 6 * M * H),
                ("linear w2 fwd (input already quantised)", lambda: f8.linear_fwd_xq(s.d_2, s.st_2, w["W2"], s.y2, s.s_2, s.ws, stream),
                 2 * M * H * D, 0),
                ("residual 2", lambda: f8.add(s.h1, s.y2, s.out, stream), 0, 6 * M * D),
            ]
        return [
            ("rmsnorm 1", lambda: f8.rmsnorm(x, w["g1"], s.eps, s.xn, s.rstd1, s.a_xn, s.ws, stream), 0, 4 * M * D),
            ("linear wq|wk|wv fwd", lambda: f8.linear_fwd_chained(s.d_qkv, s.xn, s.a_xn, w["Wqkv"], s.qkv, None, s.s_qkv, s.ws, stream),
             2 * M * D * s.Nqkv, 0),
            ("rope q (+ transposed copy)", lambda: f8.rope(q, S, Hq, hd, s.qr, s.qt, s.theta, False, stream), 0, 6 * M * Hq * hd),
            ("rope k (+ transposed copy)", lambda: f8.rope(k, S, Hkv, hd, s.kr, s.kt, s.theta, False, stream), 0, 6 * M * Hkv * hd),
            ("transpose v", lambda: f8.transpose_bf16(v, s.vt, stream), 0, 4 * M * Hkv * hd),
            ("attention fwd", lambda: f8.sdpa_fwd(s.qr, s.kr, s.vt, B, S, Hq, Hkv, hd, s.att, s.lse, stream, s.a_att), att_flops, 0),
            ("linear wo fwd", lambda: f8.linear_fwd_chained(s.d_o, s.att, s.a_att, w["Wo"], s.yo, None, s.s_o, s.ws, stream), 2 * M * D * D, 0),
            ("residual 1", lambda: f8.add(x, s.yo, s.h1, stream), 0, 6 * M * D),
            ("rmsnorm 2", lambda: f8.rmsnorm(s.h1, w["g2"], s.eps, s.hn, s.rstd2, s.a_hn, s.ws, stream), 0, 4 * M * D),
            ("linear w1|w3 fwd", lambda: f8.linear_fwd_chained(s.d_13, s.hn, s.a_hn, w["W13"], s.ab, None, s.s_13, s.ws, stream),
             2 * M * D * 2 * H, 0),
            ("silu_mul", lambda: f8.silu_mul(s.ab, s.hh, s.a_hh, s.ws, stream), 0, 6 * M * H),
            ("linear w2 fwd", lambda: f8.linear_fwd_chained(s.d_2, s.hh, s.a_hh, w["W2"], s.y2, None, s.s_2, s.ws, stream),
             2 * M * H * D, 0),
            ("residual 2", lambda: f8.add(s.h1, s.y2, s.out, stream), 0, 6 * M * D),
        ]

    def backward_stages(self, x, w, dout, stream=None):
        s, M, D, H, B, S = self, self.M, self.D, self.H, self.B, self.S
        Hq, Hkv, hd = self.Hq, self.Hkv, self.hd
        q, k, v = self._slices(self.qkv)
        dq, dk, dv = self._slices(self.dqkv)
        att_flops = 4 * B * S * S * Hq * hd // 2
        if self.delayed:
            ffn = [
                ("linear w2 bwd", lambda: f8.linear_bwd_scaled(s.d_2, s.st_2, dout, s.s_2, s.dhh, s.dW2, s.ws, stream), 4 * M * H * D, 0),
                ("silu_mul bwd fused into the cast of dAB", lambda: f8.silu_mul_bwd_quantise_delayed(
                    s.ab, s.dhh, s.gfmt, s.st_13.hist_dy, s.st_13.scale_dy, s.s_13.dy, s.ws, stream), 0, 10 * M * H),
                ("linear w1|w3 bwd (gradient already quantised)", lambda: f8.linear_bwd_dyq(s.d_13, s.s_13, s.dhn, s.dW13, stream),
                 4 * M * D * 2 * H, 0),
            ]
            lin_o = lambda: f8.linear_bwd_scaled(s.d_o, s.st_o, s.dh1, s.s_o, s.datt, s.dWo, s.ws, stream)
            lin_qkv = lambda: f8.linear_bwd_scaled(s.d_qkv, s.st_qkv, s.dqkv, s.s_qkv, s.dxn, s.dWqkv, s.ws, stream)
            a_dh1 = a_dqkv = None
        else:
            ffn = [
                ("linear w2 bwd", lambda: f8.linear_bwd(s.d_2, dout, s.s_2, s.dhh, s.dW2, s.ws, stream), 4 * M * H * D, 0),
                ("silu_mul bwd", lambda: f8.silu_mul_bwd(s.ab, s.dhh, s.dab, s.a_dab, s.ws, stream), 0, 10 * M * H),
                ("linear w1|w3 bwd", lambda: f8.linear_bwd_chained(s.d_13, s.dab, s.a_dab, s.s_13, s.dhn, None, s.dW13, s.ws, stream),
                 4 * M * D * 2 * H, 0),
            ]
            # the amax of dh1 and of dqkv come from the calls that write them
            lin_o = lambda: f8.linear_bwd_chained(s.d_o, s.dh1, s.a_bwd[0:1], s.s_o, s.datt, None, s.dWo, s.ws, stream)
            # (the attention backward reports the amax of dv only where it sums the shares of grouped heads)
            a_dh1, a_dqkv = s.a_bwd[0:1], (s.a_bwd[1:2] if Hq > Hkv else None)
            if a_dqkv is not None:
                lin_qkv = lambda: f8.linear_bwd_chained(s.d_qkv, s.dqkv, a_dqkv, s.s_qkv, s.dxn, None, s.dWqkv, s.ws, stream)
            else:
                lin_qkv = lambda: f8.linear_bwd(s.d_qkv, s.dqkv, s.s_qkv, s.dxn, s.dWqkv, s.ws, stream)
        def zero_amax():
            if stream is None or stream == torch.cuda.current_stream():
                s.a_bwd.zero_()
            else:
                with torch.cuda.stream(stream):
                    s.a_bwd.zero_()

        return [("zero the amax cells", zero_amax, 0, 0)] + ffn + [
            ("rmsnorm 2 bwd + residual", lambda: f8.rmsnorm_bwd_add(s.h1, w["g2"], s.rstd2, s.dhn, dout, s.dh1, s.dg2, s.ws, stream, a_dh1),
             0, 12 * M * D),
            ("linear wo bwd", lin_o, 4 * M * D * D, 0),
            ("transpose dO", lambda: f8.transpose_bf16(s.datt, s.datt_t, stream), 0, 4 * M * D),
            ("attention bwd", lambda: f8.sdpa_bwd(s.qr, s.qt, s.kr, s.kt, v, s.att, s.datt, s.datt_t, s.lse, B, S, Hq, Hkv, hd,
                                                  s.dqr, s.dkr, dv, s.delta, s.att_ws, stream, a_dqkv),
             5 * att_flops // 2, 0),
            ("rope q bwd", lambda: f8.rope(s.dqr, S, Hq, hd, dq, None, s.theta, True, stream, a_dqkv), 0, 4 * M * Hq * hd),
            ("rope k bwd", lambda: f8.rope(s.dkr, S, Hkv, hd, dk, None, s.theta, True, stream, a_dqkv), 0, 4 * M * Hkv * hd),
            ("linear wq|wk|wv bwd", lin_qkv, 4 * M * D * s.Nqkv, 0),
            ("rmsnorm 1 bwd + residual", lambda: f8.rmsnorm_bwd_add(x, w["g1"], s.rstd1, s.dxn, s.dh1, s.dx, s.dg1, s.ws, stream),
             0, 12 * M * D),
        ]

    def forward(self, x, w, stream=None):
        for _, call, _, _ in self.forward_stages(x, w, stream):
            call()
        return self.out

    # what selective recomputation runs again: everything the backward reads that is not the output
    # of a matrix product or of the attention (those are kept, as are the fp8 codes of the linears)
    SELECTIVE = ("rmsnorm 1", "rope q (+ transposed copy)", "rope k (+ transposed copy)", "residual 1", "rmsnorm 2")

    def backward(self, x, w, dout, stream=None, recompute=False):
        """recompute (Section 2.2.1, activation checkpointing):
        True / "full": run the whole forward again first; the backward then depends on x and the
        weights only (and, under delayed scaling, on the scales the first forward used, which
        stay next to the fp8 codes: the second forward casts with them and leaves the amax
        histories alone).
        "selective": keep the outputs of the matrix products and of the attention (and the fp8
        codes saved by the linears) and run again only the cheap operations whose results the
        backward reads: the normalisation statistics, the rotated q and k with their transposed
        copies, and the first residual sum."""
        if recompute == "selective":
            for name, call, _, _ in self.forward_stages(x, w, stream):
                if name in self.SELECTIVE:
                    call()
        elif recompute:
            for _, call, _, _ in self.forward_stages(x, w, stream, replay=self.delayed):
                call()
        for _, call, _, _ in self.backward_stages(x, w, dout, stream):
            call()
        return self.dx
