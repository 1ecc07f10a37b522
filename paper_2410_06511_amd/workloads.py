"""Seeded synthetic inputs with the shapes of the Llama-3.1 linears.

This module holds no arithmetic of the Float8 method: it only names the
workload shapes and draws random bf16 tensors.  It serves the GPU library, its
tests, the benchmark and the CPU oracle's tests alike, so that both sides see
the same bits.

The tensors stand in for the activations, weights and output gradients of the
paper's Llama 3.1 8B / 70B / 405B training runs (performance section; 70B and
405B at tensor-parallel degree 8, so N or K is the model dimension / 8).  The
training data and checkpoints themselves are not used anywhere.

Recipe: torch.Generator('cpu').manual_seed(seed); randn(fp32) * std -> bf16.
"N(0, s)" means standard deviation s.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import torch


@dataclass(frozen=True)
class Linear:
    name: str
    M: int
    K: int
    N: int

    @property
    def flops(self) -> int:
        """Forward + backward: three GEMMs of 2*M*K*N."""
        return 6 * self.M * self.K * self.N


@dataclass(frozen=True)
class Workload:
    key: str
    config_index: int            # 1-based index into the benchmark's config list
    linears: List[Linear]
    x_std: float = 1.0
    w_std: float = 0.02
    dy_std: float = 1e-3
    x_outlier_frac: float = 0.0  # fraction of X drawn from N(0, x_outlier_std) instead
    x_outlier_std: float = 100.0
    variants: tuple = (("tensorwise", "e4m3"),)  # (granularity, grad format) pairs to run
    note: str = ""
    # Groups of linear indices that read ONE input tensor: the first of a group owns X (and its
    # cast), the others take its X and its fp8 codes.  Empty: every linear has its own X.
    shared_x: tuple = ()

    def x_owner(self, li: int) -> int:
        """Index of the linear whose X (and X codes) linear `li` reads: itself unless it follows in a group."""
        for g in self.shared_x:
            if li in g:
                return g[0]
        return li


def _llama8b(M):
    return [Linear("wq", M, 4096, 4096), Linear("wk", M, 4096, 1024), Linear("wv", M, 4096, 1024),
            Linear("wo", M, 4096, 4096), Linear("w1", M, 4096, 14336), Linear("w3", M, 4096, 14336),
            Linear("w2", M, 14336, 4096)]


WORKLOADS = {
    "single": Workload("single", 1, [Linear("lin", 256, 512, 1024)]),
    "llama8b": Workload("llama8b", 2, _llama8b(8192)),
    "llama70b_tp8": Workload(
        "llama70b_tp8", 3,
        [Linear("w1", 8192, 8192, 3584), Linear("w3", 8192, 8192, 3584),
         Linear("w2", 8192, 3584, 8192), Linear("wq", 8192, 8192, 1024)],
        x_outlier_frac=1e-3, x_outlier_std=100.0,
        variants=(("tensorwise", "e4m3"), ("tensorwise", "e5m2"))),
    "llama405b_tp8": Workload(
        "llama405b_tp8", 4,
        [Linear("w1", 8192, 16384, 6656), Linear("w3", 8192, 16384, 6656),
         Linear("w2", 8192, 6656, 16384), Linear("wq", 8192, 16384, 2048)],
        w_std=0.01, variants=(("tensorwise", "e4m3"), ("rowwise", "e4m3"))),
    # wq, wk, wv read the same activation, and so do w1, w3: their X is one tensor, cast once
    "llama8b_block": Workload("llama8b_block", 5, _llama8b(16384), shared_x=((0, 1, 2), (4, 5)),
                              note="seven linears forward in model order, then backward in reverse; "
                                   "wq / wk / wv share one input (cast once), w1 / w3 another"),
    # The same block with the projections that share an input fused along N: one X cast and one
    # wide GEMM for q|k|v (4096 + 1024 + 1024) and for w1|w3 (2 x 14336).  The fused dY then has
    # ONE tensorwise scale, so results differ from the unfused linears by quantisation noise.
    "llama8b_fused": Workload(
        "llama8b_fused", 6,
        [Linear("wqkv", 16384, 4096, 6144), Linear("wo", 16384, 4096, 4096),
         Linear("w13", 16384, 4096, 28672), Linear("w2", 16384, 14336, 4096)],
        note="llama8b_block with q|k|v and w1|w3 fused along N"),
    # The feed-forward block as a real chain: X -> [w1; w3] -> silu(a) * b -> w2 -> Y and back,
    # each linear's input amax handed over by its producer (the bench runs it with --workload).
    "llama8b_ffn": Workload(
        "llama8b_ffn", 7,
        [Linear("w13", 8192, 4096, 28672), Linear("w2", 8192, 14336, 4096)],
        note="chained feed-forward block; X and the weights are seeded, the intermediate tensors are computed"),
    # One whole Llama 3.1 8B transformer block on one sequence of 8192 tokens (the paper's 8B
    # runs: sequence length 8192, local batch 1): the four Float8 linears (q|k|v and w1|w3 fused)
    # joined by the bf16 operations between them (RMSNorm, rotary embedding, causal attention
    # with 32 query and 8 key/value heads, SiLU gate, residuals), forward and backward.
    "llama8b_layer": Workload(
        "llama8b_layer", 8,
        [Linear("wqkv", 8192, 4096, 6144), Linear("wo", 8192, 4096, 4096),
         Linear("w13", 8192, 4096, 28672), Linear("w2", 8192, 14336, 4096)],
        note="whole transformer block as a chain; x, dOut and the weights are seeded, everything between is computed"),
}
LAYER_SHAPE = {"llama8b_layer": dict(B=1, S=8192, Hq=32, Hkv=8, hd=128, D=4096, H=14336)}


def seed_for(config_index: int, linear_index: int, which: str) -> int:
    """which in {'x','w','dy'}."""
    return 1000 * config_index + 10 * linear_index + {"x": 0, "w": 1, "dy": 2}[which]


def randn_bf16(shape, std: float, seed: int, outlier_frac: float = 0.0,
               outlier_std: float = 100.0, generator: Optional[torch.Generator] = None) -> torch.Tensor:
    """CPU bf16 tensor ~ N(0, std); optionally a sparse mixture of N(0, outlier_std)."""
    g = generator
    if g is None:
        g = torch.Generator("cpu")
        g.manual_seed(seed)
    x = torch.randn(shape, generator=g, dtype=torch.float32)
    x.mul_(std)
    if outlier_frac > 0.0:
        mask = torch.rand(shape, generator=g, dtype=torch.float32) < outlier_frac
        big = torch.randn(shape, generator=g, dtype=torch.float32) * outlier_std
        x = torch.where(mask, big, x)
    return x.to(torch.bfloat16)


def make_linear_inputs(wl: Workload, li: int, M: Optional[int] = None):
    """(X [M,K], W [N,K], dY [M,N]) as CPU bf16 tensors for linear `li` of a workload.
    M overrides the token count (used for reduced-size parity cases)."""
    lin = wl.linears[li]
    m = lin.M if M is None else M
    if wl.key == "single":
        # one generator, draw order X, W, dY
        g = torch.Generator("cpu")
        g.manual_seed(0)
        X = randn_bf16((m, lin.K), wl.x_std, 0, generator=g)
        W = randn_bf16((lin.N, lin.K), wl.w_std, 0, generator=g)
        dY = randn_bf16((m, lin.N), wl.dy_std, 0, generator=g)
        return X, W, dY
    # linears that share their input draw the X of the group's first linear
    X = randn_bf16((m, lin.K), wl.x_std, seed_for(wl.config_index, wl.x_owner(li), "x"),
                   wl.x_outlier_frac, wl.x_outlier_std)
    W = randn_bf16((lin.N, lin.K), wl.w_std, seed_for(wl.config_index, li, "w"))
    dY = randn_bf16((m, lin.N), wl.dy_std, seed_for(wl.config_index, li, "dy"))
    return X, W, dY


def bits(t: torch.Tensor):
    """bf16 CPU tensor -> numpy uint16 view of the same bits."""
    return t.contiguous().view(torch.uint16).numpy()
