"""Seeded synthetic inputs shaped like the paper's operator suite (GEMM / BMM / Conv2D from
BERT, GPT-2, ResNet-style layers, paper Sec. 6.1-6.2; the suite's exact shape list is not
printed, so the shapes below stand in for it).

This module draws random numbers and casts them to 16-bit floats.  It holds none of the
method's arithmetic: no products, no sums over a reduction axis.  Both the CPU oracle's tests
and the GPU path's tests call it, so both see the same bit patterns.
"""
from __future__ import annotations

import numpy as np
import torch

BASE_SEED = 20221016

_TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def bits(t: torch.Tensor) -> np.ndarray:
    """The raw 16-bit patterns of an fp16/bf16 CPU tensor, as uint16 (same shape)."""
    assert t.dtype in (torch.float16, torch.bfloat16)
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def uniform(shape, dtype: str, seed: int, lo: float = -1.0, hi: float = 1.0) -> torch.Tensor:
    t = torch.rand(shape, generator=_gen(seed), dtype=torch.float32) * (hi - lo) + lo
    return t.to(_TORCH_DT[dtype])


def normal(shape, dtype: str, seed: int, scale: float = 1.0) -> torch.Tensor:
    t = torch.randn(shape, generator=_gen(seed), dtype=torch.float32) * scale
    return t.to(_TORCH_DT[dtype])


def small_ints(shape, dtype: str, seed: int, lo: int = -2, hi: int = 2) -> torch.Tensor:
    """Integers uniform in {lo..hi}; every product and partial sum stays exactly representable."""
    t = torch.randint(lo, hi + 1, shape, generator=_gen(seed), dtype=torch.int32)
    return t.to(torch.float32).to(_TORCH_DT[dtype])


def softmax_rows(shape, dtype: str, seed: int) -> torch.Tensor:
    """Attention-probability-like rows: softmax over the last axis of N(0,1) logits, then cast."""
    t = torch.randn(shape, generator=_gen(seed), dtype=torch.float32)
    return torch.softmax(t, dim=-1).to(_TORCH_DT[dtype])


def identity(n: int, dtype: str) -> torch.Tensor:
    return torch.eye(n, dtype=torch.float32).to(_TORCH_DT[dtype])


def permutation(n: int, dtype: str, seed: int):
    """Returns (P, perm) with P[i, perm[i]] = 1."""
    perm = torch.randperm(n, generator=_gen(seed))
    p = torch.zeros(n, n, dtype=torch.float32)
    p[torch.arange(n), perm] = 1.0
    return p.to(_TORCH_DT[dtype]), perm.numpy()


# ---- the benchmark configurations (shapes, dtypes, value distributions) ---------------------
# name -> dict(kind, dims, in dtype, out dtype, distributions)
CONFIGS = {
    # correctness-sized GEMM, fp32 output; also run with small integers
    "gemm256": dict(kind="gemm", M=256, N=256, K=256, dtype="f16", out="f32", dist="uniform"),
    "gemm256_int": dict(kind="gemm", M=256, N=256, K=256, dtype="f16", out="f32", dist="ints"),
    # the motivating example of the paper's Fig. 1(b): 2048^3
    "gemm2048": dict(kind="gemm", M=2048, N=2048, K=2048, dtype="f16", out="f16", dist="uniform"),
    # BERT-base self-attention, 8 sequences x 12 heads, sequence 512, head 64
    "bmm_qk": dict(kind="bmm", batch=96, M=512, N=512, K=64, dtype="f16", out="f16",
                   transB=True, dist="attn_qk"),
    "bmm_pv": dict(kind="bmm", batch=96, M=512, N=64, K=512, dtype="f16", out="f16",
                   transB=False, dist="attn_pv"),
    # transformer linear layers at 4096 tokens, and a compute-bound square
    "ffn1": dict(kind="gemm", M=4096, N=3072, K=768, dtype="bf16", out="bf16", dist="uniform"),
    "ffn2": dict(kind="gemm", M=4096, N=768, K=3072, dtype="bf16", out="bf16", dist="uniform"),
    "gemm8192": dict(kind="gemm", M=8192, N=8192, K=8192, dtype="bf16", out="bf16", dist="uniform"),
    # between the two squares, in fp16: one 256 x 256 tile per compute unit
    "gemm4096": dict(kind="gemm", M=4096, N=4096, K=4096, dtype="f16", out="f16", dist="uniform"),
    # the shape the paper names as its best case (small output, long reduction: MM_RN50_FC, Sec. 6.1)
    # and a short-reduction batched matmul of the kind it names as its worst (GPT-2 style Q.K^T)
    "mm_rn50_fc": dict(kind="gemm", M=1024, N=64, K=2048, dtype="f16", out="f16", dist="uniform"),
    "bmm_gpt2_qk": dict(kind="bmm", batch=48, M=1024, N=1024, K=64, dtype="f16", out="f16",
                        transB=True, dist="attn_qk"),
    # ResNet-style 3x3 convolutions, NHWC
    "conv56": dict(kind="conv", N=32, H=56, W=56, C=64, K=64, R=3, S=3, stride=1, pad=1,
                   dtype="f16", out="f16", dist="conv"),
    "conv14": dict(kind="conv", N=32, H=14, W=14, C=256, K=256, R=3, S=3, stride=1, pad=1,
                   dtype="f16", out="f16", dist="conv"),
}


_SEED_ORDER = ["bmm_pv", "bmm_qk", "conv14", "conv56", "ffn1", "ffn2", "gemm2048", "gemm256",
               "gemm256_int", "gemm8192", "mm_rn50_fc", "bmm_gpt2_qk", "gemm4096"]


def _seed(name: str, idx: int) -> int:
    return BASE_SEED + 100 * _SEED_ORDER.index(name) + idx


def make_inputs(name: str, **override):
    """Input tensors (CPU, fp16/bf16) of a named configuration; ``override`` replaces dims
    (used by the tests to shrink a config while keeping its distributions)."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    dt = cfg["dtype"]
    kind = cfg["kind"]
    if kind == "gemm":
        M, N, K = cfg["M"], cfg["N"], cfg["K"]
        if cfg["dist"] == "ints":
            A = small_ints((M, K), dt, _seed(name, 0))
            B = small_ints((K, N), dt, _seed(name, 1))
        else:
            A = uniform((M, K), dt, _seed(name, 0))
            B = uniform((K, N), dt, _seed(name, 1))
        return cfg, A, B
    if kind == "bmm":
        b, M, N, K = cfg["batch"], cfg["M"], cfg["N"], cfg["K"]
        if cfg["dist"] == "attn_qk":        # Q and K both stored [batch, seq, head_dim]
            A = normal((b, M, K), dt, _seed(name, 0), 0.125)
            B = normal((b, N, K), dt, _seed(name, 1), 0.125)
        else:                               # P rows are softmax outputs, V ~ N(0,1)*0.125
            A = softmax_rows((b, M, K), dt, _seed(name, 0))
            B = normal((b, K, N), dt, _seed(name, 1), 0.125)
        return cfg, A, B
    if kind == "conv":
        scale = 1.0 / float(np.sqrt(cfg["R"] * cfg["S"] * cfg["C"]))
        x = normal((cfg["N"], cfg["H"], cfg["W"], cfg["C"]), dt, _seed(name, 0), scale)
        w = normal((cfg["R"], cfg["S"], cfg["C"], cfg["K"]), dt, _seed(name, 1), scale)
        return cfg, x, w
    raise KeyError(kind)
