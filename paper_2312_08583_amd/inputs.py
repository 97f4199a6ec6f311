"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws random fp16
tensors with the shapes and value distributions of the workloads (LLaMA-shaped
linear layers; the paper's kernel experiment uses LLaMA feed-forward shapes,
Section 5.3 / Appendix B).  Real checkpoints are neither available nor needed.

  weights ...... fp16( N(0, sigma^2) ), optionally with a Bernoulli(outlier_frac)
                 mask of entries multiplied by outlier_mult
  activations .. fp16( N(0, 1) )
"""
from typing import Dict, List, Tuple

import torch

BASE_SEED = 231208583


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def weight(N: int, K: int, seed: int, sigma: float = 0.02, outlier_frac: float = 0.0,
           outlier_mult: float = 10.0, device="cpu") -> torch.Tensor:
    """fp16 [N,K] weight with optional sparse outliers."""
    g = _gen(seed, device)
    w = torch.randn((N, K), generator=g, device=device, dtype=torch.float32) * sigma
    if outlier_frac > 0.0:
        mask = torch.rand((N, K), generator=g, device=device, dtype=torch.float32) < outlier_frac
        w = torch.where(mask, w * outlier_mult, w)
    return w.to(torch.float16).contiguous()


def activation(M: int, K: int, seed: int, device="cpu") -> torch.Tensor:
    """fp16 [M,K] activations ~ N(0,1)."""
    g = _gen(seed, device)
    return torch.randn((M, K), generator=g, device=device, dtype=torch.float32).to(torch.float16).contiguous()


# (name, N, K) lists per workload; M sweeps beside them.  sigma / outliers per config.
WORKLOADS: Dict[str, dict] = {
    "cfg1_single": dict(shapes=[("lin", 1024, 1024)], Ms=[1], sigma=0.02, outlier_frac=0.0),
    "cfg2_llama7b": dict(shapes=[("qkvo", 4096, 4096), ("up_gate", 11008, 4096), ("down", 4096, 11008)],
                         Ms=[1, 4, 16], sigma=0.02, outlier_frac=0.001),
    "cfg3_llama13b": dict(shapes=[("qkvo", 5120, 5120), ("up_gate", 13824, 5120), ("down", 5120, 13824)],
                          Ms=[1, 8, 32, 128], sigma=0.02, outlier_frac=0.001),
    "cfg4_llama70b_mlp": dict(shapes=[("up_gate", 28672, 8192), ("down", 8192, 28672)],
                              Ms=[1, 16, 64, 256, 512], sigma=0.015, outlier_frac=0.001),
    # 34B-class block: hidden 8192, MLP 22016, grouped-query attention with 8 KV heads
    # of 128 (k/v projections 1024 x 8192); 48 such layers.
    "cfg5_34b_stack": dict(shapes=[("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
                                   ("gate", 22016, 8192), ("up", 22016, 8192), ("down", 8192, 22016)],
                           Ms=[1, 512], sigma=0.015, outlier_frac=0.001, layers=48),
    # the six feed-forward shapes of the paper's kernel table (Appendix B), batch 8
    "paper_table_b1": dict(shapes=[("ffn1_1b", 5504, 2048), ("ffn2_1b", 2048, 5504),
                                   ("ffn1_13b", 13824, 5120), ("ffn2_13b", 5120, 13824),
                                   ("ffn1_65b", 22016, 8192), ("ffn2_65b", 8192, 22016)],
                           Ms=[8], sigma=0.02, outlier_frac=0.001),
}


def workload_seed(workload: str, index: int) -> int:
    """Per-tensor seed: base + 1000 * workload ordinal + tensor index."""
    order: List[str] = list(WORKLOADS.keys())
    return BASE_SEED + 1000 * (order.index(workload) + 1) + int(index)


def workload_weight(workload: str, shape_index: int, layer: int = 0, device="cpu",
                    rows: Tuple[int, int] = None) -> torch.Tensor:
    """Weight of one shape of a workload (optionally only rows [r0,r1) are returned,
    but the whole tensor is always drawn so that the bits do not depend on `rows`)."""
    cfg = WORKLOADS[workload]
    _, N, K = cfg["shapes"][shape_index]
    seed = workload_seed(workload, 16 * layer + shape_index)
    w = weight(N, K, seed, cfg["sigma"], cfg["outlier_frac"], 10.0, device)
    return w if rows is None else w[rows[0]:rows[1]].contiguous()


def mha_kv_weight(workload: str, which: int, layer: int = 0, device="cpu") -> torch.Tensor:
    """k (which = 1) or v (which = 2) projection of a stack workload without grouped-query attention:
    the shape of its q projection, same distribution, a seed of its own (slots 9 and 10 of the layer)."""
    cfg = WORKLOADS[workload]
    _, N, K = cfg["shapes"][0]
    seed = workload_seed(workload, 16 * layer + 8 + which)
    return weight(N, K, seed, cfg["sigma"], cfg["outlier_frac"], 10.0, device)


def activation_bf16(M: int, K: int, seed: int, device="cpu") -> torch.Tensor:
    """bf16 [M,K] activations ~ N(0,1) (the same draw as `activation`, rounded to bf16)."""
    g = _gen(seed, device)
    return torch.randn((M, K), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16).contiguous()
