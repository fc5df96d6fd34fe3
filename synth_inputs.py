"""Seeded synthetic inputs shaped like the paper's workloads.

Shared by the tests, the smoke check and the benchmark so that the HIP path and
the CPU oracle see the same values.  This module holds none of the method's
arithmetic: only shapes, value distributions and rounding to the storage type.

Shapes follow the paper's experiments: ImageNet at 224x224 with patch 16 gives
a 14x14 token grid (plus a class token for ViT); COCO images up to 800x1333,
padded to 800x1344, give ConvNeXt stage maps of 200x336, 100x168 and 50x84.
Activations and output gradients are i.i.d. N(0,1); weights N(0, 0.02^2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import torch


@dataclass(frozen=True)
class LinearShape:
    name: str
    Cin: int
    Cout: int


@dataclass(frozen=True)
class Workload:
    """Geometry of one benchmark/parity configuration."""
    name: str
    dtype: str                    # "f32" or "bf16"
    B: int
    P: int                        # always-kept prefix rows per sample (class token)
    H: int
    W: int
    linears: Tuple[LinearShape, ...]
    blocks: int = 1               # how many times the list of linears repeats
    ratios: Tuple[float, ...] = (0.5,)
    dw_channels: int = 0          # >0: a depthwise 7x7 conv of that width precedes the linears

    @property
    def N(self) -> int:
        return self.P + self.H * self.W

    @property
    def M(self) -> int:
        return self.B * self.N


WORKLOADS = {
    "linear_fp32": Workload(
        "linear_fp32", "f32", 2, 0, 14, 14, (LinearShape("fc", 64, 256),)),
    "vit_tiny_mlp": Workload(
        "vit_tiny_mlp", "bf16", 64, 1, 14, 14,
        (LinearShape("fc1", 192, 768), LinearShape("fc2", 768, 192))),
    "vit_base": Workload(
        "vit_base", "bf16", 64, 1, 14, 14,
        (LinearShape("qkv", 768, 2304), LinearShape("proj", 768, 768),
         LinearShape("fc1", 768, 3072), LinearShape("fc2", 3072, 768)),
        blocks=12, ratios=(0.25, 0.5, 0.75, 1.0)),
    "convnext_det_s1": Workload(
        "convnext_det_s1", "bf16", 2, 0, 200, 336,
        (LinearShape("pw1", 128, 512), LinearShape("pw2", 512, 128))),
    "convnext_det_s2": Workload(
        "convnext_det_s2", "bf16", 2, 0, 100, 168,
        (LinearShape("pw1", 256, 1024), LinearShape("pw2", 1024, 256))),
    "convnext_s3_block": Workload(
        "convnext_s3_block", "bf16", 2, 0, 50, 84,
        (LinearShape("pw1", 512, 2048), LinearShape("pw2", 2048, 512)),
        ratios=(0.25, 0.5, 1.0), dw_channels=512),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def normal(shape, std, seed, dtype: str) -> torch.Tensor:
    """N(0, std^2) values drawn in fp32 on the CPU, then rounded to the storage type."""
    t = torch.randn(*shape, generator=_gen(seed), dtype=torch.float32) * std
    return t.to(torch_dtype(dtype))


def small_ints(shape, lo, hi, seed, dtype: str) -> torch.Tensor:
    """Integer-valued tensors in [lo, hi]: every partial sum of their products is exact."""
    t = torch.randint(lo, hi + 1, shape, generator=_gen(seed), dtype=torch.int32)
    return t.to(torch_dtype(dtype))


def linear_case(M: int, Cin: int, Cout: int, seed: int, dtype: str):
    """(X [M,Cin], W [Cout,Cin], dY [M,Cout]) for one linear / pointwise-conv layer."""
    X = normal((M, Cin), 1.0, seed * 7919 + 1, dtype)
    W = normal((Cout, Cin), 0.02, seed * 7919 + 2, dtype)
    dY = normal((M, Cout), 1.0, seed * 7919 + 3, dtype)
    return X, W, dY


def dwconv_case(B: int, H: int, W: int, C: int, ks: int, seed: int, dtype: str):
    """(X [B,H,W,C], Wd [ks,ks,C], dY [B,H,W,C]) for one depthwise conv layer, channels last."""
    X = normal((B, H, W, C), 1.0, seed * 7919 + 11, dtype)
    Wd = normal((ks, ks, C), 0.02, seed * 7919 + 12, dtype)
    dY = normal((B, H, W, C), 1.0, seed * 7919 + 13, dtype)
    return X, Wd, dY


def to_f64(t: torch.Tensor):
    """Exact widening of a stored tensor to a float64 numpy array."""
    return t.detach().cpu().to(torch.float64).numpy()


def attention_case(B: int, n: int, h: int, d: int, seed: int, dtype: str):
    """Tensors of one self-attention layer, token-major as a qkv projection leaves them.

    Returns qkv [B*n, 3*h*d] (q | k | v thirds, each head-major [h, d]) and dA [B*n, h*d] in the
    storage type: unit-variance queries, keys and values (scores q.k/sqrt(d) of unit variance, the
    regime of a trained ViT's pre-softmax logits) and a unit-variance output gradient.
    """
    qkv = normal((B * n, 3 * h * d), 1.0, seed * 7919 + 21, dtype)
    dA = normal((B * n, h * d), 1.0, seed * 7919 + 22, dtype)
    return qkv, dA


def attention_forward(qkv: torch.Tensor, B: int, n: int, h: int, d: int, scale: float):
    """The model's forward over all n tokens (library softmax, float64): the attention output
    A [B*n, h*d] and the row-wise log-sum-exp of the scaled scores lse [B*n, h], both float64.
    A training forward hands these to the backward; they are inputs of the path, not part of it."""
    x = qkv.detach().cpu().to(torch.float64).view(B, n, 3, h, d)
    q, k, v = (x[:, :, i].permute(0, 2, 1, 3) for i in range(3))          # [B, h, n, d]
    m = torch.matmul(q, k.transpose(-1, -2)) * scale
    lse = torch.logsumexp(m, dim=-1)                                      # [B, h, n]
    A = torch.matmul(torch.softmax(m, dim=-1), v)                         # [B, h, n, d]
    return A.permute(0, 2, 1, 3).reshape(B * n, h * d).contiguous(), lse.permute(0, 2, 1).reshape(B * n, h).contiguous()
