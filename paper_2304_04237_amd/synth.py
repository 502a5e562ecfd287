"""Seeded synthetic inputs for the Slide Attention operator.

This module holds no arithmetic of the method: it only draws random tensors of
the shapes, value distributions and dtypes of the workloads, so that the GPU
library and the CPU oracle can be fed the same values.  The workloads stand in
for the feature maps of hierarchical ViT stages (224x224 classification input:
56x56 at stage 1, 28x28 at stage 2; an 800x1216 detection image: 200x304 at
stride 4), whose datasets and trained weights are not available here.

Draw order is fixed (q, k, v, wk, wv, bias, dout) from one CPU generator seeded
with 1000 + config index.  bf16 workloads are drawn in fp32 and rounded once to
bf16; the values returned as float32 are those rounded values, so every
consumer sees identical inputs.
"""
from collections import namedtuple

import torch

Workload = namedtuple("Workload", "name B H W C heads ksize dtype backward")

# index 0..4 mirror the five benchmark configurations
CONFIGS = [
    Workload("tiny_fp32_fwd", 1, 14, 14, 64, 2, 3, "f32", False),
    Workload("stage1_bf16_fwd", 64, 56, 56, 64, 2, 3, "bf16", False),
    Workload("stage2_k5_bf16_fwd", 64, 28, 28, 128, 4, 5, "bf16", False),
    Workload("dense_200x304_bf16_fwd", 2, 200, 304, 96, 3, 3, "bf16", False),
    Workload("stage1_bf16_train", 128, 56, 56, 64, 2, 3, "bf16", True),
]

KERNEL_STD = 0.02
BIAS_STD = 0.02


def _round_to(x, dtype):
    if dtype == "bf16":
        return x.to(torch.bfloat16).to(torch.float32)
    return x


def make_inputs(B, H, W, C, heads, ksize, dtype="f32", seed=0, with_dout=True,
                kernel_std=KERNEL_STD, bias_std=BIAS_STD):
    """Return a dict of float32 CPU tensors.

    q, k, v, dout: [B, C, H, W] ~ N(0, 1), already rounded to `dtype`;
    wk_learned, wv_learned: [C, ksize*ksize, ksize, ksize] ~ N(0, kernel_std^2) (fp32);
    bias: [heads, ksize*ksize] ~ N(0, bias_std^2) (fp32).
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    S = ksize * ksize
    out = {}
    for name in ("q", "k", "v"):
        out[name] = _round_to(torch.randn(B, C, H, W, generator=g, dtype=torch.float32), dtype)
    out["wk_learned"] = torch.randn(C, S, ksize, ksize, generator=g, dtype=torch.float32) * kernel_std
    out["wv_learned"] = torch.randn(C, S, ksize, ksize, generator=g, dtype=torch.float32) * kernel_std
    out["bias"] = torch.randn(heads, S, generator=g, dtype=torch.float32) * bias_std
    if with_dout:
        out["dout"] = _round_to(torch.randn(B, C, H, W, generator=g, dtype=torch.float32), dtype)
    return out


def make_config_inputs(index, batch=None):
    """Inputs of benchmark configuration `index` (optionally with a smaller batch)."""
    wl = CONFIGS[index]
    B = wl.B if batch is None else int(batch)
    data = make_inputs(B, wl.H, wl.W, wl.C, wl.heads, wl.ksize, wl.dtype,
                       seed=1000 + index, with_dout=True)
    return wl._replace(B=B), data
