"""Seeded synthetic inputs shaped like the linear layers of compressed vision transformers.

This module holds input generation only (shapes, distributions, seeds) and none of the method's arithmetic; it is
the one piece shared by the GPU path's tests/benchmark and by the CPU oracle's callers.  The paper evaluates on
ImageNet-1K / COCO / ADE20K through trained DeiT / Swin checkpoints (Sec. 4); none of that data is used here.  The
Gaussian tensors below take the *shapes* of those models' linear layers (Sec. 3.2: Q/K/V projection, attention output
projection, the two feed-forward linears) and stand in for them.
"""
import math

import numpy as np

def layer_shapes(hidden, mlp):
    """The four linear layers of one encoder block: (name, K, N, fused GELU, input distribution)."""
    return [
        ("qkv", hidden, 3 * hidden, False, "normal"),
        ("proj", hidden, hidden, False, "normal"),
        ("fc1", hidden, mlp, True, "normal"),
        ("fc2", mlp, hidden, False, "gelu_normal"),
    ]


CONFIGS = {
    # single linear layer, DeiT-Tiny-like
    "c0": dict(M=197, layers=[("linear", 192, 768, False, "normal_clip4")], depth=1, seed=0),
    # ViT-Base MLP fc1 at batch 64
    "c1": dict(M=64 * 197, layers=[("fc1", 768, 3072, True, "normal")], depth=1, seed=0),
    # one ViT-Base encoder block's linear chain at batch 128
    "c2": dict(M=128 * 197, layers=layer_shapes(768, 3072), depth=1, seed=0),
    # Swin-Base-like stage 3 at batch 64 (7x7 windows on a 14x14 map)
    "c3": dict(M=64 * 196, layers=layer_shapes(512, 2048), depth=1, seed=0),
    # ViT-Large/16 and ViT-Huge/14 full depth at batch 256
    "c4_vitl": dict(M=256 * 197, layers=layer_shapes(1024, 4096), depth=24, seed=0),
    "c4_vith": dict(M=256 * 257, layers=layer_shapes(1280, 5120), depth=32, seed=0),
}


def stream(seed, *ids):
    """Independent counter-based stream per (seed, ids...)."""
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), *[int(v) for v in ids]])))


def activations(M, K, dist="normal", seed=0, ids=(0,), rows=None):
    """X [M,K] fp32.  dist: 'normal' N(0,1); 'normal_clip4' N(0,1) clamped to +-4; 'gelu_normal' GELU(N(0,1))
    (non-negative-skewed, the input of a feed-forward network's second linear layer)."""
    g = stream(seed, *ids, 1)
    x = g.standard_normal((M, K), dtype=np.float32)
    if dist == "normal_clip4":
        x = np.clip(x, -4.0, 4.0)
    elif dist == "gelu_normal":
        x = _gelu_of(x)
    elif dist != "normal":
        raise ValueError(dist)
    return x if rows is None else x[rows]


def _gelu_of(x):
    from scipy.special import erf  # only shapes an input distribution

    x64 = x.astype(np.float64)
    return (0.5 * x64 * (1.0 + erf(x64 / math.sqrt(2.0)))).astype(np.float32)


def weights(N, K, seed=0, ids=(0,), sigma=0.02):
    """W [N,K] fp32 ~ N(0, sigma) (sigma is the standard deviation), dense (not yet pruned)."""
    return (stream(seed, *ids, 2).standard_normal((N, K), dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def bias(N, seed=0, ids=(0,), sigma=0.01):
    return (stream(seed, *ids, 3).standard_normal((N,), dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def small_integers(shape, lo, hi, seed=0, ids=(0,)):
    """integer-valued tensors (exactly representable in fp16/int8) for order-independent exact tests"""
    return stream(seed, *ids, 4).integers(lo, hi + 1, size=shape)
