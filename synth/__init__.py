"""Seeded synthetic gradients shaped like the paper's workloads.

Serves both the CPU oracle's tests and the GPU path's tests / benchmark; holds
none of the method's arithmetic (no compressor, no residual, no optimizer).

The paper trains ResNet-50, VGG16 (ImageNet) and BERT-base / BERT-large
(Wikipedia + BookCorpus); neither the datasets nor the models are available
here, so flat gradients of the same element counts and dtypes stand in, drawn
from heavy-tailed or per-layer-scaled distributions:

  sign_1m      1,048,576 f32, N(0, 1e-3^2)
  resnet50     25,557,032 f32, N(0, 1e-3^2) x per-partition scale, scale
               log-uniform in [1e-4, 1e-1] (layers differ by orders of magnitude)
  vgg16        138,357,544 f32, Laplace(0, 1e-3)
  bert_base    110,000,000 f16, 1e-3 x Student-t(3)
  bert_large   336,000,000 f16, 1e-3 x Student-t(3)

Two generators: ``host_gradient`` (numpy, Philox bit generator keyed by
(seed, worker, step)) for everything the oracle touches, and
``device_gradient`` (torch generator on the GPU, same distributions, different
bits) for full-size benchmark inputs, which are copied back to the host
wherever the oracle needs the same bytes.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 20210517
PART_BYTES = 4 << 20  # 4 MiB of gradient per partition

WORKLOADS = {
    "sign_1m": dict(D=1_048_576, dtype="f32", dist="normal", kind="sign", n_workers=4,
                    ef=True, opt=None),
    "resnet50": dict(D=25_557_032, dtype="f32", dist="normal_layer_scaled", kind="topk", k_ratio=0.01,
                     n_workers=8, ef=True, opt=None),
    "vgg16": dict(D=138_357_544, dtype="f32", dist="laplace", kind="randk", k_ratio=0.01,
                  value_scale=-1.0, n_workers=8, ef=True, opt=None),
    "bert_base": dict(D=110_000_000, dtype="f16", dist="student_t3", kind="sign", n_workers=16,
                      ef=True, opt="adam"),
    "bert_large": dict(D=336_000_000, dtype="f16", dist="student_t3", kind="dither", levels=4,
                       n_workers=16, ef=True, opt="adam"),
    # not a BASELINE configuration: the bert_large shape with the natural (power-of-two) level map
    "bert_large_natural": dict(D=336_000_000, dtype="f16", dist="student_t3", kind="natdither", levels=4,
                               n_workers=16, ef=True, opt="adam"),
    # nor is this: the 5-bit form of linear dithering (15 levels: nibbles and one bit plane)
    # nor this: BERT-base shape with the paper's own BERT setting, top-k of 0.1 % sent as 32-bit index + half value
    "bert_base_topk16": dict(D=110_000_000, dtype="f16", dist="student_t3", kind="topk16", k_ratio=0.001,
                             n_workers=16, ef=True, opt="adam"),
    # nor this: the FP32 -> FP16 conversion as the compressor
    "bert_large_fp16": dict(D=336_000_000, dtype="f16", dist="student_t3", kind="fp16",
                            n_workers=16, ef=True, opt="adam"),
    "bert_large_5bit": dict(D=336_000_000, dtype="f16", dist="student_t3", kind="dither", levels=15,
                            n_workers=16, ef=True, opt="adam"),
}


def part_elems(dtype: str) -> int:
    return PART_BYTES // (4 if dtype == "f32" else 2)


def _np_rng(seed: int, worker: int, step: int, tag: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed + worker) & (2**64 - 1),
                                                     (step << 8 | tag) & (2**64 - 1)]))


def partition_scales(n_parts: int, seed: int = BASE_SEED) -> np.ndarray:
    """Per-partition scale, log-uniform in [1e-4, 1e-1]; same for every worker and step."""
    rng = _np_rng(seed, 0, 0, tag=7)
    return np.exp(rng.uniform(math.log(1e-4), math.log(1e-1), size=n_parts)).astype(np.float32)


def host_gradient(dist: str, D: int, dtype: str = "f32", worker: int = 0, step: int = 0,
                  seed: int = BASE_SEED, part: int | None = None) -> np.ndarray:
    """One worker's flat gradient for one step, numpy float32 or float16."""
    rng = _np_rng(seed, worker, step)
    if dist == "normal":
        x = rng.standard_normal(D, dtype=np.float32) * np.float32(1e-3)
    elif dist == "normal_layer_scaled":
        pe = part or part_elems(dtype)
        n_parts = (D + pe - 1) // pe
        x = rng.standard_normal(D, dtype=np.float32) * np.float32(1e-3)
        scales = partition_scales(n_parts, seed)
        x *= np.repeat(scales, pe)[:D]
    elif dist == "laplace":
        x = rng.laplace(0.0, 1e-3, size=D).astype(np.float32)
    elif dist == "student_t3":
        x = (rng.standard_t(3.0, size=D) * 1e-3).astype(np.float32)
    else:
        raise ValueError(dist)
    if dtype == "f16":
        return x.astype(np.float16)
    return x


def host_params(D: int, seed: int = BASE_SEED) -> np.ndarray:
    """Model parameters x ~ N(0, 0.02^2), float32."""
    rng = _np_rng(seed, 0, 0, tag=3)
    return rng.standard_normal(D, dtype=np.float32) * np.float32(0.02)


def device_gradient(dist: str, D: int, dtype: str = "f32", worker: int = 0, step: int = 0,
                    seed: int = BASE_SEED, device="cuda", part: int | None = None):
    """Same distributions generated on the GPU with a seeded torch generator."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(((seed + worker) * 1_000_003 + step) & (2**63 - 1))
    out_dtype = torch.float16 if dtype == "f16" else torch.float32
    out = torch.empty(D, dtype=out_dtype, device=device)
    chunk = 1 << 25  # bounded temporaries
    pe = part or part_elems(dtype)
    scales = None
    if dist == "normal_layer_scaled":
        n_parts = (D + pe - 1) // pe
        scales = torch.from_numpy(partition_scales(n_parts, seed)).to(device)
    for lo in range(0, D, chunk):
        n = min(chunk, D - lo)
        if dist in ("normal", "normal_layer_scaled"):
            x = torch.randn(n, generator=g, device=device) * 1e-3
            if scales is not None:
                idx = (torch.arange(lo, lo + n, device=device) // pe)
                x = x * scales[idx]
        elif dist == "laplace":
            # inverse CDF; |u| is kept below 1/2 (rand() can return exactly 0, which would map to
            # an infinite gradient: about eight a worker at this size)
            u = torch.rand(n, generator=g, device=device) - 0.5
            x = -1e-3 * torch.sign(u) * torch.log1p(-(2.0 * u.abs()).clamp(max=1.0 - 2.0 ** -24))
        elif dist == "student_t3":
            z = torch.randn(n, generator=g, device=device)
            w = torch.randn(3, n, generator=g, device=device)
            x = 1e-3 * z / torch.sqrt((w * w).sum(0) / 3.0)
        else:
            raise ValueError(dist)
        out[lo:lo + n] = x.to(out_dtype)
    return out


def layer_blocks(D: int, hidden: int = 1024, vocab: int = 30522) -> np.ndarray:
    """Ascending element offsets (first 0, last D) that cut a flat gradient of D elements into
    blocks sized like the parameter tensors of a BERT encoder stack: the embedding tables and
    their layer norm, then per layer four hidden x hidden projections with biases, a layer norm,
    the two feed-forward matrices with biases and another layer norm, repeated until D is used
    up (the last block is cut short).  These are the layers that LANS normalises over; sizes
    range from `hidden` elements to tens of millions, and most boundaries fall inside a
    partition."""
    h = hidden
    sizes = [vocab * h, 512 * h, 2 * h, h, h]
    layer = [h * h, h] * 4 + [h, h] + [4 * h * h, 4 * h, 4 * h * h, h] + [h, h]
    offs, at, i = [0], 0, 0
    while at < D:
        size = sizes[i] if i < len(sizes) else layer[(i - len(sizes)) % len(layer)]
        at = min(D, at + size)
        offs.append(at)
        i += 1
    return np.asarray(offs, dtype=np.uint64)


def device_params(D: int, seed: int = BASE_SEED, device="cuda"):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed((seed * 7 + 3) & (2**63 - 1))
    return torch.randn(D, generator=g, device=device) * 0.02
