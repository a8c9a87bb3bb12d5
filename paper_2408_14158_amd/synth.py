"""Seeded synthetic gradient-shaped inputs.

This module holds no reduction arithmetic. It only draws random numbers with
torch's generators and lays them out as the K per-GPU gradient buffers that the
paper's intra-node reduce (Algorithm 1) consumes, or as the two node partials
that its inter-node step (Algorithm 2, pass 1) combines. Both the HIP library's
tests and the CPU oracle's tests take their inputs from here; neither side's
code is imported.

bf16 values are produced with torch's own float32 -> bfloat16 cast (a library
routine) and handed around as torch.bfloat16 tensors; ``as_numpy_bits`` turns any
buffer into the raw-bit numpy array (uint16 for bf16) the oracle works on.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

# 25 * 2**20: the bucket cap of the bucketed-gradient workload. A multiple of
# eight elements, so every full bucket starts 16-byte aligned in a flat buffer.
BUCKET_CAP_ELEMS = 25 * (1 << 20)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def uniform_pm1(n: int, seed: int, device="cpu") -> torch.Tensor:
    """n fp32 values iid uniform on [-1, 1)."""
    g = _gen(seed, device)
    x = torch.rand(n, generator=g, device=device, dtype=torch.float32)
    return x.mul_(2.0).sub_(1.0)


def normal_f32(n: int, std: float, seed: int, device="cpu") -> torch.Tensor:
    """n fp32 values iid N(0, std^2)."""
    g = _gen(seed, device)
    x = torch.randn(n, generator=g, device=device, dtype=torch.float32)
    return x.mul_(float(std))


def normal_bf16(n: int, std: float, seed: int, device="cpu") -> torch.Tensor:
    """n bf16 values: fp32 N(0, std^2) draws cast to bfloat16 by torch."""
    return normal_f32(n, std, seed, device).to(torch.bfloat16)


def normal_f16(n: int, std: float, seed: int, device="cpu") -> torch.Tensor:
    """n fp16 values: fp32 N(0, std^2) draws cast to float16 by torch."""
    return normal_f32(n, std, seed, device).to(torch.float16)


def peer_buffers_normal_f16(K: int, n: int, std: float, seed0: int, device="cpu"):
    """K fp16 gradient buffers, buffer j drawn with seed seed0 + j."""
    return [normal_f16(n, std, seed0 + j, device) for j in range(K)]


FP8_TORCH = {"e4m3": torch.float8_e4m3fn, "e5m2": torch.float8_e5m2}


def normal_fp8(n: int, std: float, seed: int, fmt: str, device="cpu") -> torch.Tensor:
    """n fp8 values (fmt "e4m3" or "e5m2"): fp32 N(0, std^2) draws cast by torch."""
    return normal_f32(n, std, seed, device).to(FP8_TORCH[fmt])


def peer_buffers_normal_fp8(K: int, n: int, std: float, seed0: int, fmt: str, device="cpu"):
    """K fp8 gradient buffers, buffer j drawn with seed seed0 + j."""
    return [normal_fp8(n, std, seed0 + j, fmt, device) for j in range(K)]


def peer_buffers_uniform_f32(K: int, n: int, seed0: int, device="cpu"):
    """K fp32 buffers, buffer j drawn with seed seed0 + j (stand-ins for the
    node's K GPUs holding the same-shaped gradient chunk)."""
    return [uniform_pm1(n, seed0 + j, device) for j in range(K)]


def peer_buffers_normal_bf16(K: int, n: int, std: float, seed0: int, device="cpu"):
    """K bf16 gradient buffers, buffer j drawn with seed seed0 + j."""
    return [normal_bf16(n, std, seed0 + j, device) for j in range(K)]


@dataclass(frozen=True)
class GradTensor:
    name: str
    numel: int
    fan_in: int


def transformer_grad_tensors(n_layers: int = 8, d_model: int = 4096, ffn: int = 11008,
                             vocab: int = 32000):
    """Parameter tensors of a decoder-only transformer, in registration order
    (embedding first, final norm last). Per layer: two RMSNorm vectors, Q/K/V/O
    projections and the gate/up/down MLP matrices. fan_in is the input width of
    each matrix and 1 for norm vectors."""
    ts = [GradTensor("embed", vocab * d_model, d_model)]
    for l in range(n_layers):
        p = "layer%d." % l
        ts.append(GradTensor(p + "attn_norm", d_model, 1))
        for nm in ("q", "k", "v", "o"):
            ts.append(GradTensor(p + nm, d_model * d_model, d_model))
        ts.append(GradTensor(p + "mlp_norm", d_model, 1))
        ts.append(GradTensor(p + "gate", d_model * ffn, d_model))
        ts.append(GradTensor(p + "up", d_model * ffn, d_model))
        ts.append(GradTensor(p + "down", ffn * d_model, ffn))
    ts.append(GradTensor("final_norm", d_model, 1))
    return ts


def flat_gradient_bf16(tensors, seed: int, device="cpu", base_std: float = 1e-3) -> torch.Tensor:
    """One peer's flat bf16 gradient buffer: tensors laid back to back in
    REVERSE registration order (the order gradients become ready in backward),
    tensor t drawn N(0, (base_std / sqrt(fan_in))^2) with its own seed."""
    total = sum(t.numel for t in tensors)
    flat = torch.empty(total, dtype=torch.bfloat16, device=device)
    off = 0
    for idx, t in enumerate(reversed(tensors)):
        std = base_std / math.sqrt(t.fan_in)
        # distinct stream per (peer seed, tensor)
        flat[off:off + t.numel] = normal_bf16(t.numel, std, seed * 1000003 + idx, device)
        off += t.numel
    return flat


def bucket_cuts(total: int, cap: int = BUCKET_CAP_ELEMS):
    """Flat packing: (offset, length) of consecutive buckets of at most cap
    elements covering [0, total); tensors may straddle bucket edges."""
    cuts = []
    off = 0
    while off < total:
        ln = min(cap, total - off)
        cuts.append((off, ln))
        off += ln
    return cuts


def bucket_cuts_whole_tensors(tensors, cap: int = BUCKET_CAP_ELEMS):
    """Whole-tensor packing of the same flat buffer: walk the tensors in the
    order they lie in it (reverse registration), append each to the open
    bucket and close the bucket once it holds at least cap elements. No tensor
    straddles a bucket edge; buckets are uneven (one large matrix can fill a
    bucket alone). Returns (offset, length) pairs covering the flat buffer."""
    cuts = []
    start = 0
    held = 0
    for t in reversed(tensors):
        held += t.numel
        if held >= cap:
            cuts.append((start, held))
            start += held
            held = 0
    if held:
        cuts.append((start, held))
    return cuts


def as_numpy_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a 1-D buffer as the oracle's array type: float32 stays
    float32, bfloat16 and float16 become uint16 bit patterns, fp8 uint8."""
    t = t.detach()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).cpu().numpy().view(np.uint16).copy()
    if t.dtype in (torch.float8_e4m3fn, torch.float8_e5m2):
        return t.view(torch.uint8).cpu().numpy().copy()
    if t.dtype == torch.float32:
        return t.cpu().numpy().copy()
    raise TypeError("unsupported dtype %s" % t.dtype)
