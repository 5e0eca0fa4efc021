"""Shared test plumbing: numpy views of the seeded workloads for the CPU oracle."""
from __future__ import annotations

from typing import List, Sequence

import numpy as np
import torch

import workloads as W


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """torch CPU tensor -> numpy; bfloat16 comes back as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def split_np(flat: np.ndarray, sizes: Sequence[int]) -> List[np.ndarray]:
    out, pos = [], 0
    for n in sizes:
        out.append(np.ascontiguousarray(flat[pos:pos + n]))
        pos += n
    return out


def grads_np(w: W.Workload, it: int) -> List[List[np.ndarray]]:
    """grads[p][l] for iteration `it`, from the seeded CPU generator."""
    return [split_np(to_numpy(W.make_flat_grad(w, p, it)), w.sizes) for p in range(w.P)]


def params_np(w: W.Workload) -> List[List[np.ndarray]]:
    """params[p][l]: P identical replicas of the seeded initial parameters."""
    flat = to_numpy(W.make_flat_param(w))
    return [split_np(flat.copy(), w.sizes) for _ in range(w.P)]


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


def as_f32(a: np.ndarray) -> np.ndarray:
    return a if a.dtype == np.float32 else bf16_bits_to_f32(a)


def small_workload(sizes: Sequence[int], P: int, threshold_bytes: int, grad_dtype: str = "f32",
                   index: int = 7, std: float = 0.01) -> W.Workload:
    return W.Workload("custom", index, P, list(sizes), grad_dtype, std, threshold_bytes)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 (8 significand bits) at |x|: 2^(floor(log2|x|) - 7)."""
    ax = np.abs(x.astype(np.float64))
    ax = np.maximum(ax, 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)
