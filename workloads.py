"""Seeded synthetic workloads for the DeAR gradient-aggregation path.

This module holds input recipes only: parameter-tensor size lists shaped like the
paper's models (Table I) and seeded random gradients / parameters.  It contains
none of the method's arithmetic (no grouping, no reduction, no update), so the
CPU oracle's tests and the HIP path's tests can both draw inputs from it without
sharing any code of the method itself.

Tensor lists are in forward order (index 0 = first layer); gradients become ready
in the reverse order during back-propagation (Section III-B).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import torch

KB = 1024
MB = 1 << 20


# --------------------------------------------------------------------------- shapes
def tiny_sizes() -> List[int]:
    return [4096, 64, 65536, 128, 262144, 256, 16384, 10]


def resnet50_sizes() -> List[int]:
    """ResNet-50 parameter tensors: conv weights, BatchNorm weight+bias, fc weight+bias.

    Table I lists 161 tensors / 25.6 M parameters for this model.
    """
    s: List[int] = []

    def conv(cout, cin, k):
        s.append(cout * cin * k * k)

    def bn(c):
        s.extend([c, c])

    conv(64, 3, 7)
    bn(64)
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(blocks):
            conv(planes, inplanes, 1)
            bn(planes)
            conv(planes, planes, 3)
            bn(planes)
            conv(planes * 4, planes, 1)
            bn(planes * 4)
            if blk == 0:  # projection shortcut of the first block of a stage
                conv(planes * 4, inplanes, 1)
                bn(planes * 4)
            inplanes = planes * 4
    s.append(1000 * 2048)
    s.append(1000)
    return s


def densenet201_sizes() -> List[int]:
    """DenseNet-201 (growth rate 32, bottleneck width 4, blocks of 6/12/48/32 layers).

    Table I lists 604 tensors / 20.0 M parameters for this model.
    """
    s: List[int] = []
    growth, bn_size, feats = 32, 4, 64
    s.append(64 * 3 * 7 * 7)
    s.extend([64, 64])
    blocks = (6, 12, 48, 32)
    for bi, layers in enumerate(blocks):
        for _ in range(layers):
            s.extend([feats, feats])                          # norm1
            s.append(bn_size * growth * feats)                # 1x1 bottleneck conv
            s.extend([bn_size * growth, bn_size * growth])    # norm2
            s.append(growth * bn_size * growth * 9)           # 3x3 conv
            feats += growth
        if bi != len(blocks) - 1:                             # transition: norm + 1x1 conv halving the width
            s.extend([feats, feats])
            s.append((feats // 2) * feats)
            feats //= 2
    s.extend([feats, feats])                                  # final norm
    s.append(1000 * feats)
    s.append(1000)
    return s


def inception_v4_sizes() -> List[int]:
    """Inception-v4: 149 convolution + BatchNorm units (weight, BN weight, BN bias) and the
    classifier.  Table I lists 449 tensors / 42.7 M parameters for this model."""
    s: List[int] = []

    def unit(cin, cout, kh, kw):
        s.append(cout * cin * kh * kw)
        s.extend([cout, cout])

    # stem
    unit(3, 32, 3, 3); unit(32, 32, 3, 3); unit(32, 64, 3, 3)
    unit(64, 96, 3, 3)                                         # mixed 3a (beside a max-pool)
    unit(160, 64, 1, 1); unit(64, 96, 3, 3)                    # mixed 4a, branch 0
    unit(160, 64, 1, 1); unit(64, 64, 1, 7); unit(64, 64, 7, 1); unit(64, 96, 3, 3)
    unit(192, 192, 3, 3)                                       # mixed 5a (beside a max-pool)
    for _ in range(4):                                         # Inception-A, 384 channels
        unit(384, 96, 1, 1)
        unit(384, 64, 1, 1); unit(64, 96, 3, 3)
        unit(384, 64, 1, 1); unit(64, 96, 3, 3); unit(96, 96, 3, 3)
        unit(384, 96, 1, 1)
    unit(384, 384, 3, 3)                                       # Reduction-A -> 1024 channels
    unit(384, 192, 1, 1); unit(192, 224, 3, 3); unit(224, 256, 3, 3)
    for _ in range(7):                                         # Inception-B
        unit(1024, 384, 1, 1)
        unit(1024, 192, 1, 1); unit(192, 224, 1, 7); unit(224, 256, 7, 1)
        unit(1024, 192, 1, 1); unit(192, 192, 7, 1); unit(192, 224, 1, 7); unit(224, 224, 7, 1); unit(224, 256, 1, 7)
        unit(1024, 128, 1, 1)
    unit(1024, 192, 1, 1); unit(192, 192, 3, 3)                # Reduction-B -> 1536 channels
    unit(1024, 256, 1, 1); unit(256, 256, 1, 7); unit(256, 320, 7, 1); unit(320, 320, 3, 3)
    for _ in range(3):                                         # Inception-C
        unit(1536, 256, 1, 1)
        unit(1536, 384, 1, 1); unit(384, 256, 1, 3); unit(384, 256, 3, 1)
        unit(1536, 384, 1, 1); unit(384, 448, 3, 1); unit(448, 512, 1, 3); unit(512, 256, 1, 3); unit(512, 256, 3, 1)
        unit(1536, 256, 1, 1)
    s.append(1000 * 1536)
    s.append(1000)
    return s


def bert_sizes(layers: int, hidden: int, ffn: int, vocab: int = 30522,
               max_pos: int = 512, type_vocab: int = 2) -> List[int]:
    """BERT pre-training model (MLM + NSP heads) parameter tensors.

    Table I lists 206 tensors / 110.1 M (Base) and 398 tensors / 336.2 M (Large).
    """
    h = hidden
    s: List[int] = [vocab * h, max_pos * h, type_vocab * h, h, h]  # embeddings + LayerNorm
    for _ in range(layers):
        for _ in range(4):            # Q, K, V, attention output
            s.extend([h * h, h])
        s.extend([h, h])              # attention LayerNorm
        s.extend([h * ffn, ffn])      # FFN in
        s.extend([ffn * h, h])        # FFN out
        s.extend([h, h])              # output LayerNorm
    s.extend([h * h, h])              # pooler
    s.extend([h * h, h, h, h, vocab])  # MLM head: dense, LayerNorm, vocabulary bias
    s.extend([2 * h, 2])              # NSP classifier
    return s


def bert_base_sizes() -> List[int]:
    return bert_sizes(12, 768, 3072)


def bert_large_sizes() -> List[int]:
    return bert_sizes(24, 1024, 4096)


# --------------------------------------------------------------------------- configs
@dataclass
class Workload:
    name: str
    index: int                 # position in the config list; enters the seeds
    P: int                     # emulated workers
    sizes: List[int] = field(repr=False)
    grad_dtype: str            # "f32" | "bf16"
    grad_std: float
    threshold_bytes: int       # fusion buffer size x, in bytes of the gradient dtype
    lr: float = 0.1
    momentum: float = 0.9

    @property
    def n_layers(self) -> int:
        return len(self.sizes)

    @property
    def N(self) -> int:
        return sum(self.sizes)

    @property
    def grad_elem_bytes(self) -> int:
        return 4 if self.grad_dtype == "f32" else 2

    @property
    def base_seed(self) -> int:
        return 20230212 + self.index

    def algorithmic_bytes(self) -> dict:
        """Bytes the three phases must move per iteration (reads + writes)."""
        g, P, N = self.grad_elem_bytes, self.P, self.N
        return {"rs": g * P * N + 4 * N, "update": 20 * N, "ag": 4 * N + 4 * P * N,
                "total": N * (g * P + 4 * P + 28)}


NO_LIMIT = (1 << 63) - 1


def get_workload(name: str) -> Workload:
    if name == "tiny":
        return Workload("tiny", 0, 4, tiny_sizes(), "f32", 0.01, 256 * KB)
    if name == "resnet50":
        return Workload("resnet50", 1, 8, resnet50_sizes(), "f32", 1e-3, 25 * MB)
    if name == "bert_base":
        return Workload("bert_base", 2, 16, bert_base_sizes(), "f32", 1e-3, 64 * MB)
    if name == "bert_large":
        return Workload("bert_large", 3, 8, bert_large_sizes(), "bf16", 1e-3, 64 * MB)
    if name == "densenet201":
        return Workload("densenet201", 5, 8, densenet201_sizes(), "f32", 1e-3, 25 * MB)
    if name == "inception_v4":
        return Workload("inception_v4", 6, 8, inception_v4_sizes(), "f32", 1e-3, 25 * MB)
    if name == "stress_single":
        return Workload("stress_single", 4, 64, bert_base_sizes(), "f32", 1e-3, NO_LIMIT)
    if name == "stress_16mb":
        return Workload("stress_16mb", 4, 64, bert_base_sizes(), "f32", 1e-3, 16 * MB)
    raise KeyError(name)


WORKLOAD_NAMES = ["tiny", "resnet50", "bert_base", "bert_large", "stress_single", "stress_16mb",
                  "densenet201", "inception_v4"]


# --------------------------------------------------------------------------- seeded inputs
def _torch_dtype(grad_dtype: str):
    return torch.float32 if grad_dtype == "f32" else torch.bfloat16


def grad_seed(w: Workload, p: int, it: int) -> int:
    return w.base_seed * 1000 + p + 100 * it


def param_seed(w: Workload) -> int:
    return w.base_seed * 1000 + 999


def make_flat_grad(w: Workload, p: int, it: int, device="cpu") -> torch.Tensor:
    """Replica p's gradient at iteration `it`, all tensors concatenated in forward order.

    fp32 N(0, std); for bf16 workloads the fp32 draw is rounded to nearest-even bf16.
    """
    gen = torch.Generator(device=device)
    gen.manual_seed(grad_seed(w, p, it))
    x = torch.empty(w.N, dtype=torch.float32, device=device)
    x.normal_(0.0, w.grad_std, generator=gen)
    return x.to(_torch_dtype(w.grad_dtype))


def make_flat_param(w: Workload, device="cpu") -> torch.Tensor:
    """Initial parameters ~U(-0.1, 0.1), fp32, identical on every replica."""
    gen = torch.Generator(device=device)
    gen.manual_seed(param_seed(w))
    x = torch.empty(w.N, dtype=torch.float32, device=device)
    x.uniform_(-0.1, 0.1, generator=gen)
    return x


def split_layers(flat: torch.Tensor, sizes: List[int], align_elems: int = 1) -> List[torch.Tensor]:
    """Per-layer views of a flat tensor (no copy).  With align_elems > 1 the flat tensor
    must have been sized by `padded_total` and every view starts on that multiple."""
    out, pos = [], 0
    for n in sizes:
        out.append(flat[pos:pos + n])
        pos += n
        if align_elems > 1:
            pos = (pos + align_elems - 1) // align_elems * align_elems
    return out


def padded_total(sizes: List[int], align_elems: int) -> int:
    pos = 0
    for n in sizes:
        pos += n
        pos = (pos + align_elems - 1) // align_elems * align_elems
    return pos


def scatter_into_aligned(flat: torch.Tensor, sizes: List[int], align_elems: int) -> List[torch.Tensor]:
    """Copy a dense flat tensor into a fresh buffer whose per-layer views start on
    `align_elems` multiples (so every layer's base address keeps the 16-byte alignment
    the device library requires) and return those views."""
    buf = torch.zeros(padded_total(sizes, align_elems), dtype=flat.dtype, device=flat.device)
    views = split_layers(buf, sizes, align_elems)
    pos = 0
    for v, n in zip(views, sizes):
        v.copy_(flat[pos:pos + n])
        pos += n
    return views
