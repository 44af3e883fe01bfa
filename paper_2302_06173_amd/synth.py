"""Seeded synthetic workloads: tensor-shape lists and value distributions.

This module holds NO optimizer or digest arithmetic.  It only says which shapes a workload has
and how its inputs are drawn, so that the GPU library, the CPU oracle and the benchmark can all
be fed the same bits.  The shape lists stand in for the models the paper trains (ResNet-50-class
CNNs, BERT-large, GPT-class transformers); datasets and trained weights are not needed because
the update path depends only on shapes and value distributions.

Draw order (fixed, so a seed defines the bits): for each tensor in list order: theta, g, m, v;
then, if requested, the zero mask and the outlier mask of g.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import torch

Shape = Tuple[int, ...]


def numel(shape: Shape) -> int:
    n = 1
    for s in shape:
        n *= s
    return n


def resnet50_shapes() -> List[Shape]:
    """Standard ResNet-50: 161 tensors, 25,557,032 parameters."""
    out: List[Shape] = [(64, 3, 7, 7), (64,), (64,)]
    cin = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            out += [(width, cin, 1, 1), (width,), (width,),
                    (width, width, 3, 3), (width,), (width,),
                    (4 * width, width, 1, 1), (4 * width,), (4 * width,)]
            if b == 0:
                out += [(4 * width, cin, 1, 1), (4 * width,), (4 * width,)]
            cin = 4 * width
    out += [(1000, 2048), (1000,)]
    return out


def bert_large_shapes() -> List[Shape]:
    """BERT-large encoder with pooler: 391 tensors, 335,141,888 parameters."""
    h, f = 1024, 4096
    out: List[Shape] = [(30522, h), (512, h), (2, h), (h,), (h,)]
    for _ in range(24):
        for _ in range(4):
            out += [(h, h), (h,)]
        out += [(h,), (h,), (f, h), (f,), (h, f), (h,), (h,), (h,)]
    out += [(h, h), (h,)]
    return out


def gpt2_xl_shapes() -> List[Shape]:
    """GPT-2 1.5B: 580 tensors, 1,557,611,200 parameters."""
    d, f = 1600, 6400
    out: List[Shape] = [(50257, d), (1024, d)]
    for _ in range(48):
        out += [(d,), (d,), (d, 3 * d), (3 * d,), (d, d), (d,), (d,), (d,), (d, f), (f,), (f, d), (d,)]
    out += [(d,), (d,)]
    return out


def llama7b_shapes() -> List[Shape]:
    """Llama-7B: 291 tensors, 6,738,415,616 parameters."""
    d, f, vocab = 4096, 11008, 32000
    out: List[Shape] = [(vocab, d)]
    for _ in range(32):
        out += [(d, d)] * 4 + [(f, d)] * 2 + [(d, f)] + [(d,)] * 2
    out += [(d,), (vocab, d)]
    return out


def vit_128_32_shapes() -> List[Shape]:
    """ViT-Large/32 deepened from 24 to 128 transformer layers, hidden size unchanged (the paper's
    ViT-128/32, section "Experimental setup"), 224x224 input, 1000 classes: 1,544 tensors,
    1,616,542,696 parameters (the paper's table says 1.64 B; the text does not give the head or
    the input size, the difference is about 1 %)."""
    h, f, patch, tokens = 1024, 4096, 32, (224 // 32) ** 2 + 1
    out: List[Shape] = [(1, 1, h), (1, tokens, h), (h, 3, patch, patch), (h,)]
    for _ in range(128):
        out += [(h,), (h,), (3 * h, h), (3 * h,), (h, h), (h,), (h,), (h,), (f, h), (f,), (h, f), (h,)]
    out += [(h,), (h,), (1000, h), (1000,)]
    return out


@dataclass
class Workload:
    """One benchmark / parity configuration: shapes, value recipe and hyper-parameters."""
    name: str
    shapes: List[Shape]
    kind: str                      # "sgdm" | "adam" | "adamw"
    hyper: dict                    # lr, weight_decay, momentum, dampening, beta1, beta2, eps, step
    seed: int
    grad_bf16: bool = False
    std_theta: float = 0.02
    std_grad: float = 1e-3
    std_m: float = 1e-4
    std_v: float = 1e-6
    zero_frac: float = 0.0         # fraction of gradient elements forced to zero
    outlier_frac: float = 0.0      # fraction of gradient elements multiplied by outlier_scale
    outlier_scale: float = 1e3
    digest_shard: int = 0          # 0: one digest per tensor; else fixed shard length
    masked_fraction: float = 0.0   # selective step/undo on this fraction of the tensors
    extra: dict = field(default_factory=dict)

    @property
    def n_params(self) -> int:
        return sum(numel(s) for s in self.shapes)


_ADAM = dict(lr=1e-3, weight_decay=0.0, beta1=0.9, beta2=0.999, eps=1e-8)


def workloads() -> dict:
    """The five benchmark configurations, smallest first, then the additional SGD-momentum list."""
    return {
        "sgdm_flat_1m": Workload(
            "sgdm_flat_1m", [(1 << 20,)], "sgdm",
            dict(lr=0.1, momentum=0.9, dampening=0.0, weight_decay=1e-4, step=1),
            seed=1, std_m=1e-3, digest_shard=1 << 16),
        "resnet50_adam": Workload(
            "resnet50_adam", resnet50_shapes(), "adam", dict(_ADAM, step=1000), seed=2),
        "bert_large_adamw": Workload(
            "bert_large_adamw", bert_large_shapes(), "adamw", dict(_ADAM, weight_decay=0.01, step=10000), seed=3),
        "gpt2_xl_adamw_bf16g": Workload(
            "gpt2_xl_adamw_bf16g", gpt2_xl_shapes(), "adamw",
            dict(lr=6e-4, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8, step=50000), seed=4, grad_bf16=True),
        # the configuration gives no lr/betas/eps/decay of its own: the GPT-2 values are used
        "llama7b_adamw": Workload(
            "llama7b_adamw", llama7b_shapes(), "adamw",
            dict(lr=6e-4, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8, step=100000), seed=5,
            zero_frac=0.10, outlier_frac=0.01, masked_fraction=0.5),
        # beyond the five: the paper trains its ViT-128/32 (and Wide-ResNet-50) with SGD-momentum
        "vit_128_32_sgdm": Workload(
            "vit_128_32_sgdm", vit_128_32_shapes(), "sgdm",
            dict(lr=0.1, momentum=0.9, dampening=0.0, weight_decay=1e-4, step=1), seed=6, std_m=1e-3,
            masked_fraction=0.5),
    }


def padded_extent(nbytes: int) -> int:
    """Bytes from the start of one buffer to the start of the next in the "padded" layout: the size
    rounded up to 8 KiB, plus 2 KiB.  Consecutive buffers are then an odd multiple of 2 KiB apart, so
    theta, g, m, v of a tensor start in four different quarters of an 8 KiB window instead of at the
    same address modulo 8 KiB -- the placement in which the memory system serves the same tile of all
    four streams from the same place (measured: 5-10 % slower for tensors of a few MiB, 2-3 % for the
    7B list).  Buffers under 1 MiB are only rounded to 256 B."""
    if nbytes < (1 << 20):
        return (nbytes + 255) // 256 * 256
    return (nbytes + 8191) // 8192 * 8192 + 2048


@dataclass
class State:
    """Tensor lists of one replica: theta, gradient, first moment, second moment (None for SGDM)."""
    theta: List[torch.Tensor]
    grad: List[torch.Tensor]
    m: List[torch.Tensor]
    v: Optional[List[torch.Tensor]]

    def clone(self) -> "State":
        c = lambda ts: None if ts is None else [t.clone() for t in ts]
        return State(c(self.theta), c(self.grad), c(self.m), c(self.v))


def make_state(w: Workload, device, shapes: Optional[Sequence[Shape]] = None, with_v: Optional[bool] = None,
               layout: str = "padded") -> State:
    """Draw the workload's state on `device` (same seed and device type => same bits, whatever the
    layout).

    layout says where the tensors are allocated, not what they hold.
      "padded" (default): one arena, theta, g, m, v of a tensor next to each other, tensor after tensor,
          consecutive buffers padded_extent() apart (an odd multiple of 2 KiB);
      "by_tensor": the same order, every buffer an allocation of its own (torch's caching allocator);
      "by_stream": every theta, then every gradient, then every m, then every v;
      "framework": as a training framework allocates (every theta when the model is built, gradients
          in backward order, then m and v of one tensor after the other at the first optimizer step).
    Achieved HBM bandwidth depends on where the four streams lie relative to each other (up to 10 %
    for tensors of a few MiB), so benchmarks state the layout they used."""
    shapes = list(w.shapes if shapes is None else shapes)
    with_v = (w.kind != "sgdm") if with_v is None else with_v
    if layout not in ("by_stream", "by_tensor", "framework", "padded"):
        raise ValueError(f"unknown layout {layout!r}")
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    gdt = torch.bfloat16 if w.grad_bf16 else torch.float32
    sizes = [numel(shp) for shp in shapes]
    new = lambda n, dt=torch.float32: torch.empty(n, dtype=dt, device=dev)
    if layout == "by_stream":
        th = [new(n) for n in sizes]
        gr = [new(n, gdt) for n in sizes]
        mo = [new(n) for n in sizes]
        vo = [new(n) for n in sizes] if with_v else None
    elif layout == "padded":
        # by_tensor order inside one arena; see padded_extent for the distance between consecutive buffers
        slots, off = [], 0
        for n in sizes:
            row = []
            for dt in (torch.float32, gdt, torch.float32) + ((torch.float32,) if with_v else ()):
                row.append((off, n, dt))
                off += padded_extent(n * (2 if dt == torch.bfloat16 else 4))
            slots.append(row)
        arena = torch.empty(max(off, 256), dtype=torch.uint8, device=dev)
        view = lambda o, n, dt: arena[o:o + n * (2 if dt == torch.bfloat16 else 4)].view(dt)
        th = [view(*row[0]) for row in slots]
        gr = [view(*row[1]) for row in slots]
        mo = [view(*row[2]) for row in slots]
        vo = [view(*row[3]) for row in slots] if with_v else None
    elif layout == "framework":
        th = [new(n) for n in sizes]                   # the model is built first,
        gr = [new(n, gdt) for n in reversed(sizes)][::-1]   # gradients appear in backward order,
        mo, vo = [], ([] if with_v else None)          # optimizer state tensor by tensor at the first step
        for n in sizes:
            mo.append(new(n))
            if with_v:
                vo.append(new(n))
    else:
        th, gr, mo, vo = [], [], [], ([] if with_v else None)
        for n in sizes:
            th.append(new(n))
            gr.append(new(n, gdt))
            mo.append(new(n))
            if with_v:
                vo.append(new(n))
    for i, n in enumerate(sizes):                      # draw order: theta, g, m, v, selector; tensor by tensor
        th[i].normal_(0.0, w.std_theta, generator=gen)
        g = new(n).normal_(0.0, w.std_grad, generator=gen) if w.grad_bf16 else gr[i].normal_(0.0, w.std_grad, generator=gen)
        mo[i].normal_(0.0, w.std_m, generator=gen)
        if with_v:
            vo[i].normal_(0.0, w.std_v, generator=gen).abs_()
        if w.zero_frac > 0 or w.outlier_frac > 0:
            r = new(n).uniform_(0.0, 1.0, generator=gen)
            g[r < w.zero_frac] = 0.0
            g[r >= 1.0 - w.outlier_frac] *= w.outlier_scale
            del r
        if w.grad_bf16:
            gr[i].copy_(g)                # round to nearest even; the kernels widen it back exactly
        del g
    return State(th, gr, mo, vo)


def tensor_mask(w: Workload, n_tensors: int) -> List[int]:
    """Seeded choice of which tensors a partial step reaches (the paper's 'marked as updated' set)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed + 1000)
    k = int(round(w.masked_fraction * n_tensors))
    perm = torch.randperm(n_tensors, generator=gen)[:k]
    mask = [0] * n_tensors
    for i in perm.tolist():
        mask[i] = 1
    return mask
