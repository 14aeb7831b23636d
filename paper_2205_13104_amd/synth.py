"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds NO arithmetic of the method: it only draws checkpoints and gradients.
It serves the tests (oracle side and HIP side alike) and the benchmark.  Tensors are
produced with torch's seeded generators on the requested device (CPU or the GPU); the
side that did not generate them receives a copy, so both sides always see identical bits.

The paper averages checkpoints of one training trajectory (one per epoch, n = 60..100,
Sec. 5.1) or of several fine-tuning runs from one pre-trained model (Sec. 5.2) and notes
that such weights are almost collinear (pairwise cosine ~0.99, Sec. 5.3.4).  The recipes
below reproduce the SHAPES (D = parameter count, n = number of checkpoints) and that
correlation structure; none of the paper's data sets or trained weights is involved.

Layout: a D x n matrix is a tensor of shape (n, ld), ld >= D, row j = checkpoint j,
elements [D, ld) of every row are zero padding.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch


def padded_ld(D: int, mult: int = 128) -> int:
    return (D + mult - 1) // mult * mult


@dataclass(frozen=True)
class Workload:
    name: str
    D: int
    n: int
    kind: str            # "trajectory" | "finetune"
    decay: float = 0.97  # per-checkpoint decay of the step noise (trajectory)
    drift: float = 0.3   # weight of the shared drift direction (trajectory)
    sigma_g: float = 1e-2
    lr: float = 0.1
    steps: int = 1000
    k: int = 1


# The five benchmark configurations (shapes: ResNet-18 / ResNet-50 / ViT-B/16 parameter counts).
WORKLOADS = {
    "tiny": Workload("tiny", 1_000_000, 10, "trajectory", decay=0.9, drift=0.5, sigma_g=1e-2, steps=100),
    "cifar_resnet18": Workload("cifar_resnet18", 11_173_962, 100, "trajectory", sigma_g=1e-2),
    "imagenet_resnet50": Workload("imagenet_resnet50", 25_557_032, 100, "trajectory", sigma_g=5e-3),
    "vit_b16_finetune": Workload("vit_b16_finetune", 86_567_656, 20, "finetune", sigma_g=1e-2, k=8),
    "large": Workload("large", 350_000_000, 128, "trajectory", sigma_g=1e-2, steps=200),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def trajectory(D: int, n: int, decay: float, drift: float, seed: int = 0, device="cpu",
               ld: Optional[int] = None, out: Optional[torch.Tensor] = None,
               w0_std: float = 0.05, step_std: float = 1e-3) -> torch.Tensor:
    """Checkpoints of a synthetic training trajectory, fp32, shape (n, ld).

    w_0 ~ N(0, w0_std^2);  c ~ N(0, step_std^2) is one fixed drift direction;
    w_i = w_{i-1} + drift * c + N(0, (step_std * decay^i)^2),  i = 1 .. n-1.
    Row i of the result is w_i.  The rows are nearly collinear (ill-conditioned)."""
    ld = padded_ld(D) if ld is None else ld
    gen = _gen(seed, device)
    W = torch.zeros((n, ld), dtype=torch.float32, device=device) if out is None else out
    assert W.shape == (n, ld) and W.dtype == torch.float32
    if out is not None:
        W[:, D:].zero_()
    W[0, :D] = torch.randn(D, generator=gen, device=device, dtype=torch.float32) * w0_std
    c = torch.randn(D, generator=gen, device=device, dtype=torch.float32) * step_std
    for i in range(1, n):
        noise = torch.randn(D, generator=gen, device=device, dtype=torch.float32)
        noise *= step_std * (decay ** i)
        noise.add_(c, alpha=drift)
        torch.add(W[i - 1, :D], noise, out=W[i, :D])
    return W


def trajectory_panel(rows: int, n: int, decay: float, drift: float, seed: int, r0: int, out: torch.Tensor,
                     w0_std: float = 0.05, step_std: float = 1e-3) -> torch.Tensor:
    """Rows [r0, r0 + rows) of all n checkpoints of a synthetic trajectory, written to out[:, :rows] (fp32, on out's
    device): the recipe of `trajectory`, with every panel drawn from a generator of its own seeded by (seed, r0), so that
    a panel can be produced again at any time without the rest of the matrix -- what a caller does whose checkpoints
    are too large to sit in memory at once (D = 350 M, n = 128 is 179 GB in fp32)."""
    assert out.dtype == torch.float32 and out.shape[0] == n and out.shape[1] >= rows
    gen = _gen(seed * 2_000_003 + 104_729 * (r0 // 2048 + 1), out.device)
    dev = out.device
    out[0, :rows] = torch.randn(rows, generator=gen, device=dev, dtype=torch.float32) * w0_std
    c = torch.randn(rows, generator=gen, device=dev, dtype=torch.float32) * step_std
    for i in range(1, n):
        noise = torch.randn(rows, generator=gen, device=dev, dtype=torch.float32)
        noise *= step_std * (decay ** i)
        noise.add_(c, alpha=drift)
        torch.add(out[i - 1, :rows], noise, out=out[i, :rows])
    return out


def finetune_offsets(D: int, n: int, seed: int = 0, device="cpu", ld: Optional[int] = None,
                     base_std: float = 0.02, offset_std: float = 2e-3,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Checkpoints fine-tuned from one base model: w_i = w_base + N(0, offset_std^2)."""
    ld = padded_ld(D) if ld is None else ld
    gen = _gen(seed, device)
    W = torch.zeros((n, ld), dtype=torch.float32, device=device) if out is None else out
    assert W.shape == (n, ld) and W.dtype == torch.float32
    if out is not None:
        W[:, D:].zero_()
    base = torch.randn(D, generator=gen, device=device, dtype=torch.float32) * base_std
    for i in range(n):
        off = torch.randn(D, generator=gen, device=device, dtype=torch.float32) * offset_std
        torch.add(base, off, out=W[i, :D])
    return W


def checkpoints(wl: Workload, seed: int = 0, device="cpu", D: Optional[int] = None,
                n: Optional[int] = None, ld: Optional[int] = None) -> torch.Tensor:
    """Checkpoints of workload `wl`, optionally at a reduced D / n (same recipe)."""
    D = wl.D if D is None else D
    n = wl.n if n is None else n
    if wl.kind == "trajectory":
        return trajectory(D, n, wl.decay, wl.drift, seed=seed, device=device, ld=ld)
    return finetune_offsets(D, n, seed=seed, device=device, ld=ld)


def gradient(D: int, sigma: float, seed: int, step: int = 0, device="cpu", k: int = 1,
             ldg: Optional[int] = None) -> torch.Tensor:
    """k synthetic gradients ~ N(0, sigma^2), fp32, shape (D,) for k == 1 else (k, ldg)."""
    gen = _gen(seed * 1_000_003 + 7919 * (step + 1), device)
    if k == 1 and ldg is None:
        return torch.randn(D, generator=gen, device=device, dtype=torch.float32) * sigma
    ldg = D if ldg is None else ldg
    G = torch.zeros((k, ldg), dtype=torch.float32, device=device)
    for c in range(k):
        G[c, :D] = torch.randn(D, generator=gen, device=device, dtype=torch.float32) * sigma
    return G


# --------------------------------------------------------------------------- layer structure (Sec. 4.5)
def _bn(c):
    return [c, c]                                   # scale and shift of one normalisation layer


def resnet_bottleneck_sizes(blocks=(3, 4, 6, 3), classes=1000):
    """Sizes of the parameter tensors, in definition order, of a bottleneck residual network with a
    7x7 stem (stage widths 64/128/256/512, expansion 4).  blocks = (3, 4, 6, 3) is the ResNet-50
    shape: 161 tensors, 25,557,032 parameters -- convolutions next to 64-element normalisation
    vectors, which is what makes the layer-wise reduction ragged."""
    sizes = [64 * 3 * 7 * 7] + _bn(64)
    cin = 64
    for stage, nb in enumerate(blocks):
        p = 64 << stage
        for b in range(nb):
            sizes += [cin * p] + _bn(p) + [p * p * 9] + _bn(p) + [p * 4 * p] + _bn(4 * p)
            if b == 0:
                sizes += [cin * 4 * p] + _bn(4 * p)     # projection shortcut
            cin = 4 * p
    return sizes + [cin * classes, classes]


def resnet_basic_sizes(blocks=(2, 2, 2, 2), classes=10):
    """Same for a basic-block residual network with a 3x3 stem (the CIFAR ResNet-18 shape:
    62 tensors, 11,173,962 parameters at 10 classes)."""
    sizes = [64 * 3 * 9] + _bn(64)
    cin = 64
    for stage, nb in enumerate(blocks):
        p = 64 << stage
        for b in range(nb):
            sizes += [cin * p * 9] + _bn(p) + [p * p * 9] + _bn(p)
            if cin != p:
                sizes += [cin * p] + _bn(p)
            cin = p
    return sizes + [cin * classes, classes]


def random_layer_sizes(D: int, L: int, seed: int = 0):
    """L layer sizes that add up to D, log-uniform between tiny and large, a few of them empty."""
    gen = _gen(seed, "cpu")
    wgt = torch.exp(torch.rand(L, generator=gen, dtype=torch.float64) * 9.0)
    wgt[torch.rand(L, generator=gen) < 0.05] = 0.0
    if float(wgt.sum()) == 0.0:
        wgt[0] = 1.0
    cuts = torch.floor(torch.cumsum(wgt, 0) / wgt.sum() * D).to(torch.int64)
    cuts[-1] = D
    prev = torch.cat([torch.zeros(1, dtype=torch.int64), cuts[:-1]])
    return [int(x) for x in (cuts - prev)]


def layer_offsets(sizes) -> torch.Tensor:
    """Offsets (L+1 int64 values, CPU): layer l covers elements [off[l], off[l+1])."""
    off = torch.zeros(len(sizes) + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.tensor(list(sizes), dtype=torch.int64), 0)
    return off


def workload_layers(name: str) -> torch.Tensor:
    """Layer offsets of a benchmark workload: the architecture's own tensors where the parameter
    count identifies it, otherwise 150 seeded ragged layers."""
    wl = WORKLOADS[name]
    if name == "imagenet_resnet50":
        sizes = resnet_bottleneck_sizes()
    elif name == "cifar_resnet18":
        sizes = resnet_basic_sizes()
    else:
        sizes = random_layer_sizes(wl.D, 150 if wl.D > 10_000_000 else 12, seed=11)
    off = layer_offsets(sizes)
    assert int(off[-1]) == wl.D, (name, int(off[-1]), wl.D)
    return off
