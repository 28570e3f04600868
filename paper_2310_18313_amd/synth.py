"""Seeded synthetic inputs: tensor layouts and gradient / weight generators.

This module holds none of the method's arithmetic (no scaling rule, no FP8/FP16 encoding, no
optimizer maths).  It only lays tensors out in a flat buffer and fills bf16 buffers with random
numbers, so that the HIP path and the CPU oracle can be fed exactly the same bits.

Layouts follow the GPT shapes of the paper's model table (Sec. 3.1.2, Tab. 1: hidden size and
layer count of the 125M / 7B / 13B / 175B models, sequence length 2048) with a Megatron-style
tensor list per layer.  The gradients stand in for the paper's real training gradients, which
need its dataset and cluster.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

ALIGN = 256  # element alignment of every tensor start in the flat buffers


@dataclass
class Layout:
    names: List[str]
    numels: List[int]
    offsets: List[int] = field(default_factory=list)
    total: int = 0  # elements of the flat buffer, padding included

    def __post_init__(self):
        off = 0
        self.offsets = []
        for n in self.numels:
            self.offsets.append(off)
            off += (n + ALIGN - 1) // ALIGN * ALIGN
        self.total = max(off, ALIGN)

    @property
    def n_tensors(self) -> int:
        return len(self.numels)

    @property
    def n_params(self) -> int:
        return int(sum(self.numels))

    def tensors(self) -> List[Tuple[int, int]]:
        return list(zip(self.offsets, self.numels))

    def prefix(self, max_params: int) -> "Layout":
        """The leading tensors whose parameter count stays within max_params (at least one)."""
        names, numels, acc = [], [], 0
        for nm, n in zip(self.names, self.numels):
            if names and acc + n > max_params:
                break
            names.append(nm)
            numels.append(n)
            acc += n
        return Layout(names, numels)


def flat_layout(n: int) -> Layout:
    return Layout(["flat"], [n])


def gpt_layout(hidden: int, layers: int, ffn: int, vocab: int, pos: int = 0) -> Layout:
    h, f = hidden, ffn
    names, numels = [], []

    def add(nm, n):
        names.append(nm)
        numels.append(n)

    if vocab:
        add("emb", vocab * h)
    if pos:
        add("pos", pos * h)
    for l in range(layers):
        p = f"l{l}."
        add(p + "ln1.w", h); add(p + "ln1.b", h)
        add(p + "qkv.w", 3 * h * h); add(p + "qkv.b", 3 * h)
        add(p + "proj.w", h * h); add(p + "proj.b", h)
        add(p + "ln2.w", h); add(p + "ln2.b", h)
        add(p + "fc1.w", f * h); add(p + "fc1.b", f)
        add(p + "fc2.w", h * f); add(p + "fc2.b", h)
    if vocab:
        add("lnf.w", h); add("lnf.b", h)
    return Layout(names, numels)


@dataclass
class Workload:
    name: str
    layout: Layout
    lr: float
    grad_kind: str = "normal"          # "normal" | "student_t"
    sigma: Optional[float] = 1e-4      # None: per-tensor log-uniform in [1e-5, 1e-2]
    steps: int = 1
    hist_window: int = 1
    ramp_steps: int = 1000


def workload(name: str) -> Workload:
    """The five synthetic configurations (shapes from Tab. 1 of the paper, see module docstring)."""
    if name == "flat1m":
        return Workload(name, flat_layout(1 << 20), lr=1e-4, sigma=1e-3, steps=1)
    if name == "gpt125m":
        return Workload(name, gpt_layout(768, 12, 3072, 50304, pos=2048), lr=6e-4, sigma=None, steps=10)
    if name == "gpt7b":
        return Workload(name, gpt_layout(4096, 32, 16384, 50304), lr=3e-4, sigma=1e-4, steps=5, hist_window=4)
    if name == "gpt13b":
        return Workload(name, gpt_layout(5120, 40, 20480, 50304), lr=3e-4, sigma=1e-4, steps=20)
    if name == "gpt175b_layer":
        return Workload(name, gpt_layout(12288, 1, 49152, 0), lr=3e-5, grad_kind="student_t",
                        sigma=1e-4, steps=100, ramp_steps=20)
    if name == "tiny":  # a few ragged tensors for quick checks
        return Workload(name, Layout(["a", "b", "c", "d", "e", "f"], [70001, 1, 4096, 333, 0, 16385]),
                        lr=1e-3, sigma=None, steps=3)
    raise KeyError(name)


def per_tensor_sigma(wl: Workload, seed: int) -> np.ndarray:
    n = wl.layout.n_tensors
    if wl.sigma is not None:
        return np.full(n, wl.sigma, dtype=np.float64)
    rng = np.random.default_rng(seed)
    return 10.0 ** rng.uniform(-5.0, -2.0, n)


def _gen(device, seed: int, step: int, index: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed << 32) + (step << 16) + index)
    return g


_PIECE = 1 << 26  # generate large tensors piecewise to bound the fp32 temporaries


def fill_gradients(dst: torch.Tensor, wl: Workload, seed: int, step: int) -> None:
    """Fill the flat buffer `dst` (bf16, fp16 or fp32) with this step's gradients (padding stays zero)."""
    assert dst.dtype in (torch.bfloat16, torch.float16, torch.float32) and dst.numel() >= wl.layout.total
    sig = per_tensor_sigma(wl, seed)
    dev = dst.device
    for i, (off, n) in enumerate(wl.layout.tensors()):
        if n == 0:
            continue
        g = _gen(dev, seed, step, i)
        for p0 in range(0, n, _PIECE):
            pn = min(_PIECE, n - p0)
            x = torch.randn(pn, generator=g, device=dev, dtype=torch.float32)
            if wl.grad_kind == "student_t":
                # Student-t with 3 degrees of freedom, plus rare large outliers
                z = torch.randn(3, pn, generator=g, device=dev, dtype=torch.float32)
                x = x / torch.sqrt((z * z).mean(dim=0))
                del z
                out = torch.rand(pn, generator=g, device=dev, dtype=torch.float32) < 1e-4
                x = torch.where(out, x * 1e3, x)
            x = x * float(sig[i])
            dst[off + p0: off + p0 + pn] = x.to(dst.dtype)


def fill_weights(dst: torch.Tensor, layout: Layout, seed: int) -> None:
    """Initial weights as bf16: N(0, 0.02); LayerNorm weights 1; biases 0."""
    assert dst.dtype == torch.bfloat16 and dst.numel() >= layout.total
    dev = dst.device
    for i, ((off, n), name) in enumerate(zip(layout.tensors(), layout.names)):
        if n == 0:
            continue
        if name.endswith(".b"):
            dst[off: off + n] = 0
        elif "ln" in name and name.endswith(".w"):
            dst[off: off + n] = 1
        else:
            g = _gen(dev, seed + 7919, 0, i)
            for p0 in range(0, n, _PIECE):
                pn = min(_PIECE, n - p0)
                x = torch.randn(pn, generator=g, device=dev, dtype=torch.float32) * 0.02
                dst[off + p0: off + p0 + pn] = x.to(torch.bfloat16)


def bits16(t: torch.Tensor) -> np.ndarray:
    """Host copy of a 16-bit tensor as uint16 bit patterns."""
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def bits8(t: torch.Tensor) -> np.ndarray:
    return t.detach().view(torch.uint8).cpu().numpy()
