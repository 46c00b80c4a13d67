"""Synthetic workloads: matrix layouts of the five benchmark configurations and
the seeded generators of their gradients and initial right factors.

This module holds inputs only -- none of the method's arithmetic -- so that the
GPU path, the CPU oracle, the tests and the benchmark can all draw the very
same tensors from it.  The paper's experiments (Section 5) use gradients of
ResNet-18, LSTM and transformer models trained on public datasets; those are
not available here, so tensors with the same per-layer shapes and plausible
value distributions stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

F32, BF16 = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                       # position in the list of configurations (1-based seeds)
    layout: Tuple[Tuple[int, int], ...]   # (rows, cols) of every compressed matrix, model order
    rank: int
    bits: int
    block: int
    grad_dtype: int                  # F32 or BF16
    dist: str                        # "normal", "normal_fanin", "laplace", "student_t3"
    scale: float
    lib_seed: int

    @property
    def elements(self) -> int:
        return sum(n * m for n, m in self.layout)

    @property
    def grad_bytes(self) -> int:
        return self.elements * (4 if self.grad_dtype == F32 else 2)

    def model_bytes(self) -> int:
        """HBM bytes of one step under the three-pass model: the gradient, codes and scales
        are read three times, codes and scales written once; P is written, orthonormalised
        in place (read + write) and read twice; Q is read, written and read."""
        G = 4 if self.grad_dtype == F32 else 2
        tot = 0.0
        for n, m in self.layout:
            tot += n * m * (3 * G + 4 * self.bits / 8 + 4 * 4 / self.block) + (5 * n + 3 * m) * self.rank * 4
        return int(tot)


def _resnet18_layout() -> List[Tuple[int, int]]:
    L = [(64, 3 * 7 * 7)]
    L += [(64, 64 * 9)] * 4
    L += [(128, 64 * 9), (128, 128 * 9), (128, 64), (128, 128 * 9), (128, 128 * 9)]
    L += [(256, 128 * 9), (256, 256 * 9), (256, 128), (256, 256 * 9), (256, 256 * 9)]
    L += [(512, 256 * 9), (512, 512 * 9), (512, 256), (512, 512 * 9), (512, 512 * 9)]
    L += [(1000, 512)]
    return L


def _gpt_layout(layers: int, d: int, ffn: int, vocab: int) -> List[Tuple[int, int]]:
    L = [(vocab, d)]
    for _ in range(layers):
        L += [(d, 3 * d), (d, d), (d, ffn), (ffn, d)]
    return L


def _transformer_big_layout() -> List[Tuple[int, int]]:
    d, ffn = 1024, 4096
    L = [(32768, d)]
    for _ in range(6):
        L += [(d, d)] * 4 + [(d, ffn), (ffn, d)]
    for _ in range(6):
        L += [(d, d)] * 8 + [(d, ffn), (ffn, d)]
    return L


WORKLOADS = {
    "tiny": Workload("tiny", 1, ((256, 128),), 2, 8, 64, F32, "normal", 1.0, 0x5EED0001),
    "cnn": Workload("cnn", 2, tuple(_resnet18_layout()), 4, 4, 128, F32, "normal_fanin", 1.0, 0x5EED0002),
    "lm": Workload("lm", 3, tuple(_gpt_layout(12, 768, 3072, 50257)), 4, 4, 128, F32, "laplace", 1e-3,
                   0x5EED0003),
    "translation": Workload("translation", 4, tuple(_transformer_big_layout()), 8, 2, 256, BF16,
                            "normal", 1e-3, 0x5EED0004),
    "large": Workload("large", 5, tuple(_gpt_layout(24, 2048, 8192, 50304)), 32, 4, 128, BF16,
                      "student_t3", 1e-3, 0x5EED0005),
}


def sketch_rows(layout, keep: float) -> List[int]:
    """Table rows per matrix of a count sketch that keeps `keep` table entries per entry of the error
    (Section 5.2 quotes the memory saved: a table of fp16 entries with keep = 0.8 saves 60 % of an fp32
    error vector, keep = 0.2 saves 90 %)."""
    return [max(1, min(n, int(n * keep))) for n, _ in layout]


def random_block_keep(layout, fraction: float) -> List[int]:
    """Coordinates kept per matrix by the random-block gradient compressor: `fraction` of its elements, at
    least one (Section 5.3 uses a tenth: "90 % communication efficiency")."""
    return [max(1, int(n * m * fraction)) for n, m in layout]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, np.uint16).astype(np.uint32) << 16).view(np.float32)


def _draw(rng: np.random.Generator, dist: str, scale: float, n: int, m: int) -> np.ndarray:
    if dist == "normal":
        x = rng.standard_normal((n, m)) * scale
    elif dist == "normal_fanin":
        x = rng.standard_normal((n, m)) * (scale / np.sqrt(m))
    elif dist == "laplace":
        x = rng.laplace(0.0, scale, (n, m))
    elif dist == "student_t3":
        x = rng.standard_t(3.0, (n, m)) * scale
    else:
        raise ValueError(dist)
    return x.astype(np.float32)


def host_gradient(w: Workload, step: int, mat: int, shape=None) -> np.ndarray:
    """Gradient of matrix `mat` at `step`, drawn on the host: float32 array, or uint16 bf16
    bit patterns for bf16 workloads.  `shape` overrides the layout's (for cut-down cases)."""
    n, m = shape if shape is not None else w.layout[mat]
    rng = np.random.Generator(np.random.PCG64([w.index, step, mat]))
    x = _draw(rng, w.dist, w.scale, n, m)
    return x if w.grad_dtype == F32 else f32_to_bf16_bits(x)


def host_q0(w: Workload, mat: int, shape=None, rank=None) -> np.ndarray:
    """Initial right factor Q (cols x rank), iid N(0,1)."""
    _, m = shape if shape is not None else w.layout[mat]
    rng = np.random.Generator(np.random.PCG64([w.index, 999, mat]))
    return rng.standard_normal((m, rank or w.rank)).astype(np.float32)


def graded_panel(n: int, r: int, cond: float, seed: int) -> np.ndarray:
    """An n x r fp32 panel with singular values 1, cond^(-1/(r-1)), ..., 1/cond (geometric) and random
    orthonormal singular vectors on both sides: the left factor P = p Q of a gradient with a decaying spectrum
    after a few warm-started steps looks like this (its condition number is a power of the spectrum's decay)."""
    rng = np.random.default_rng([77, seed, n, r])
    U, _ = np.linalg.qr(rng.standard_normal((n, r)))
    V, _ = np.linalg.qr(rng.standard_normal((r, r)))
    sig = np.asarray([cond ** (-j / max(1, r - 1)) for j in range(r)])
    return np.ascontiguousarray(((U * sig) @ V.T).astype(np.float32))


def decaying_gradient(n: int, m: int, decay: float, noise: float, seed: int, step: int = 0) -> np.ndarray:
    """An n x m fp32 matrix with singular values decay^j on fixed singular vectors (the same for every step) plus
    iid N(0, noise^2) entries that change with the step: a gradient whose leading subspace persists from step
    to step, which is what warm-started subspace iteration locks on to."""
    k = min(n, m, 48)
    rng = np.random.default_rng([78, seed, n, m])
    U, _ = np.linalg.qr(rng.standard_normal((n, k)))
    V, _ = np.linalg.qr(rng.standard_normal((m, k)))
    sig = decay ** np.arange(k)
    g = (U * sig) @ V.T
    g += noise * np.random.default_rng([79, seed, n, m, step]).standard_normal((n, m))
    return np.ascontiguousarray(g.astype(np.float32))


def device_fill_gradients(w: Workload, step: int, flat, offsets) -> None:
    """Fills the flat device gradient buffer `flat` (a torch tensor of the workload's gradient
    dtype) matrix by matrix at the given element offsets, drawing on the device with a torch
    generator seeded from (workload, step).  Same distributions as host_gradient, different
    stream of numbers; used at full model sizes where host generation would take minutes."""
    import torch

    gen = torch.Generator(device=flat.device)
    gen.manual_seed((w.index << 32) ^ (step * 1000003 + 12345))
    for (n, m), off in zip(w.layout, offsets):
        N = n * m
        if w.dist in ("normal", "normal_fanin"):
            sc = w.scale / np.sqrt(m) if w.dist == "normal_fanin" else w.scale
            x = torch.randn(N, device=flat.device, generator=gen) * sc
        elif w.dist == "laplace":
            u = torch.rand(N, device=flat.device, generator=gen) - 0.5
            # inverse CDF; 1 - 2|u| is kept away from 0 (rand() can return exactly 0)
            x = -w.scale * torch.sign(u) * torch.log(torch.clamp(1.0 - 2.0 * u.abs(), min=2.0 ** -24))
        elif w.dist == "student_t3":
            z = torch.randn(N, device=flat.device, generator=gen)
            chi = torch.zeros(N, device=flat.device)
            for _ in range(3):
                chi += torch.randn(N, device=flat.device, generator=gen) ** 2
            x = z / torch.sqrt(chi / 3.0) * w.scale
        else:
            raise ValueError(w.dist)
        flat[off:off + N] = x.to(flat.dtype)


def device_q0(w: Workload, flat, offsets) -> None:
    import torch

    gen = torch.Generator(device=flat.device)
    gen.manual_seed((w.index << 32) ^ 999)
    for (n, m), off in zip(w.layout, offsets):
        flat[off:off + m * w.rank] = torch.randn(m * w.rank, device=flat.device, generator=gen)
