"""Seeded synthetic inputs for the AdaScale step: parameter-list shapes, gradient
generators, lr tables.

This module serves both the HIP path and the CPU oracle and therefore holds none of
the method's arithmetic: it only produces tensors (w_0, v_0, the S gradient buffers
of a step) and the learning-rate table.  Nothing here computes a mean gradient, a
norm, a gain ratio or an update.

The five workloads imitate the *parameter-list shapes* of the model families the
paper trains (Table 1: ResNet-18, ResNet-50, Transformer-base, plus a larger
transformer); no dataset, trained weight or benchmark item is involved.  Gradients
are g_i = signal + noise_i with the signal shared by the S replicas, which is the
structure the gain ratio of Sec. 3.2 (eq. 3) responds to.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
import torch

F32 = 0
BF16 = 1

_ALIGN_BYTES = 256  # start of every tensor inside a flat buffer (allocator-like)
_ROW_ALIGN_BYTES = 2 << 20  # start of every replica's row inside the one gradient allocation


# --------------------------------------------------------------------------- shapes
def _bn(c: int) -> List[Tuple[int, ...]]:
    return [(c,), (c,)]


def resnet18_like() -> List[Tuple[int, ...]]:
    """62 tensors, 11,181,642 elements: 7x7 stem, 4 stages x 2 basic blocks, 10-way FC."""
    t: List[Tuple[int, ...]] = [(64, 3, 7, 7)] + _bn(64)
    cin = 64
    for si, wd in enumerate((64, 128, 256, 512)):
        for blk in range(2):
            t += [(wd, cin if blk == 0 else wd, 3, 3)] + _bn(wd)
            t += [(wd, wd, 3, 3)] + _bn(wd)
            if blk == 0 and si > 0:
                t += [(wd, cin, 1, 1)] + _bn(wd)
        cin = wd
    t += [(10, 512), (10,)]
    return t


def resnet50_like() -> List[Tuple[int, ...]]:
    """161 tensors, 25,557,032 elements: 7x7 stem, [3,4,6,3] bottleneck blocks, 1000-way FC."""
    t: List[Tuple[int, ...]] = [(64, 3, 7, 7)] + _bn(64)
    cin = 64
    for wd, nblk in zip((64, 128, 256, 512), (3, 4, 6, 3)):
        for blk in range(nblk):
            t += [(wd, cin, 1, 1)] + _bn(wd)
            t += [(wd, wd, 3, 3)] + _bn(wd)
            t += [(4 * wd, wd, 1, 1)] + _bn(4 * wd)
            if blk == 0:
                t += [(4 * wd, cin, 1, 1)] + _bn(4 * wd)
            cin = 4 * wd
    t += [(1000, 2048), (1000,)]
    return t


def _attn(dm: int) -> List[Tuple[int, ...]]:
    return [(dm, dm), (dm,)] * 4


def _ffn(dm: int, dff: int) -> List[Tuple[int, ...]]:
    return [(dff, dm), (dff,), (dm, dff), (dm,)]


def transformer_base_like() -> List[Tuple[int, ...]]:
    """257 tensors, 60,524,544 elements: 32000x512 embedding, 6 encoder + 6 decoder layers."""
    dm, dff = 512, 2048
    t: List[Tuple[int, ...]] = [(32000, dm)]
    for _ in range(6):
        t += _attn(dm) + _ffn(dm, dff) + _bn(dm) * 2
    for _ in range(6):
        t += _attn(dm) + _attn(dm) + _ffn(dm, dff) + _bn(dm) * 3
    t += _bn(dm) * 2
    return t


def transformer_350m_like() -> List[Tuple[int, ...]]:
    """387 tensors, 351,463,424 elements: 48000x1024 embedding, 24 blocks of width 1024."""
    dm, dff = 1024, 4096
    t: List[Tuple[int, ...]] = [(48000, dm)]
    for _ in range(24):
        t += _attn(dm) + _ffn(dm, dff) + _bn(dm) * 2
    t += _bn(dm)
    return t


# ------------------------------------------------------------------------ lr tables
def lr_constant(value: float, length: int = 1) -> np.ndarray:
    return np.full((length,), value, dtype=np.float32)


def lr_step_decay(lr0: float, length: int, drops: Sequence[float] = (0.5, 0.75),
                  factor: float = 0.1, warmup: int = 0, warmup_from: float = 0.0) -> np.ndarray:
    """Step decay (App. B.1 form): lr0 * factor^(number of drop points passed), with an
    optional linear warm-up over the first `warmup` entries."""
    j = np.arange(length, dtype=np.float64)
    lr = np.full(length, lr0, dtype=np.float64)
    for frac in drops:
        lr = np.where(j >= int(round(frac * length)), lr * factor, lr)
    if warmup > 0:
        ramp = warmup_from + (lr0 - warmup_from) * j / warmup
        lr = np.where(j < warmup, ramp, lr)
    return lr.astype(np.float32)


def lr_exponential_decay(lr0: float, length: int, decay: float) -> np.ndarray:
    """Exponential decay (App. B.1 form): lr0 * decay^(t / T)."""
    j = np.arange(length, dtype=np.float64)
    return (lr0 * decay ** (j / length)).astype(np.float32)


def lr_inverse_sqrt(lr0: float, length: int, warm: int = 100) -> np.ndarray:
    j = np.arange(length, dtype=np.float64)
    return (lr0 * np.sqrt(warm / np.maximum(j + 1, warm))).astype(np.float32)


# ------------------------------------------------------------------------- workload
@dataclass
class Workload:
    name: str
    shapes: List[Tuple[int, ...]]
    S: int
    grad_dtype: int              # F32 | BF16
    momentum: float
    weight_decay: float
    theta: float                 # < 0: library default max(1 - S/1000, 0)
    eps: float
    lr_table: np.ndarray         # float32 [L]
    steps: int
    seed: int
    recipe: str                  # which gradient generator below
    numel: List[int] = field(init=False)

    def __post_init__(self) -> None:
        self.numel = [int(np.prod(s)) for s in self.shapes]

    @property
    def d(self) -> int:
        return sum(self.numel)

    @property
    def n_tensors(self) -> int:
        return len(self.numel)

    @property
    def grad_bytes(self) -> int:
        return 4 if self.grad_dtype == F32 else 2

    def torch_grad_dtype(self) -> torch.dtype:
        return torch.float32 if self.grad_dtype == F32 else torch.bfloat16


def config(i: int) -> Workload:
    """The five configurations of the benchmark definition, numbered 1..5."""
    if i == 1:
        return Workload("cfg1_flat_1M_S4", [(1_000_000,)], 4, F32, 0.9, 0.0, 0.9, 1e-6,
                        lr_constant(0.1), 10, 0, "shared_fresh_signal")
    if i == 2:
        return Workload("cfg2_resnet18like_S8", resnet18_like(), 8, F32, 0.9, 5e-4, -1.0, 1e-6,
                        lr_step_decay(0.1, 800), 200, 0, "decaying_signal")
    if i == 3:
        return Workload("cfg3_resnet50like_S16", resnet50_like(), 16, F32, 0.9, 1e-4, -1.0, 1e-6,
                        lr_step_decay(0.1, 800, warmup=40, warmup_from=0.01), 100, 0,
                        "per_tensor_scale")
    if i == 4:
        return Workload("cfg4_transformerbase_like_S32_bf16", transformer_base_like(), 32, BF16,
                        0.99, 0.0, -1.0, 1e-6, lr_inverse_sqrt(0.01, 3200), 100, 0,
                        "per_tensor_variance")
    if i == 5:
        return Workload("cfg5_transformer350M_like_S64_bf16", transformer_350m_like(), 64, BF16,
                        0.9, 0.0, -1.0, 1e-6, lr_constant(0.01, 3200), 50, 0, "student_t_snr_sweep")
    raise ValueError(f"no config {i}")


def custom(shapes: Sequence[Tuple[int, ...]], S: int, grad_dtype: int = F32, momentum: float = 0.9,
           weight_decay: float = 0.0, theta: float = -1.0, eps: float = 1e-6,
           lr_table: np.ndarray | None = None, steps: int = 4, seed: int = 0,
           recipe: str = "shared_fresh_signal", name: str = "custom") -> Workload:
    if lr_table is None:
        lr_table = lr_constant(0.1)
    return Workload(name, [tuple(s) for s in shapes], S, grad_dtype, momentum, weight_decay, theta,
                    eps, np.asarray(lr_table, dtype=np.float32), steps, seed, recipe)


# --------------------------------------------------------------------- flat buffers
def layout(numel: Sequence[int], elem_bytes: int, align_bytes: int = _ALIGN_BYTES,
           skew_elems: int = 0) -> Tuple[List[int], int]:
    """Element offsets of each tensor inside one flat buffer and the buffer length.
    `skew_elems` shifts every tensor start by that many elements (to build buffers whose
    tensors are only element-aligned)."""
    a = max(1, align_bytes // elem_bytes)
    offs, pos = [], 0
    for n in numel:
        pos = (pos + a - 1) // a * a
        offs.append(pos + skew_elems)
        pos += n + skew_elems
    return offs, pos


def views(flat: torch.Tensor, numel: Sequence[int], offs: Sequence[int]) -> List[torch.Tensor]:
    return [flat[o:o + n] for n, o in zip(numel, offs)]


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _fill_by_tensor(wl: Workload, offs, total, values: np.ndarray, device) -> torch.Tensor:
    """Flat fp32 vector holding values[k] over tensor k's extent (0 in the padding)."""
    out = torch.zeros(total, dtype=torch.float32, device=device)
    for n, o, s in zip(wl.numel, offs, values):
        out[o:o + n] = float(s)
    return out


class Inputs:
    """Owns the flat device buffers of one workload: w, v (fp32) and S gradient buffers.

    All randomness is drawn with torch generators seeded from (seed, step, replica);
    both consumers read the same bits out of these buffers.
    """

    # What `poison` puts into every element of the flat buffers that belongs to no tensor: a NaN
    # with this bit pattern in w and v, plain NaNs in the gradient buffers.
    SENTINEL_BITS = 0x7FC0ABCD

    def __init__(self, wl: Workload, device: str | torch.device = "cpu", skew_elems: int = 0,
                 one_allocation: bool = True, poison: bool = False):
        """`one_allocation`: the S gradient buffers are rows of one [S, length] allocation, the
        layout a gathered set of per-replica gradients has (False: one allocation per replica).
        `poison`: the elements between tensors (and between gradient rows) hold NaNs instead of
        zeros, so a consumer that reads outside a tensor's extent gets a NaN into its sums, and
        `padding_intact()` tells whether one has written there."""
        self.wl, self.device = wl, torch.device(device)
        self.poison = poison
        self.offs32, self.len32 = layout(wl.numel, 4, skew_elems=skew_elems)
        self.offs_g, self.len_g = layout(wl.numel, wl.grad_bytes, skew_elems=skew_elems)
        dev = self.device
        self.w_flat = torch.zeros(self.len32, dtype=torch.float32, device=dev)
        self.v_flat = torch.zeros(self.len32, dtype=torch.float32, device=dev)
        tmp = torch.randn(self.len32, generator=_gen(dev, wl.seed * 7919 + 17), device=dev) * 0.02
        for n, o in zip(wl.numel, self.offs32):
            self.w_flat[o:o + n] = tmp[o:o + n]
        del tmp
        if one_allocation:
            # rows start on 2 MiB boundaries once they are that long (256 bytes for the small shapes)
            nbytes = self.len_g * wl.grad_bytes
            a = _ROW_ALIGN_BYTES if nbytes >= _ROW_ALIGN_BYTES else _ALIGN_BYTES
            row = (nbytes + a - 1) // a * a // wl.grad_bytes
            self.g_all = torch.full((max(1, wl.S * row),), float("nan") if poison else 0.0,
                                    dtype=wl.torch_grad_dtype(), device=dev)
            self.g_flat = [self.g_all[i * row: i * row + self.len_g] for i in range(wl.S)]
        else:
            self.g_flat = [torch.zeros(self.len_g, dtype=wl.torch_grad_dtype(), device=dev)
                           for _ in range(wl.S)]
        if poison:
            pad = self._pad_mask32() == 0
            self.w_flat.view(torch.int32)[pad] = self.SENTINEL_BITS
            self.v_flat.view(torch.int32)[pad] = self.SENTINEL_BITS
        self.w = views(self.w_flat, wl.numel, self.offs32)
        self.v = views(self.v_flat, wl.numel, self.offs32)
        self.g = [views(f, wl.numel, self.offs_g) for f in self.g_flat]
        self._u = None        # fixed direction (recipes with a persistent signal)
        self._scale = None    # per-element scale vector

    # -- helpers --------------------------------------------------------------
    def _fixed_u(self) -> torch.Tensor:
        if self._u is None:
            self._u = torch.randn(self.len_g, generator=_gen(self.device, self.wl.seed * 7919 + 29),
                                  device=self.device)
        return self._u

    def _per_tensor_scale(self) -> torch.Tensor:
        if self._scale is None:
            wl = self.wl
            rng = np.random.default_rng(wl.seed)
            if wl.recipe == "per_tensor_scale":          # s_k log-uniform in [1e-4, 1e-1]
                s = 10.0 ** rng.uniform(-4.0, -1.0, size=wl.n_tensors)
            else:                                        # s_k^2 log-uniform in [1e-6, 1e-2]
                s = np.sqrt(10.0 ** rng.uniform(-6.0, -2.0, size=wl.n_tensors))
            self._scale = _fill_by_tensor(wl, self.offs_g, self.len_g, s, self.device)
        return self._scale

    def _noise(self, step: int, i: int) -> torch.Tensor:
        return torch.randn(self.len_g, generator=_gen(self.device, self.wl.seed + 1000 * step + i + 1),
                           device=self.device)

    def signal_amplitude(self, step: int) -> float:
        wl = self.wl
        if wl.recipe == "decaying_signal":               # 1.0 -> 0.05 geometrically over the run
            return float(0.05 ** (step / max(1, wl.steps - 1)))
        if wl.recipe == "student_t_snr_sweep":
            # amplitude that makes the signal-to-noise ratio sweep so the gain visits
            # the whole range (1, S): target ratio rises log-uniformly 1.05 -> 60
            r = 1.05 * (60.0 / 1.05) ** (step / max(1, wl.steps - 1))
            return math.sqrt(3.0 * (wl.S - r) / (wl.S * (r - 1.0)))
        return 1.0

    # -- the gradient generator ----------------------------------------------
    def fill_grads(self, step: int) -> None:
        """Overwrite the S gradient buffers with the gradients of iteration `step`."""
        wl, dev = self.wl, self.device
        rec = wl.recipe
        if rec == "shared_fresh_signal":                 # m_t ~ N(0, 0.1^2) fresh each step
            m = torch.randn(self.len_g, generator=_gen(dev, wl.seed + 1000 * step), device=dev) * 0.1
            for i in range(wl.S):
                self.g_flat[i].copy_(m + self._noise(step, i))
        elif rec == "decaying_signal":
            m = self._fixed_u() * self.signal_amplitude(step)
            for i in range(wl.S):
                self.g_flat[i].copy_(m + self._noise(step, i))
        elif rec in ("per_tensor_scale", "per_tensor_variance"):
            c = 0.25 if rec == "per_tensor_scale" else 0.2
            sc = self._per_tensor_scale()
            m = self._fixed_u() * c
            for i in range(wl.S):
                self.g_flat[i].copy_(sc * (m + self._noise(step, i)))
        elif rec == "student_t_snr_sweep":
            m = self._fixed_u() * self.signal_amplitude(step)
            for i in range(wl.S):
                gen = _gen(dev, wl.seed + 1000 * step + i + 1)
                z = torch.randn(self.len_g, generator=gen, device=dev)
                chi = torch.zeros_like(z)
                for _ in range(3):
                    chi.addcmul_(t := torch.randn(self.len_g, generator=gen, device=dev), t)
                z.div_(chi.div_(3.0).sqrt_())             # Student-t, nu = 3
                self.g_flat[i].copy_(z.add_(m))
                del z, chi
        elif rec == "identical":                         # all replicas equal (zero variance)
            m = torch.randn(self.len_g, generator=_gen(dev, wl.seed + 1000 * step), device=dev)
            for i in range(wl.S):
                self.g_flat[i].copy_(m)
        elif rec == "zero_mean":                         # pure noise
            for i in range(wl.S):
                self.g_flat[i].copy_(self._noise(step, i))
        elif rec == "zeros":
            for i in range(wl.S):
                self.g_flat[i].zero_()
        else:
            raise ValueError(f"unknown recipe {rec}")
        # padding between tensors: zero, so that flat-buffer consumers see no garbage -- or, with
        # `poison`, NaN, so that a read outside a tensor's extent shows in the consumer's sums
        if self.len_g != wl.d:
            mask = self._pad_mask()
            for i in range(wl.S):
                self.g_flat[i].mul_(mask.to(self.g_flat[i].dtype))
                if self.poison:
                    self.g_flat[i][mask == 0] = float("nan")

    def _pad_mask(self) -> torch.Tensor:
        if not hasattr(self, "_mask"):
            self._mask = _fill_by_tensor(self.wl, self.offs_g, self.len_g,
                                         np.ones(self.wl.n_tensors), self.device)
        return self._mask

    def _pad_mask32(self) -> torch.Tensor:
        if not hasattr(self, "_mask32"):
            self._mask32 = _fill_by_tensor(self.wl, self.offs32, self.len32,
                                           np.ones(self.wl.n_tensors), self.device)
        return self._mask32

    def grad_bits(self) -> List[torch.Tensor]:
        """Copies of the gradient allocations as raw integers (to check that nobody wrote to them)."""
        bufs = [self.g_all] if hasattr(self, "g_all") else self.g_flat
        return [b.view(torch.int32 if b.dtype == torch.float32 else torch.int16).clone() for b in bufs]

    def padding_intact(self) -> bool:
        """With `poison`: does every element of w and v outside the tensors still hold the sentinel?"""
        pad = self._pad_mask32() == 0
        return all(bool((f.view(torch.int32)[pad] == self.SENTINEL_BITS).all()) for f in (self.w_flat, self.v_flat))
