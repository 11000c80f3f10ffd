"""Seeded synthetic inputs and the named workloads.

This module holds no arithmetic of the method: it only describes workloads (sizes and
hyper-parameters) and draws the random tensors the method consumes -- the common initial
model and the per-worker stochastic gradients -- so that the GPU path and the CPU oracle
can be fed identical bits.  The gradients stand in for the ones the paper's networks
(a Wide-ResNet on CIFAR-100, a ResNet-50 on ImageNet, Section 5.1) would produce; the
update path is data-oblivious, so i.i.d. normal values of the stated variance exercise it
exactly as real gradients would.
"""
from dataclasses import dataclass, replace
import math

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    d: int            # parameters per worker
    W: int            # workers n (Section 3: n workers; Section 5.1 uses 8)
    block: int        # elements per GRBS block
    R_step: int       # per-iteration compressor ratio (paper's R_C2)
    R_reset: int      # error-reset compressor ratio (paper's R_C1)
    H: int            # error-reset interval
    lr: float
    momentum: float
    x_var: float      # variance of the common initial model
    g_var: float      # variance of the synthetic gradients
    seed: int
    steps: int

    @property
    def B(self) -> int:
        return -(-self.d // self.block)

    @property
    def ld(self) -> int:
        """Row stride used for device buffers: d rounded up to 1024 elements, so that every worker's
        row starts on a 4 KiB boundary (measured 4 % faster than rows that start on odd 256-byte
        boundaries: a wavefront's 1 KiB access then never straddles an interleave unit)."""
        return -(-self.d // 1024) * 1024


WORKLOADS = {
    "tiny": Workload("tiny", 65_536, 4, 256, 8, 4, 4, 0.1, 0.9, 1e-2, 1e-2, 0, 20),
    "small_cnn": Workload("small_cnn", 855_770, 8, 512, 32, 8, 8, 0.1, 0.9, 1e-2, 1e-3, 1, 200),
    "large_cnn": Workload("large_cnn", 25_557_032, 8, 1024, 256, 16, 32, 0.1, 0.9, 1e-2, 1e-3, 2, 200),
    "transformer": Workload("transformer", 335_000_000, 8, 4096, 512, 32, 64, 1e-3, 0.9, 1e-2, 1e-4, 4, 20),
}


def sweep_workloads():
    """Compression sweep at the large-CNN size: R_step x block x H, 50 steps each."""
    base = WORKLOADS["large_cnn"]
    out = []
    for H in (4, 32):
        for block in (64, 256, 1024, 4096):
            for R_step in (2, 8, 32, 256, 1024):
                out.append(replace(base, name=f"sweep_R{R_step}_bs{block}_H{H}", block=block,
                                   R_step=R_step, R_reset=16, H=H, seed=3, steps=50))
    return out


# Appendix C, Table 4 ("Compressor configurations"), optimizer CSER: for each overall compression ratio the tuned
# (R_C2, R_C1, H) = (per-iteration compressor, error-reset compressor, reset interval).  Section 5.1:
# overall = 1 / (1/R_C2 + 1/(R_C1 H)).
TABLE4_CSER = ((2, 4, 2, 2), (4, 8, 2, 4), (8, 16, 2, 8), (16, 32, 8, 4), (32, 64, 8, 8), (64, 128, 8, 16),
               (128, 256, 4, 64), (256, 512, 16, 32), (512, 1024, 8, 128), (1024, 2048, 32, 64))


def table4_workloads():
    """The ten CSER rows of the paper's Table 4 at the large-CNN size (block 1024, 8 workers), long enough for at
    least two error resets each."""
    base = WORKLOADS["large_cnn"]
    return [replace(base, name=f"table4_R{overall}", R_step=r_step, R_reset=r_reset, H=H, seed=5, steps=max(64, 2 * H))
            for overall, r_step, r_reset, H in TABLE4_CSER]


def _generator(device, *key) -> torch.Generator:
    """A torch generator on `device`, seeded by mixing the integers in `key` (splitmix-style)."""
    s = 0x9E3779B97F4A7C15
    for k in key:
        s = (s ^ (int(k) & 0xFFFFFFFFFFFFFFFF)) * 0xBF58476D1CE4E5B9 & 0xFFFFFFFFFFFFFFFF
        s ^= s >> 31
    gen = torch.Generator(device=device)
    gen.manual_seed(s & 0x7FFFFFFFFFFFFFFF)
    return gen


def initial_model_row(wl: Workload, device="cpu") -> torch.Tensor:
    """The common starting point x_hat_0 ~ N(0, x_var), one row of d float32 values."""
    gen = _generator(device, wl.seed, 0xA11CE)
    return torch.randn(wl.d, generator=gen, device=device, dtype=torch.float32) * math.sqrt(wl.x_var)


def initial_model(wl: Workload, device="cpu", ld=None) -> torch.Tensor:
    """x[W][ld] with the same x_hat_0 in every row (Algorithm 3's initialisation); padding is zero."""
    ld = wl.ld if ld is None else ld
    x = torch.zeros(wl.W, ld, device=device, dtype=torch.float32)
    x[:, :wl.d] = initial_model_row(wl, device)
    return x


def gradient(wl: Workload, t: int, device="cpu", ld=None, out=None) -> torch.Tensor:
    """g[W][ld] for iteration t (counted from 1): i.i.d. N(0, g_var) per worker, padding zero."""
    ld = wl.ld if ld is None else ld
    if out is None:
        out = torch.zeros(wl.W, ld, device=device, dtype=torch.float32)
    gen = _generator(out.device, wl.seed, 0x6EAD, t)
    out[:, :wl.d].normal_(0.0, math.sqrt(wl.g_var), generator=gen)
    return out
