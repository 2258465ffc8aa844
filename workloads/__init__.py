"""Seeded synthetic activation streams for the residual codec.

These stand in for the per-layer activations of the diffusion transformers the
paper measures on (FLUX.1-dev, 28 steps; CogVideoX-2b, 50 steps): unit-variance
tensors that drift by a small step each denoising step, so that the step-wise
residual is a fraction of the activation (Sec. 3.1, Fig. 5 of arxiv 2507.17511).
No model, prompt or dataset item is involved.

This module only makes inputs.  It holds none of the codec's arithmetic and is
the one module the CPU oracle's tests and the HIP path's tests both use.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Sequence

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_tensors: int            # layer tensors per step (K and V count separately)
    n_tokens: int
    n_channels: int
    dtype: str                # "f32" | "bf16"
    bits: Sequence[int]       # cycled over the tensors
    scale: str                # "channel" | "group"
    group: int
    steps: int                # T, warm-up step included: codec steps are 1 .. T-1
    seed: int
    drift_start: float        # sigma of the per-step drift at t = 1
    drift_end: float          # ... and at t = T-1 (linear in between)
    drift_dist: str = "normal"   # "normal" | "student_t3"
    outlier_frac: float = 0.0    # fraction of channels multiplied by outlier_gain
    outlier_gain: float = 1.0

    def bits_of(self, tensor: int) -> int:
        return self.bits[tensor % len(self.bits)]

    def drift_sigma(self, t: int) -> float:
        if self.steps <= 2 or self.drift_start == self.drift_end:
            return self.drift_start
        return self.drift_start + (self.drift_end - self.drift_start) * (t - 1) / (self.steps - 2)

    def scaled(self, **kw) -> "Workload":
        """The same recipe at another size (tests use small ones)."""
        return replace(self, **kw)


# The five configurations of the build's baseline, in order.
CONFIGS = {
    "cfg1_tiny": Workload("cfg1_tiny", 1, 256, 64, "f32", (2,), "channel", 128, 5, 0, 0.05, 0.05),
    "cfg2_flux_patch": Workload("cfg2_flux_patch", 57, 1024, 3072, "bf16", (2,), "channel", 128, 28, 2,
                                0.03, 0.03, outlier_frac=0.01, outlier_gain=20.0),
    "cfg3_kv_fullseq": Workload("cfg3_kv_fullseq", 114, 4096, 3072, "bf16", (1,), "channel", 128, 28, 3,
                                0.02, 0.02),
    "cfg4_video": Workload("cfg4_video", 42, 16384, 3072, "bf16", (4,), "group", 128, 50, 4, 0.1, 0.01),
    "cfg5_batched_mixed": Workload("cfg5_batched_mixed", 57, 4096, 3072, "bf16", (1, 2, 4), "channel", 128, 28, 7,
                                   0.02, 0.02, drift_dist="student_t3"),
}


def to_bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """fp32 tensor -> bf16 tensor (torch's round-to-nearest-even cast)."""
    return x.to(torch.bfloat16)


class ActivationStream:
    """x_0 ~ N(0,1); x_t = x_{t-1} + sigma_t * noise, times a fixed channel gain.

    An fp32 master copy per tensor is kept on ``device``; ``current`` holds the
    tensors in the workload's dtype, which is what the codec is fed.  The
    generator is torch's, seeded once; the call order is fixed (step-major,
    tensor-major within a step), so a (workload, device type) pair always
    yields the same stream.
    """

    def __init__(self, wl: Workload, device: str | torch.device = "cpu"):
        self.wl = wl
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(wl.seed)
        self.t = 0
        shape = (wl.n_tokens, wl.n_channels)
        self.gain = torch.ones(wl.n_channels, dtype=torch.float32, device=self.device)
        n_out = int(round(wl.outlier_frac * wl.n_channels))
        if n_out > 0:
            # a fixed seeded choice of channels, made on the host so it is device independent
            pick = np.random.default_rng(wl.seed).choice(wl.n_channels, size=n_out, replace=False)
            self.gain[torch.as_tensor(np.sort(pick), device=self.device)] = wl.outlier_gain
        self.master: List[torch.Tensor] = [self._normal(shape) for _ in range(wl.n_tensors)]
        self.current: List[torch.Tensor] = [self._emit(m) for m in self.master]

    def _normal(self, shape) -> torch.Tensor:
        return torch.randn(shape, generator=self.gen, device=self.device, dtype=torch.float32)

    def _noise(self, shape) -> torch.Tensor:
        if self.wl.drift_dist == "student_t3":
            # t_3 = Z / sqrt(chi2_3 / 3), chi2_3 the sum of three squared normals
            z = self._normal(shape)
            c = self._normal(shape) ** 2 + self._normal(shape) ** 2 + self._normal(shape) ** 2
            return z / torch.sqrt(c / 3.0)
        return self._normal(shape)

    def _emit(self, master: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        x = master * self.gain
        x = x if self.wl.dtype == "f32" else to_bf16_bits(x)
        if out is None:
            return x.contiguous()
        out.copy_(x)
        return out

    def advance(self) -> List[torch.Tensor]:
        """Move to the next step; refreshes ``current`` in place and returns it."""
        self.t += 1
        sigma = self.wl.drift_sigma(self.t)
        shape = (self.wl.n_tokens, self.wl.n_channels)
        for k, m in enumerate(self.master):
            m.add_(self._noise(shape), alpha=sigma)
            self._emit(m, self.current[k])
        return self.current


def as_numpy(x: torch.Tensor) -> np.ndarray:
    """Host numpy view of a tensor for the oracle: fp32 as is, bf16 as uint16 bit patterns."""
    x = x.detach().cpu().contiguous()
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16).copy()
    return x.numpy().copy()


def cfg1_numpy(seed: int = 0, steps: int = 5, n_tokens: int = 256, n_channels: int = 64) -> List[np.ndarray]:
    """Config 1 exactly as stated: numpy default_rng(seed), float32, x_t = x_{t-1} + 0.05 N(0,1).

    Returns [x_0, ..., x_{steps-1}] as float32 arrays."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n_tokens, n_channels)).astype(np.float32)
    out = [x.copy()]
    for _ in range(1, steps):
        x = (x + np.float32(0.05) * rng.standard_normal((n_tokens, n_channels)).astype(np.float32)).astype(np.float32)
        out.append(x.copy())
    return out
