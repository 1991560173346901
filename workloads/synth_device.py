"""The frame stream of ``synth.py`` drawn on the GPU, for workloads too large to generate on the host.

Same recipe (per-head cluster centres, raster cluster map, within-cluster noise 0.3, frame f = frame f-1 plus
sigma_d drift on a random fraction p of the tokens, the rest re-drawn, queries = key centre + fresh noise), same
constants, but the random numbers come from torch's seeded device generator instead of numpy's PCG64, so the
values are not those of ``FrameStream`` with the same seed: only the distribution is.  The world-model-scale
benchmark fills its 64-frame cache with it (4.7 GB of keys and values) and copies the heads the CPU oracle
replays to the host; both sides then see the same bits.

Input generation only: none of the method's arithmetic lives here.
"""
from __future__ import annotations

import torch

from .synth import SIGMA_W


class DeviceFrameStream:
    """Yields frames (K, V) as device tensors [H, T, d] in the storage dtype, plus queries."""

    def __init__(self, seed: int, cfg_id: int, H: int, d: int, T: int, n_c: int, p: float, sigma_d: float,
                 dtype: str, device: str = "cuda"):
        self.H, self.d, self.T, self.n_c, self.p, self.sigma_d = H, d, T, n_c, p, sigma_d
        self.dt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.device = device
        self.g = torch.Generator(device=device).manual_seed((seed << 20) + cfg_id * 7919 + 13)
        self.centreK = torch.randn((H, n_c, d), device=device, generator=self.g)
        self.centreV = torch.randn((H, n_c, d), device=device, generator=self.g)
        self.cluster = (torch.arange(T, device=device, dtype=torch.int64) * n_c) // T
        self._K = None
        self._V = None
        self.frames_emitted = 0

    def _fresh(self, centres: torch.Tensor) -> torch.Tensor:
        noise = torch.randn((self.H, self.T, self.d), device=self.device, generator=self.g)
        return centres[:, self.cluster, :] + SIGMA_W * noise

    def next_frame(self):
        if self._K is None:
            self._K = self._fresh(self.centreK)
            self._V = self._fresh(self.centreV)
        else:
            keep = torch.rand((self.T,), device=self.device, generator=self.g) < self.p    # shared by all heads
            m = keep[None, :, None]
            driftK = torch.randn((self.H, self.T, self.d), device=self.device, generator=self.g)
            driftV = torch.randn((self.H, self.T, self.d), device=self.device, generator=self.g)
            self._K = torch.where(m, self._K + self.sigma_d * driftK, self._fresh(self.centreK))
            self._V = torch.where(m, self._V + self.sigma_d * driftV, self._fresh(self.centreV))
        self.frames_emitted += 1
        return self._K.to(self.dt), self._V.to(self.dt)

    def queries(self, n_frames: int) -> torch.Tensor:
        return torch.cat([self._fresh(self.centreK) for _ in range(n_frames)], dim=1).to(self.dt)
