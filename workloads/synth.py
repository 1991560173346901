"""Synthetic Wan-shaped attention inputs: clustered, temporally repeating Q/K/V and prompts.

The paper's motivation section observes three structures in the attention features of
autoregressive video DiTs: queries and keys form semantic clusters, a large share of
the keys of one frame reappear almost unchanged in the next, and only a few prompt
tokens matter for a given frame.  The generators below emulate exactly that structure
(and nothing else of the real models) with a seeded Gaussian mixture:

* per head, ``n_c`` key centres and ``n_c`` value centres ~ N(0, I_d);
* token ``t`` of a frame of ``T`` tokens belongs to cluster ``floor(t * n_c / T)``
  (contiguous raster runs, the same map for every frame and for the queries), its key
  is ``centreK + sigma_w * N(0, I)``, its value ``centreV + sigma_w * N(0, I)`` and its
  query ``centreK + sigma_w * N(0, I)`` with fresh noise;
* frame ``f`` equals frame ``f-1`` plus ``sigma_d * N(0, I)`` drift on a random fraction
  ``p`` of its tokens (the mask is shared by the heads, the noise is not); the other
  tokens are re-drawn from their own cluster;
* prompt tokens come from a second mixture of which only ``n_near`` centres sit next
  to (randomly chosen) query-cluster centres.

Everything is drawn on the host with numpy's PCG64 from ``SeedSequence([seed, cfg_id])``
so that the oracle and the GPU path are fed the same bits.  Tensors are handed out in
*storage form*: ``float32`` arrays for fp32 workloads and ``uint16`` arrays holding
bfloat16 bit patterns for bf16 workloads.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# --------------------------------------------------------------------------------------
# storage-format helpers (no method arithmetic)
# --------------------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact float32 value of bfloat16 bit patterns."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> storage form of ``dtype`` ('fp32' or 'bf16')."""
    if dtype == "fp32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def to_f32(x: np.ndarray) -> np.ndarray:
    """Storage form -> exact float32 values."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x)
    return np.ascontiguousarray(x, dtype=np.float32)


# --------------------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------------------

#: Shapes and generator constants of the five synthetic workloads.
CONFIGS = {
    # tiny fp32 case the oracle finishes in seconds
    "cfg1": dict(cfg_id=1, seed=0, dtype="fp32", H=2, d=64, T=256, n_c=16, p=0.7, sigma_d=0.02,
                 chunk_frames=1, cache_frames=4, BQ=128, BK=64, n_rep=4, r=32, sel_frac=0.25,
                 n_p=64, n_pc=8, n_near=2, n_sel_cross=16),
    # Wan-1.3B-shaped self-attention layer
    "cfg2": dict(cfg_id=2, seed=0, dtype="bf16", H=12, d=128, T=1560, n_c=64, p=0.8, sigma_d=0.02,
                 chunk_frames=3, cache_frames=21, BQ=128, BK=64, n_rep=4, r=32, sel_frac=0.10,
                 n_p=512, n_pc=32, n_near=3, n_sel_cross=64),
    # long-rollout sweep of cfg2's layer: cache grows 3 -> 120 frames, capped at 24 frames of slots
    "cfg3": dict(cfg_id=3, seed=0, dtype="bf16", H=12, d=128, T=1560, n_c=64, p=0.8, sigma_d=0.02,
                 chunk_frames=3, cache_frames=120, cap_frames=24, BQ=128, BK=64, n_rep=4, r=32,
                 sel_frac=0.10, n_p=512, n_pc=32, n_near=3, n_sel_cross=64),
    # cross-attention over a 512- or 2048-token prompt
    "cfg4": dict(cfg_id=4, seed=0, dtype="bf16", H=12, d=128, T=1560, n_c=64, p=0.8, sigma_d=0.02,
                 chunk_frames=3, cache_frames=3, BQ=128, BK=64, n_rep=4, r=32, sel_frac=0.10,
                 n_p=512, n_p_long=2048, n_pc=32, n_near=3, n_sel_cross=64),
    # world-model-scale layer
    "cfg5": dict(cfg_id=5, seed=0, dtype="bf16", H=40, d=128, T=3600, n_c=128, p=0.9, sigma_d=0.01,
                 chunk_frames=1, cache_frames=64, BQ=128, BK=64, n_rep=4, r=32, sel_frac=0.10,
                 n_p=512, n_pc=32, n_near=3, n_sel_cross=64),
}

SIGMA_W = 0.3          # within-cluster standard deviation
CODEC_RANGE = 4.5      # |x| mapped to the int8 limit 127 by the quantiser
CODEC_SHIFT = 4        # right shift applied to the projected sums


@dataclass
class Codec:
    """Parameters of the shared low-dimensional 8-bit code (inputs of the method, drawn here)."""
    R: np.ndarray          # [d, r] int8, entries -1 / +1
    qscale: np.float32     # 127 / CODEC_RANGE, rounded once to float32
    shift: int


def make_codec(seed: int, cfg_id: int, d: int, r: int) -> Codec:
    rng = np.random.default_rng(np.random.SeedSequence([seed, cfg_id, 0xC0DEC]))
    R = (rng.integers(0, 2, size=(d, r)).astype(np.int8) * 2 - 1).astype(np.int8)
    return Codec(R=np.ascontiguousarray(R), qscale=np.float32(127.0 / CODEC_RANGE), shift=CODEC_SHIFT)


def make_sign_matrix(seed: int, cfg_id: int, d: int, n_bits: int) -> np.ndarray:
    """Random +-1 hyperplane matrix [d, n_bits] of the sign-code (LSH) variant; input data for oracle and GPU."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, cfg_id, 0x51C4]))
    return np.ascontiguousarray((rng.integers(0, 2, size=(d, n_bits)).astype(np.int8) * 2 - 1).astype(np.int8))


# --------------------------------------------------------------------------------------
# frame stream
# --------------------------------------------------------------------------------------


class FrameStream:
    """Yields frames of (K, V) with cluster structure and frame-to-frame repetition, plus queries."""

    def __init__(self, seed: int, cfg_id: int, H: int, d: int, T: int, n_c: int, p: float,
                 sigma_d: float, dtype: str, heads: slice | None = None):
        self.H, self.d, self.T, self.n_c, self.p, self.sigma_d, self.dtype = H, d, T, n_c, p, sigma_d, dtype
        self.rng = np.random.default_rng(np.random.SeedSequence([seed, cfg_id]))
        self.centreK = self.rng.standard_normal((H, n_c, d), dtype=np.float32)
        self.centreV = self.rng.standard_normal((H, n_c, d), dtype=np.float32)
        self.cluster = (np.arange(T, dtype=np.int64) * n_c // T).astype(np.int64)  # token -> cluster
        self._K = None
        self._V = None
        self.frames_emitted = 0

    @classmethod
    def from_config(cls, name: str, **over) -> "FrameStream":
        c = dict(CONFIGS[name])
        c.update(over)
        return cls(c["seed"], c["cfg_id"], c["H"], c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])

    def _fresh(self, centres: np.ndarray) -> np.ndarray:
        noise = self.rng.standard_normal((self.H, self.T, self.d), dtype=np.float32)
        return centres[:, self.cluster, :] + np.float32(SIGMA_W) * noise

    def next_frame(self):
        """Return (K, V), each [H, T, d] in storage form, for the next frame of the stream."""
        if self._K is None:
            self._K = self._fresh(self.centreK)
            self._V = self._fresh(self.centreV)
        else:
            keep = self.rng.random(self.T) < self.p                     # shared by all heads
            driftK = self.rng.standard_normal((self.H, self.T, self.d), dtype=np.float32)
            driftV = self.rng.standard_normal((self.H, self.T, self.d), dtype=np.float32)
            newK = self._fresh(self.centreK)
            newV = self._fresh(self.centreV)
            m = keep[None, :, None]
            self._K = np.where(m, self._K + np.float32(self.sigma_d) * driftK, newK)
            self._V = np.where(m, self._V + np.float32(self.sigma_d) * driftV, newV)
        self.frames_emitted += 1
        return to_storage(self._K, self.dtype), to_storage(self._V, self.dtype)

    def queries(self, n_frames: int) -> np.ndarray:
        """Queries of a chunk of ``n_frames`` frames: [H, n_frames*T, d] in storage form."""
        out = [self._fresh(self.centreK) for _ in range(n_frames)]
        return to_storage(np.concatenate(out, axis=1), self.dtype)


class PromptSet:
    """Prompt keys/values: ``n_pc`` clusters of which ``n_near`` sit next to query clusters."""

    def __init__(self, seed: int, cfg_id: int, centreK: np.ndarray, n_p: int, n_pc: int, n_near: int,
                 dtype: str):
        H, n_c, d = centreK.shape
        rng = np.random.default_rng(np.random.SeedSequence([seed, cfg_id, 0x9707, n_p]))
        cK = rng.standard_normal((H, n_pc, d), dtype=np.float32)
        cV = rng.standard_normal((H, n_pc, d), dtype=np.float32)
        near_src = rng.choice(n_c, size=n_near, replace=False)
        near_dst = rng.choice(n_pc, size=n_near, replace=False)
        for s, t in zip(near_src, near_dst):
            cK[:, t, :] = centreK[:, s, :] + np.float32(0.1) * rng.standard_normal((H, d), dtype=np.float32)
        self.near_clusters = np.sort(near_dst)
        self.cluster = rng.integers(0, n_pc, size=n_p)
        K = cK[:, self.cluster, :] + np.float32(SIGMA_W) * rng.standard_normal((H, n_p, d), dtype=np.float32)
        V = cV[:, self.cluster, :] + np.float32(SIGMA_W) * rng.standard_normal((H, n_p, d), dtype=np.float32)
        self.K = to_storage(K, dtype)
        self.V = to_storage(V, dtype)
