"""Seeded VGGT-shaped Q/K/V tensors for one global-attention layer.

The paper evaluates on real VGGT activations (7Scenes, NRGBD, ETH3D, ScanNet);
those are not available, so the tensors here only copy their *shape* (S frames
of P patch tokens + 5 special tokens, 16 heads of 64 channels) and the
*structure* the paper reports for them (Sec. 3.1: neighbouring patches are
similar, and the same region of consecutive frames is similar).

Recipe, per workload:
  * base field F[Hp, Wp, 1024] ~ N(0,1), Gaussian-smoothed per channel with
    sigma = 2 patches (wrap-around), rescaled to unit std per channel;
  * frame f = F circularly shifted by an integer (dy, dx) drawn per frame from
    {-s..s}^2, plus N(0, 0.1^2) noise per element;
  * 5 special-token vectors ~ N(0,1), shared by all frames, plus the same noise;
  * token order inside a frame: 5 specials, then patches row-major;
  * Q/K/V = X @ W_{q,k,v} with W ~ N(0, (1/32)^2) of shape 1024x1024, computed
    in fp32, reshaped to [H, N, 64] and rounded ONCE to bf16.

The bf16 tensors returned are the single input of both the oracle (which
up-casts them) and the HIP path.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

SEED_BASE = 251121317
D_MODEL = 1024
N_HEADS = 16
D_HEAD = 64
N_SPECIAL = 5


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    S: int            # frames
    Hp: int           # patch rows
    Wp: int           # patch columns
    b: int            # spatial block edge, in patches
    T: int            # temporal block length, in frames
    rho: float        # merge ratio (fraction of a block's tokens that are merged away)
    max_shift: int    # per-frame shift range {-max_shift..max_shift}^2
    H: int = N_HEADS
    d_head: int = D_HEAD
    n_special: int = N_SPECIAL
    anchor: bool = False   # first-frame anchoring switched on for this workload
    chunked: bool = False  # spatial blocks are runs of b consecutive tokens (the paper's n_s) instead of windows
    dst_frac: float = 0.0  # > 0: fixed share of dst tokens per block and top-r selection of the src that merge

    @property
    def tokens_per_frame(self) -> int:
        return self.Hp * self.Wp + self.n_special

    @property
    def N(self) -> int:
        return self.S * self.tokens_per_frame


CONFIGS = {
    1: Workload("cfg1_S2_16x16_b4T2_r0.5", 1, 2, 16, 16, 4, 2, 0.5, 1),
    2: Workload("cfg2_S8_37x37_b4T2_r0.5", 2, 8, 37, 37, 4, 2, 0.5, 1),
    3: Workload("cfg3_S32_21x37_b4T4_r0.75", 3, 32, 21, 37, 4, 4, 0.75, 1),
    4: Workload("cfg4_S100_37x37_b4T4_r0.8", 4, 100, 37, 37, 4, 4, 0.8, 2),
    5: Workload("cfg5_S200_37x37_b8T4_r0.9", 5, 200, 37, 37, 8, 4, 0.9, 1),
}


def workload(index: int) -> Workload:
    return CONFIGS[index]


def _smooth_field(rng: np.random.Generator, Hp: int, Wp: int) -> np.ndarray:
    from scipy.ndimage import gaussian_filter

    field = rng.standard_normal((Hp, Wp, D_MODEL), dtype=np.float32)
    field = gaussian_filter(field, sigma=(2.0, 2.0, 0.0), mode="wrap")
    std = field.reshape(-1, D_MODEL).std(axis=0)
    return (field / std).astype(np.float32)


def make_qkv(w: Workload, device: str = "cpu", seed: int | None = None):
    """Return (q, k, v): three contiguous bf16 tensors of shape [H, N, d_head] on `device`.

    The random draws come from NumPy's PCG64 on the host; only the three
    projections run on `device` (a plain matmul, outside the path under test).
    """
    if seed is None:
        seed = SEED_BASE + w.index
    rng = np.random.Generator(np.random.PCG64(seed))
    field = _smooth_field(rng, w.Hp, w.Wp)
    special = rng.standard_normal((w.n_special, D_MODEL), dtype=np.float32)
    shifts = rng.integers(-w.max_shift, w.max_shift + 1, size=(w.S, 2))
    w_qkv = (rng.standard_normal((D_MODEL, 3 * D_MODEL), dtype=np.float32) / 32.0)
    w_dev = torch.from_numpy(w_qkv).to(device)

    tpf = w.tokens_per_frame
    out = [torch.empty((w.H, w.N, w.d_head), dtype=torch.bfloat16, device=device) for _ in range(3)]
    for f in range(w.S):
        dy, dx = int(shifts[f, 0]), int(shifts[f, 1])
        frame = np.roll(field, shift=(dy, dx), axis=(0, 1)).reshape(w.Hp * w.Wp, D_MODEL)
        x = np.concatenate([special, frame], axis=0)
        x = x + 0.1 * rng.standard_normal(x.shape, dtype=np.float32)
        proj = torch.from_numpy(x).to(device) @ w_dev          # [tpf, 3*1024] fp32
        proj = proj.view(tpf, 3, N_HEADS, D_HEAD).permute(1, 2, 0, 3)  # [3, 16, tpf, 64]
        for t in range(3):
            out[t][:, f * tpf:(f + 1) * tpf, :] = proj[t, :w.H].to(torch.bfloat16)  # first H heads
    return out[0], out[1], out[2]


def bf16_to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Exact up-cast of a bf16 tensor to a float32 NumPy array on the host."""
    return t.detach().to("cpu", torch.float32).numpy()
