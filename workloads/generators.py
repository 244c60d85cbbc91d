"""Synthetic Q/K/V generators and seeded k-means initial index draws.

The paper evaluates on Wan2.2 and HunyuanVideo generations (Experiments, "Models" and
"Datasets"); neither the models nor the prompts are available here, so these generators
stand in for them: they keep the token counts, head counts and head dimension of those
models and draw every token from a Gaussian mixture whose component correlates with the
token's (t, h, w) position, which gives k-means the spatially coherent clusters that the
method relies on (Motivation, "Structured Redundancy in Attention Computation").

Nothing here computes any part of the method; both the HIP harness and the oracle's tests
consume the tensors produced here.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int  # tokens per head including the tail
    n_tail: int  # trailing (text) tokens: never clustered, always routed exactly
    d: int
    Cq: int
    Ck: int
    iters: int
    rho: float
    dtype: str  # "f32" | "bf16"
    n_comp: int
    center_std: float
    sigma: float
    grid: Optional[Tuple[int, int, int]]  # (T, Hh, Ww) token grid, None = iid components
    cells: Optional[Tuple[int, int, int]]  # component cells along (t, h, w)
    seed: int = 0

    @property
    def n_video(self) -> int:
        return self.N - self.n_tail

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    # Tiny fp32 single layer: the oracle finishes every stage in seconds.
    "tiny": Workload("tiny", 1, 1, 4096, 0, 64, 32, 64, 10, 0.25, "f32", 16, 3.0, 0.5, None, None, 0),
    # Wan2.2-shaped layer: 21 latent frames x 45 x 80 patches, 40 heads, d = 128.
    "wan": Workload("wan", 1, 40, 75600, 0, 128, 100, 500, 10, 0.25, "bf16", 256, 1.0, 0.3,
                    (21, 45, 80), (4, 8, 8), 0),
    # HunyuanVideo-shaped layer: 33 x 45 x 80 video tokens + 256 text tokens, 24 heads.
    "hunyuan": Workload("hunyuan", 1, 24, 118800 + 256, 256, 128, 100, 500, 10, 0.25, "bf16", 256,
                        1.0, 0.3, (33, 45, 80), (4, 8, 8), 0),
    # The same layers with the cluster counts the paper's experiments use (Experiment setup:
    # Q_C / K_C = 300 / 1000 and 400 / 1000; Turbo variant 200 / 500 at a lower budget)
    "wan_c300": Workload("wan_c300", 1, 40, 75600, 0, 128, 300, 1000, 10, 0.25, "bf16", 256, 1.0, 0.3,
                         (21, 45, 80), (4, 8, 8), 0),
    "hunyuan_c400": Workload("hunyuan_c400", 1, 24, 118800 + 256, 256, 128, 400, 1000, 10, 0.25, "bf16", 256,
                             1.0, 0.3, (33, 45, 80), (4, 8, 8), 0),
    "wan_turbo": Workload("wan_turbo", 1, 40, 75600, 0, 128, 200, 500, 10, 0.15, "bf16", 256, 1.0, 0.3,
                          (21, 45, 80), (4, 8, 8), 0),
    # Scaled-down video-shaped cases used by the parity tests (oracle runs them in seconds).
    "mini_video": Workload("mini_video", 1, 2, 6 * 10 * 16, 0, 128, 12, 40, 4, 0.25, "bf16", 32,
                           1.0, 0.3, (6, 10, 16), (2, 4, 4), 3),
    # bf16 with d = 64 (the generic MFMA kernel), query clusters spanning several 128-row tiles
    "mini_d64": Workload("mini_d64", 1, 2, 1500, 0, 64, 5, 37, 3, 0.3, "bf16", 8, 1.0, 0.3, None, None, 7),
    # more query clusters than one probe workgroup covers (140 > 128), few key clusters
    "mini_manyq": Workload("mini_manyq", 1, 2, 900, 0, 128, 140, 20, 3, 0.25, "bf16", 24, 1.0, 0.3, None, None, 9),
    # fp32 with d = 128, batch of two
    "mini_f32_d128": Workload("mini_f32_d128", 2, 1, 700, 0, 128, 9, 33, 3, 0.25, "f32", 12, 1.5, 0.4, None, None, 11),
    # many small key clusters (about 12 rows each, like K_C = 1000 on a full layer's scale
    # relative to the 64-key tile) and more query clusters than key tiles
    "mini_manyk": Workload("mini_manyk", 1, 2, 4 * 12 * 20, 0, 128, 30, 80, 3, 0.25, "bf16", 48, 1.0, 0.3,
                           (4, 12, 20), (3, 4, 4), 13),
    "mini_video_tail": Workload("mini_video_tail", 1, 2, 5 * 9 * 14 + 37, 37, 128, 10, 30, 4,
                                0.25, "bf16", 32, 1.0, 0.3, (5, 9, 14), (2, 4, 4), 5),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def budget_pairs(rho: float, Nq: int, Nk: int) -> int:
    """Routing budget as a whole number of (query, key) pairs: floor(rho * Nq * Nk)."""
    return int(np.floor(np.float64(rho) * np.float64(Nq) * np.float64(Nk)))


def _torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _component_ids(wl: Workload, gen: torch.Generator, device) -> torch.Tensor:
    """Mixture component of every video token of one head."""
    n = wl.n_video
    if wl.grid is None:
        # iid categorical with Dirichlet(1) weights (normalised unit exponentials)
        e = -torch.log(torch.rand(wl.n_comp, generator=gen, device=device, dtype=torch.float64))
        w = e / e.sum()
        return torch.multinomial(w.float(), n, replacement=True, generator=gen)
    T, Hh, Ww = wl.grid
    ct, ch, cw = wl.cells
    assert ct * ch * cw == wl.n_comp and T * Hh * Ww == n
    idx = torch.arange(n, device=device)
    t = idx // (Hh * Ww)
    h = (idx // Ww) % Hh
    w = idx % Ww
    cell = ((t * ct) // T) * (ch * cw) + ((h * ch) // Hh) * cw + (w * cw) // Ww
    stray = torch.rand(n, generator=gen, device=device) >= 0.8
    rnd = torch.randint(0, wl.n_comp, (n,), generator=gen, device=device)
    return torch.where(stray, rnd, cell)


def make_head(wl: Workload, head: int, device="cpu", step_drift: int = 0):
    """Q, K, V of one head, each [N, d] in the workload's dtype.

    A token's q, k and v share one mixture component (they come from one hidden state)
    but use separate centre tables. `step_drift` > 0 adds that many rounds of N(0, 0.05^2)
    drift (the denoising-trajectory workload), re-rounded to the dtype each round.
    """
    gen = torch.Generator(device=device)
    gen.manual_seed(1_000_003 * wl.seed + 7919 * head + 17)
    z = _component_ids(wl, gen, device)
    out = []
    for _tensor in range(3):
        mu = wl.center_std * torch.randn(wl.n_comp, wl.d, generator=gen, device=device)
        x = mu[z] + wl.sigma * torch.randn(wl.n_video, wl.d, generator=gen, device=device)
        if wl.n_tail:
            mu_t = wl.center_std * torch.randn(1, wl.d, generator=gen, device=device)
            xt = mu_t + wl.sigma * torch.randn(wl.n_tail, wl.d, generator=gen, device=device)
            x = torch.cat([x, xt], 0)
        x = x.to(_torch_dtype(wl.dtype))
        for _ in range(step_drift):
            x = (x.float() + 0.05 * torch.randn(x.shape, generator=gen, device=device)).to(x.dtype)
        out.append(x)
    return out


def make_qkv(wl: Workload, device="cpu", heads=None):
    """Q, K, V as [B, H', N, d] tensors (H' = len(heads) or wl.H), contiguous."""
    heads = list(range(wl.H)) if heads is None else list(heads)
    dt = _torch_dtype(wl.dtype)
    Q = torch.empty(wl.B, len(heads), wl.N, wl.d, dtype=dt, device=device)
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)
    for b in range(wl.B):
        for i, h in enumerate(heads):
            q, k, v = make_head(wl, b * wl.H + h, device)
            Q[b, i], K[b, i], V[b, i] = q, k, v
    return Q, K, V


_M64 = (1 << 64) - 1


def _splitmix64(state: int):
    state = (state + 0x9E3779B97F4A7C15) & _M64
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return state, z ^ (z >> 31)


def kmeans_init_indices(seed: int, head: int, tensor_id: int, n: int, c: int) -> np.ndarray:
    """First `c` entries of a seeded Fisher-Yates shuffle of 0..n-1 (distinct row indices).

    The initial centroid of cluster j is row idx[j] of the tensor being clustered; the
    draw is made here, outside the method, and handed to both implementations.
    """
    assert 0 < c <= n
    state = (seed * 0x9E3779B97F4A7C15 + head * 0xD1B54A32D192ED03 + tensor_id * 0x8CB92BA72F3D8DD7 + 1) & _M64
    swapped = {}
    out = np.empty(c, dtype=np.int64)
    for i in range(c):
        state, r = _splitmix64(state)
        j = i + r % (n - i)
        vi = swapped.get(i, i)
        vj = swapped.get(j, j)
        out[i] = vj
        swapped[j] = vi
    return out
