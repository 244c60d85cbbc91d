"""Shared helpers of the GPU parity tests: oracle <-> device tensor plumbing."""
import numpy as np
import torch

from oracle import svgear_oracle as orc
from workloads import kmeans_init_indices


def dev():
    return torch.device("cuda:0")


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu()
    return t.float().numpy() if t.dtype == torch.bfloat16 else t.numpy()


def init_centroids(X: torch.Tensor, C: int, seed: int, tensor_id: int, n_tail: int = 0) -> torch.Tensor:
    """[B,H,C,d] fp32 initial centroids: seeded distinct rows of each head (on X's device)."""
    B, H, N, d = X.shape
    out = torch.empty(B, H, C, d, dtype=torch.float32, device=X.device)
    for b in range(B):
        for h in range(H):
            idx = kmeans_init_indices(seed, b * H + h, tensor_id, N - n_tail, C)
            out[b, h] = X[b, h][torch.from_numpy(idx).to(X.device)].float()
    return out


def mask_to_bits(mask: np.ndarray, Cq: int, Ck: int) -> np.ndarray:
    """Oracle mask (rows Cq or Cq+1, cols Ck or Ck+1) -> [Cq+1, W] uint32 words."""
    W = (Ck + 1 + 31) // 32
    full = np.zeros((Cq + 1, W * 32), dtype=bool)
    full[: mask.shape[0], : mask.shape[1]] = mask
    bits = np.zeros((Cq + 1, W), dtype=np.uint32)
    for j in range(32):
        bits |= full[:, j::32].astype(np.uint32) << np.uint32(j)
    return bits


def bits_to_mask(bits: np.ndarray, Ck: int) -> np.ndarray:
    bits = bits.astype(np.uint32)
    R, W = bits.shape
    out = np.zeros((R, W * 32), dtype=bool)
    for j in range(32):
        out[:, j::32] = (bits >> np.uint32(j)) & 1
    return out[:, : Ck + 1]


def csr_from_mask(mask_full: np.ndarray):
    """[Cq+1, Ck+1] bool -> (row_ptr [Cq+2], col_idx padded to (Cq+1)*(Ck+1))."""
    R, Cc = mask_full.shape
    row_ptr = np.zeros(R + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(mask_full.sum(1))
    col = np.zeros(R * Cc, dtype=np.int32)
    nz = np.concatenate([np.nonzero(mask_full[a])[0] for a in range(R)]) if R else np.zeros(0)
    col[: nz.shape[0]] = nz
    return row_ptr, col


def full_mask(mask: np.ndarray, Cq: int, Ck: int) -> np.ndarray:
    out = np.zeros((Cq + 1, Ck + 1), dtype=bool)
    out[: mask.shape[0], : mask.shape[1]] = mask
    return out


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def oracle_head(Q, K, V, b, h, wl, iters=None, budget=None, **kw):
    """Runs the oracle's whole path on head (b,h) of device/cpu tensors Q,K,V."""
    from workloads import budget_pairs

    q, k, v = (to_np(t[b, h]) for t in (Q, K, V))
    nv = wl.N - wl.n_tail
    iq = kmeans_init_indices(wl.seed, b * wl.H + h, 0, nv, wl.Cq)
    ik = kmeans_init_indices(wl.seed, b * wl.H + h, 1, nv, wl.Ck)
    budget = budget_pairs(wl.rho, wl.N, wl.N) if budget is None else budget
    return orc.hot_path_head(q, k, v, q[iq], k[ik], wl.iters if iters is None else iters, budget,
                             n_tail=wl.n_tail, **kw)
