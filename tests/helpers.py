"""Shared helpers of the GPU parity tests: oracle <-> device tensor plumbing."""
import numpy as np
import torch

from oracle import svgear_oracle as orc
from workloads import kmeans_init_indices, structural_rows


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


def check_top_p_row_budgets(got, qbar, kbar, q_sizes, k_sizes, p, scale):
    """GPU row budgets of the adaptive (top-p reading) rule against the oracle's real-valued rule.

    The length of the kept prefix is an integer decided by floating point. The oracle sums fp64
    masses |k_b| exp(S_ab - m_a); the library evaluates the logits and exponentials in fp32
    (relative error of a mass: a few 1e-6 from the d-term fp32 dot product times the logit's size,
    bounded here by 2.5e-5) and counts masses in integer units of 2^-20 (each mass loses less than
    one unit, so a row's sums move by less than Ck 2^-20). The fraction of the row's mass held by
    any prefix therefore moves by at most
        delta = 2 * 2.5e-5 + Ck * 2^-20 / (row's total mass),
    so the library's answer must equal the oracle's wherever the oracle's answer is the same for
    p (1 - delta) and p (1 + delta), and lie between those two answers elsewhere.
    Returns the number of rows that differ from the oracle's answer at p itself."""
    qbar64, kbar64 = np.asarray(qbar, np.float64), np.asarray(kbar, np.float64)
    live = np.asarray(k_sizes) > 0
    S = np.where(live[None, :], (qbar64 @ kbar64.T) * scale, -np.inf)
    total = (np.asarray(k_sizes, np.float64)[None, :] * np.exp(S - S.max(axis=1, keepdims=True))).sum(axis=1)
    delta = 5e-5 + kbar64.shape[0] * 2.0 ** -20 / float(total.min())
    args = (qbar, kbar, q_sizes, k_sizes)
    mid = orc.top_p_row_budgets(*args, p, scale)[0]
    lo = orc.top_p_row_budgets(*args, p * (1 - delta), scale)[0]
    hi = orc.top_p_row_budgets(*args, min(p * (1 + delta), 1.0), scale)[0]
    got = np.asarray(got)
    assert np.all(lo <= got) and np.all(got <= hi), (got, lo, hi)
    settled = lo == hi
    assert np.array_equal(got[settled], mid[settled])
    return int((got != mid).sum())


def check_sampled_rows(wl, Qh, Oh, Kp, Vp, qoff, koff, perm_q, kbar, vbar, mask_bits, row_ptr, rng, n_random=40,
                       tol_pooled=1e-2, tol_row=2e-2, what=""):
    """Output rows of one head (token order, Oh [N,d] on the device) against Eq. (1) + Eq. (6)
    evaluated by the oracle on the GPU's own clustering and mask, on structurally chosen rows
    (cluster and tile edges, smallest / largest cluster, rows with nothing / the most routed, text
    rows) plus random ones. Every row must be within tol_row, all rows pooled within tol_pooled;
    a failure names the row."""
    named = structural_rows(qoff, row_ptr, wl.Cq, rng, n_random)
    names = list(named)
    rows = np.array([named[k] for k in names], np.int64)
    mask = bits_to_mask(mask_bits, wl.Ck)
    lq = np.repeat(np.arange(wl.Cq + 1), np.diff(qoff))
    lk = np.repeat(np.arange(wl.Ck + 1), np.diff(koff))
    kb = np.concatenate([kbar, np.zeros((1, wl.d), np.float32)])
    vb = np.concatenate([vbar, np.zeros((1, wl.d), np.float32)])
    tok = torch.from_numpy(perm_q[rows]).long().to(Qh.device)
    ref = orc.attention_comp(to_np(Qh[tok]), Kp, Vp, lq[rows], lk, kb, vb, mask, orc.scale_of(wl.d), row_chunk=16)
    got = to_np(Oh[tok])  # permuted row p of the output sits at token perm_q[p]
    per_row = np.linalg.norm(got - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-30)
    worst = int(np.argmax(per_row))
    assert per_row[worst] <= tol_row, f"{what}: {names[worst]} (permuted row {rows[worst]}): rel-L2 {per_row[worst]:.3e}"
    pooled = rel_l2(got, ref)
    assert pooled <= tol_pooled, f"{what}: pooled rel-L2 {pooled:.3e} over {len(rows)} rows"
    return pooled, float(per_row[worst])
