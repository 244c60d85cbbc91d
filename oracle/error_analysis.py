"""Error-analysis study on synthetic data (test infrastructure, CPU only, fp64).

Re-runs, on the seeded synthetic generator, the two experiments of the paper's "Error
Analysis" section:

  (a) "Strategy of block selection": attention-map mean squared error
      (1 / (Nq Nk)) ||A_sparse - A_full||_F^2 against density for
        - top-p block selection without compensation (the keys of skipped blocks get no
          attention; the kept ones are renormalised),
        - the same selection with linear compensation (Eq. (1)),
        - error-aware routing (value-aware probe, Eq. (7)) with linear compensation,
        - the "Oracle solution" of the Methodology: greedy routing by the exact per-entry
          squared errors of the relaxed objective, which needs all Nq Nk logits,
      all four at the same routed cost.
  (b) "Effect of clustering": the clustering error of Proposition 1,
      delta_q^2 = (1/N_q) sum_i |q_i - qbar_i|^2 (the MEAN over the queries of the squared
      distance to the mean of the query's cluster), and the attention-map error against the
      number of query clusters at a fixed selection.

The paper does not define the top-p rule it inherits; the reading used here (and labelled as
such wherever its numbers are shown) is: per query cluster, key clusters in descending order
of centroid attention mass |k_b| exp(qbar_a . kbar_b / sqrt(d)), the shortest prefix whose
mass reaches the fraction p of the row's total.

Run:  python -m oracle.error_analysis            (prints the two tables)
Only `oracle/` and the seeded input generators are used; nothing here touches the GPU path.
"""
from __future__ import annotations

import sys

import numpy as np

from oracle import svgear_oracle as orc
from workloads.generators import Workload, kmeans_init_indices, make_head


def exact_block_errors(Q, K, lab_q, lab_k, kbar, Cq: int, Ck: int, scale: float) -> np.ndarray:
    """Sum over the entries of every block of the squared error of the relaxed objective
    ("Oracle solution": (exp(q_i.kbar_j*scale) - exp(q_i.k_j*scale))^2, kbar_j the mean of key
    j's cluster). One global shift of the logits keeps the exponentials finite; it scales all
    blocks alike and leaves the greedy order unchanged."""
    Q, K, kbar = (np.asarray(t, np.float64) for t in (Q, K, kbar))
    lab_q, lab_k = np.asarray(lab_q), np.asarray(lab_k)
    exact = (Q @ K.T) * scale
    approx = ((Q @ kbar.T) * scale)[:, lab_k]
    shift = max(exact.max(), approx.max())
    err = (np.exp(approx - shift) - np.exp(exact - shift)) ** 2
    onehot_q = np.zeros((Q.shape[0], Cq))
    onehot_q[np.arange(Q.shape[0]), lab_q] = 1.0
    onehot_k = np.zeros((K.shape[0], Ck))
    onehot_k[np.arange(K.shape[0]), lab_k] = 1.0
    return onehot_q.T @ err @ onehot_k


def top_p_mask(qbar, kbar, k_sizes, p: float, scale: float) -> np.ndarray:
    """The reading of top-p selection stated in the module docstring."""
    qbar, kbar = np.asarray(qbar, np.float64), np.asarray(kbar, np.float64)
    k_sizes = np.asarray(k_sizes, np.float64)
    S = (qbar @ kbar.T) * scale
    S = np.where(k_sizes[None, :] > 0, S, -np.inf)
    mass = k_sizes[None, :] * np.exp(S - S.max(axis=1, keepdims=True))
    mask = np.zeros(mass.shape, dtype=bool)
    for a in range(mass.shape[0]):
        order = np.argsort(-mass[a], kind="stable")
        cum = np.cumsum(mass[a][order])
        n_keep = int(np.searchsorted(cum, p * cum[-1], side="left")) + 1
        mask[a, order[:n_keep]] = True
    return mask & (k_sizes[None, :] > 0)


def dense_map(Q, K, scale: float) -> np.ndarray:
    L = (np.asarray(Q, np.float64) @ np.asarray(K, np.float64).T) * scale
    L -= L.max(axis=1, keepdims=True)
    P = np.exp(L)
    return P / P.sum(axis=1, keepdims=True)


def dropped_map(Q, K, lab_q, lab_k, mask, scale: float) -> np.ndarray:
    """Block-sparse attention without compensation: softmax over the kept keys only."""
    M = np.asarray(mask)[np.asarray(lab_q)][:, np.asarray(lab_k)]
    L = (np.asarray(Q, np.float64) @ np.asarray(K, np.float64).T) * scale
    L = np.where(M, L, -np.inf)
    L -= L.max(axis=1, keepdims=True)
    P = np.exp(L)
    return P / P.sum(axis=1, keepdims=True)


def map_mse(A, A_full) -> float:
    d = A - A_full
    return float((d * d).mean())


def clustering_error(Q, qbar, lab_q) -> float:
    """delta_q^2 of Proposition 1: the average over all queries of |q_i - qbar_i|_2^2, qbar_i
    the centroid of query i's cluster."""
    dq = np.asarray(Q, np.float64) - np.asarray(qbar, np.float64)[np.asarray(lab_q)]
    return float((dq * dq).sum(axis=1).mean())


def cluster(wl: Workload, head: int, Cq: int, Ck: int, iters: int):
    """Q, K, V of one head (fp64) with the method's k-means (seeded init) on Q and K."""
    Q, K, V = (t.float().numpy() for t in make_head(wl, head))
    n = Q.shape[0]
    cq0 = Q[kmeans_init_indices(wl.seed, head, 0, n, Cq)]
    ck0 = K[kmeans_init_indices(wl.seed, head, 1, n, Ck)]
    qbar, lab_q, q_cnt, _ = orc.kmeans(Q, cq0, iters)
    kbar, lab_k, k_cnt, vbar = orc.kmeans(K, ck0, iters, X2=V, prev2=np.zeros((Ck, Q.shape[1]), np.float32))
    return Q, K, V, qbar, lab_q, q_cnt, kbar, vbar, lab_k, k_cnt


def selection_study(wl: Workload, head: int = 0, ps=(0.5, 0.7, 0.85, 0.95), iters: int = 10):
    """Rows (p, density, mse_top_p, mse_top_p_comp, mse_ear_comp, mse_exact_routing_comp)."""
    scale = orc.scale_of(wl.d)
    Q, K, V, qbar, lab_q, q_cnt, kbar, vbar, lab_k, k_cnt = cluster(wl, head, wl.Cq, wl.Ck, iters)
    A_full = dense_map(Q, K, scale)
    perm_k, k_off = orc.permute(lab_k, wl.Ck)
    _, probe_scores, _ = orc.probe_errors(qbar, kbar, vbar, K[perm_k], V[perm_k], k_off, scale)
    cost = q_cnt.astype(np.float64)[:, None] * k_cnt.astype(np.float64)[None, :]
    exact = exact_block_errors(Q, K, lab_q, lab_k, kbar, wl.Cq, wl.Ck, scale)
    exact_ratio = np.where(cost > 0, exact / np.maximum(cost, 1.0), 0.0)
    rows = []
    for p in ps:
        m_top = top_p_mask(qbar, kbar, k_cnt, p, scale)
        budget = int((cost * m_top).sum())
        m_ear = orc.route(probe_scores, q_cnt, k_cnt, budget)[0]
        m_exact = orc.route(exact_ratio, q_cnt, k_cnt, budget)[0]
        rows.append((p, budget / float(Q.shape[0] * K.shape[0]),
                     map_mse(dropped_map(Q, K, lab_q, lab_k, m_top, scale), A_full),
                     map_mse(orc.attention_map_comp(Q, K, lab_q, lab_k, kbar, m_top, scale)[0], A_full),
                     map_mse(orc.attention_map_comp(Q, K, lab_q, lab_k, kbar, m_ear, scale)[0], A_full),
                     map_mse(orc.attention_map_comp(Q, K, lab_q, lab_k, kbar, m_exact, scale)[0], A_full)))
    return rows


def clustering_study(wl: Workload, head: int = 0, cqs=(8, 16, 32, 64, 128), p: float = 0.85, iters: int = 10):
    """Rows (Cq, delta_q^2, mse of top-p selection with compensation at that Cq)."""
    scale = orc.scale_of(wl.d)
    rows = []
    A_full = None
    for Cq in cqs:
        Q, K, V, qbar, lab_q, q_cnt, kbar, vbar, lab_k, k_cnt = cluster(wl, head, Cq, wl.Ck, iters)
        if A_full is None:
            A_full = dense_map(Q, K, scale)
        delta_q2 = clustering_error(Q, qbar, lab_q)
        m_top = top_p_mask(qbar, kbar, k_cnt, p, scale)
        rows.append((Cq, delta_q2,
                     map_mse(orc.attention_map_comp(Q, K, lab_q, lab_k, kbar, m_top, scale)[0], A_full)))
    return rows


STUDY = Workload("study", 1, 1, 4 * 24 * 32, 0, 64, 48, 160, 10, 0.25, "f32", 64, 1.0, 0.3,
                 (4, 24, 32), (4, 4, 4), 21)


def main() -> int:
    wl = STUDY
    print(f"synthetic layer: N={wl.N} d={wl.d} Cq={wl.Cq} Ck={wl.Ck} ({wl.n_comp}-component position-correlated mixture)")
    print("p      density   mse top-p      mse top-p+comp  mse EAR+comp   mse exact-error routing+comp")
    for p, dens, a, b, c, e in selection_study(wl):
        print(f"{p:4.2f}   {dens:7.4f}   {a:.4e}   {b:.4e}      {c:.4e}     {e:.4e}")
    print("Cq     delta_q^2   mse top-p(0.85)+comp")
    for Cq, dq2, mse in clustering_study(wl):
        print(f"{Cq:4d}   {dq2:9.4f}   {mse:.4e}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
