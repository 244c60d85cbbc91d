"""TEST INFRASTRUCTURE ONLY -- plain CPU oracle for the SVG-EAR attention hot path.

Every function evaluates, slowly and in fp64 (numpy), what the paper defines; each cites
the passage it follows. Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this package. It shares no code with the HIP library and never calls it.

Stages (one attention head at a time; batch and head dimensions are independent,
Appendix "Kernel Implementation Details"):

  kmeans          Methodology, "Problem Formulation": Q and K are clustered, centroids
                  are cluster means; V follows K's assignment ("Linear Compensation").
  permute         Motivation, "Structured Redundancy": tokens of a cluster are laid out
                  contiguously.
  probe_errors    Eq. (7) (value-aware) or Eq. (5) (plain) summed over each block, with the
                  per-row stabiliser of Algorithm 1 (first line: m_i = max_j S_ij).
  route           "Error-Aware Routing": greedy by error-to-size ratio under the budget.
  top_p_row_budgets  Experiments, "Implementation": one adaptive budget per query cluster (a
                  labelled reading: the paper inherits the rule and does not define it).
  attention_comp  Eq. (1) and Eq. (6) evaluated literally.

Readings taken where the paper is silent or inconsistent are listed next to each function.

Parity pins: every function here is pinned by tests/test_oracle_*.py against closed forms,
brute force or library routines. One caveat: top_p_row_budgets implements a reading of a rule
the paper inherits without printing it; it is pinned to that stated definition and is "parity
unpinned" with respect to whatever rule the paper's own implementation used.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

from .build_oracle import build as _build_c

_lib = None


def _clib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build_c())
        _lib.svgear_oracle_assign_f32.argtypes = [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p,
        ]
        _lib.svgear_oracle_assign_f32.restype = None
        _lib.svgear_oracle_max_threads.restype = ctypes.c_int
    return _lib


def host_threads() -> int:
    """Threads the C assignment loop uses (OpenMP's maximum on this host)."""
    return int(_clib().svgear_oracle_max_threads())


# --------------------------------------------------------------------------- k-means


def kmeans_assign(X: np.ndarray, cent: np.ndarray, return_scores: bool = False):
    """Nearest-centroid label of every row, decided in the fixed fp32 order.

    Squared Euclidean distance with the row's own norm dropped: score = |c|^2 - 2 x.c,
    each dot product one fp32 fma chain over t = 0..d-1; ties go to the lowest index
    (see assign_f32.c). X [n, d] and cent [C, d] are taken as float32 exactly.
    """
    X = np.ascontiguousarray(X, dtype=np.float32)
    cent = np.ascontiguousarray(cent, dtype=np.float32)
    n, d = X.shape
    C = cent.shape[0]
    assert cent.shape[1] == d
    labels = np.empty(n, dtype=np.int32)
    best = np.empty(n, dtype=np.float32) if return_scores else None
    _clib().svgear_oracle_assign_f32(
        X.ctypes.data, n, d, cent.ctypes.data, C, labels.ctypes.data,
        best.ctypes.data if return_scores else None,
    )
    return (labels, best) if return_scores else labels


def cluster_means(X: np.ndarray, labels: np.ndarray, C: int, prev: np.ndarray):
    """Mean of the members of each cluster (fp64 sums, rounded once to fp32).

    "Problem Formulation": the centroid is the mean token of the cluster. A cluster with
    no member keeps its previous centroid and reports count 0 (the paper does not treat
    empty clusters; with weight |k_c| = 0 they contribute nothing downstream).
    """
    X64 = np.asarray(X, dtype=np.float64)
    out = np.array(prev, dtype=np.float32, copy=True)
    counts = np.zeros(C, dtype=np.int32)
    for c in range(C):
        sel = labels == c
        k = int(sel.sum())
        counts[c] = k
        if k:
            out[c] = (X64[sel].sum(axis=0) / k).astype(np.float32)
    return out, counts


def kmeans(X, init, iters: int, X2=None, prev2=None):
    """`iters` Lloyd iterations (assign, then recompute means) from `init`.

    Returns (centroids f32 [C,d], labels i32 [n], counts i32 [C], centroids2 or None).
    The final centroids are the exact means of the final labels, as "Problem Formulation"
    requires of q-bar and k-bar; centroids2 are the means of X2 (the values) under the same
    labels ("Linear Compensation": V follows K's assignment). Fixed iteration count, no
    early exit (the paper states neither; the benchmark configurations fix the count).
    """
    assert iters >= 1
    cent = np.array(init, dtype=np.float32, copy=True)
    C = cent.shape[0]
    labels = counts = None
    for _ in range(iters):
        labels = kmeans_assign(X, cent)
        cent, counts = cluster_means(X, labels, C, cent)
    cent2 = None
    if X2 is not None:
        if prev2 is None:
            prev2 = np.zeros((C, X2.shape[1]), dtype=np.float32)
        cent2, _ = cluster_means(X2, labels, C, prev2)
    return cent, labels, counts, cent2


def inertia(X, cent, labels) -> float:
    """Sum of squared distances of rows to their assigned centroid (fp64)."""
    diff = np.asarray(X, np.float64) - np.asarray(cent, np.float64)[labels]
    return float((diff * diff).sum())


# --------------------------------------------------------------------------- permute


def permute(labels: np.ndarray, C: int, n_tail: int = 0):
    """Cluster-contiguous order: stable sort of token indices by label.

    perm[p] is the original index of the token at sorted position p. The n_tail trailing
    tokens (text tokens, which are not clustered) form pseudo-cluster C in original order.
    offsets has C + 2 entries: cluster c occupies [offsets[c], offsets[c+1]) and the tail
    [offsets[C], offsets[C+1]).
    """
    labels = np.asarray(labels)
    n_clustered = labels.shape[0]
    full = np.concatenate([labels.astype(np.int64), np.full(n_tail, C, dtype=np.int64)])
    perm = np.argsort(full, kind="stable").astype(np.int32)
    counts = np.bincount(full, minlength=C + 1)
    offsets = np.zeros(C + 2, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    assert offsets[C] == n_clustered
    return perm, offsets


def unpermute_rows(Op: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """O[perm[p]] = Op[p]."""
    out = np.empty_like(Op)
    out[perm] = Op
    return out


# --------------------------------------------------------------------------- probe


def probe_errors(qbar, kbar, vbar, Kp, Vp, k_offsets, scale: float, value_aware: bool = True):
    """Estimated compensation error of every (query cluster a, key cluster b) block.

    Value-aware, Eq. (7) summed over the keys of the block, every term carrying the row
    factor exp(-m_a) that Algorithm 1 introduces (m_a = max_b qbar_a.kbar_b * scale over
    non-empty b):

        E[a,b] = sum_{j in b} || exp(Sbar_ab - m_a) vbar_b - exp(qbar_a.k_j*scale - m_a) v_j ||^2

    Plain, Eq. (5): the same without the value vectors (scalar difference squared).
    Returns (E [Cq,Ck], scores = E / |k_b| [Cq,Ck], m [Cq]). Because every query of cluster
    a shares the estimate, the block's total error is |q_a| E[a,b] and its cost |q_a||k_b|,
    so the error-to-cost ratio of "Error-Aware Routing" is E[a,b]/|k_b|. Empty key clusters
    get E = score = 0 and are never routed nor compensated.

    Readings: Algorithm 1 as printed starts its accumulator at ||Y||^2 instead of 0 and
    rescales by exp(2(m_i - m_local)) at the end; Eq. (7) and the text ("aggregate the
    estimated errors within each block") have no initial term, and moving an accumulator
    from exp(-2 m_local) units to exp(-2 m_i) units needs exp(2(m_local - m_i)). This oracle
    follows Eq. (7): it starts at 0 and needs no running maximum at all in fp64 (the tests
    check the change-of-units identity that any streaming evaluation relies on).
    Kp, Vp are cluster-contiguous (k_offsets); only clustered keys enter.
    """
    qbar = np.asarray(qbar, np.float64)
    kbar = np.asarray(kbar, np.float64)
    vbar = np.asarray(vbar, np.float64)
    Cq, Ck = qbar.shape[0], kbar.shape[0]
    sizes = np.diff(np.asarray(k_offsets[: Ck + 1], np.int64))
    Sbar = (qbar @ kbar.T) * scale
    nonempty = sizes > 0
    m = np.where(nonempty[None, :], Sbar, -np.inf).max(axis=1)
    E = np.zeros((Cq, Ck), dtype=np.float64)
    for b in range(Ck):
        if not nonempty[b]:
            continue
        Kb = np.asarray(Kp[k_offsets[b]: k_offsets[b + 1]], np.float64)
        Vb = np.asarray(Vp[k_offsets[b]: k_offsets[b + 1]], np.float64)
        w = np.exp((qbar @ Kb.T) * scale - m[:, None])  # [Cq, nb]
        W = np.exp(Sbar[:, b] - m)  # [Cq]
        if value_aware:
            diff = W[:, None, None] * vbar[b][None, None, :] - w[:, :, None] * Vb[None, :, :]
            E[:, b] = (diff * diff).sum(axis=(1, 2))
        else:
            diff = W[:, None] - w
            E[:, b] = (diff * diff).sum(axis=1)
    scores = np.where(nonempty[None, :], E / np.maximum(sizes, 1)[None, :], 0.0)
    return E, scores, m


# --------------------------------------------------------------------------- route


def route(scores, q_sizes, k_sizes, budget: int, per_row: bool = False,
          n_tail_q: int = 0, n_tail_k: int = 0, row_budgets=None):
    """Greedy error-to-cost routing under a cost budget ("Error-Aware Routing").

    Blocks with both sizes non-zero are ordered by score descending (NaN counts as +inf),
    equal scores by ascending linear index a*Ck + b. The cost of a block is |q_a||k_b|
    (integer). Walking that order, blocks are routed while the running cost stays within
    the budget; the walk stops at the first block that does not fit (the paper says
    "until the budget is exhausted"; stop-at-first-misfit is the reading taken).

    Tail (text) tokens form one extra query row (index Cq) and one extra key column
    (index Ck); their blocks are always routed and are charged to the budget first (if
    they alone exceed it, nothing else is routed).

    per_row=True applies the same rule independently to each query cluster a with budget
    floor(budget * |q_a| / Nq_total) (the granularity of the paper's implementation,
    Experiments, "Implementation"). row_budgets (one integer per query cluster, e.g. from
    top_p_row_budgets) replaces that split: row a then routes clustered blocks up to
    row_budgets[a]; the forced tail column comes on top and is not charged to it.

    Returns (mask bool [R, Cc], row_ptr i32 [R+1], col_idx i32, routed_cost int) with
    R = Cq + (n_tail_q > 0), Cc = Ck + (n_tail_k > 0); col_idx ascending within a row.
    """
    scores = np.asarray(scores)
    Cq, Ck = scores.shape
    qs = [int(v) for v in q_sizes[:Cq]] + ([int(n_tail_q)] if n_tail_q > 0 else [])
    ks = [int(v) for v in k_sizes[:Ck]] + ([int(n_tail_k)] if n_tail_k > 0 else [])
    R, Cc = len(qs), len(ks)
    nq_total = sum(qs)
    mask = np.zeros((R, Cc), dtype=bool)
    row_forced = [0] * R
    for a in range(R):
        for b in range(Cc):
            forced = (a >= Cq) or (b >= Ck)
            if forced and qs[a] > 0 and ks[b] > 0:
                mask[a, b] = True
                row_forced[a] += qs[a] * ks[b]
    routed_cost = sum(row_forced)

    def key(a, b):
        s = float(scores[a, b])
        if np.isnan(s):
            s = np.inf
        return (-s, a * Ck + b)

    def greedy(items, remaining):
        spent = 0
        for (a, b) in sorted(items, key=lambda ab: key(*ab)):
            c = qs[a] * ks[b]
            if spent + c > remaining:
                break
            spent += c
            mask[a, b] = True
        return spent

    if per_row or row_budgets is not None:
        for a in range(Cq):
            if qs[a] == 0:
                continue
            if row_budgets is not None:
                rem = max(int(row_budgets[a]), 0)
            else:
                rem = max((int(budget) * qs[a]) // max(nq_total, 1) - row_forced[a], 0)
            routed_cost += greedy([(a, b) for b in range(Ck) if ks[b] > 0], rem)
    else:
        rem = max(int(budget) - routed_cost, 0)
        items = [(a, b) for a in range(Cq) for b in range(Ck) if qs[a] > 0 and ks[b] > 0]
        routed_cost += greedy(items, rem)

    row_ptr = np.zeros(R + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(mask.sum(axis=1))
    col_idx = np.concatenate([np.nonzero(mask[a])[0] for a in range(R)]).astype(np.int32) \
        if R else np.zeros(0, np.int32)
    return mask, row_ptr, col_idx, int(routed_cost)


def top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, p: float, scale: float):
    """Adaptive per-query-cluster budgets (Experiments, "Implementation": the method inherits
    a top-p budget allocation and routes per query cluster; hyper-parameter table, "TopP").

    The paper does not define the rule. Reading taken (a labelled guess): for query cluster a,
    the non-empty key clusters carry the centroid attention mass
        mass_b = |k_b| exp(qbar_a . kbar_b * scale - m_a),  m_a the largest such logit,
    i.e. the share of a centroid query's softmax that falls on cluster b when every key sits at
    its centroid (real numbers, fp64 here). Clusters are ordered by mass descending, equal ones
    by ascending b; the prefix kept is the shortest whose summed mass reaches p times the
    row's total mass. The budget of row a is the cost of exact attention over that prefix,
    |q_a| * sum_{b kept} |k_b| query-key pairs; error-aware routing then spends it on the
    blocks of row a with the largest error-to-cost ratio.

    p is taken at float32 precision (the value an implementation receives through a float
    argument). Returns (budgets int64 [Cq], n_keep int32 [Cq]); empty query clusters get 0."""
    qbar, kbar = np.asarray(qbar, np.float64), np.asarray(kbar, np.float64)
    Cq, Ck = qbar.shape[0], kbar.shape[0]
    qs = [int(v) for v in q_sizes[:Cq]]
    ks = [int(v) for v in k_sizes[:Ck]]
    p = float(np.float32(p))
    budgets = np.zeros(Cq, dtype=np.int64)
    n_keep = np.zeros(Cq, dtype=np.int32)
    live = [b for b in range(Ck) if ks[b] > 0]
    for a in range(Cq):
        if qs[a] == 0 or not live:
            continue
        logit = {b: float(qbar[a] @ kbar[b]) * scale for b in live}
        m = max(logit.values())
        mass = {b: ks[b] * float(np.exp(logit[b] - m)) for b in live}
        order = sorted(live, key=lambda b: (-mass[b], b))
        total = 0.0
        for b in order:  # the row's total, added in the same order as the running sum below
            total += mass[b]
        run = 0.0
        keys = 0
        n_keep[a] = len(live)
        for n, b in enumerate(order, start=1):
            run += mass[b]
            keys += ks[b]
            if run >= p * total:
                n_keep[a] = n
                break
        budgets[a] = qs[a] * keys
    return budgets, n_keep


# --------------------------------------------------------------------------- attention


def dense_attention(Q, K, V, scale: float):
    """softmax(Q K^T * scale) V in fp64 (A_full of Eq. (2))."""
    Q, K, V = (np.asarray(t, np.float64) for t in (Q, K, V))
    L = (Q @ K.T) * scale
    L -= L.max(axis=1, keepdims=True)
    P = np.exp(L)
    return (P / P.sum(axis=1, keepdims=True)) @ V


def attention_map_comp(Q, K, lab_q, lab_k, kbar, mask, scale: float):
    """The compensated attention map of Eq. (1), rows [n_q, n_k], and the boolean
    per-entry mask M. Entries with M = 1 use the exact logit, the others the logit against
    the key's cluster mean (the text after Eq. (1): the product with M selects, it does
    not multiply a logit by zero)."""
    Q, K, kbar = (np.asarray(t, np.float64) for t in (Q, K, kbar))
    M = np.asarray(mask)[np.asarray(lab_q)][:, np.asarray(lab_k)]
    exact = (Q @ K.T) * scale
    comp = ((Q @ kbar.T) * scale)[:, np.asarray(lab_k)]
    L = np.where(M, exact, comp)
    L -= L.max(axis=1, keepdims=True)
    P = np.exp(L)
    return P / P.sum(axis=1, keepdims=True), M


def attention_comp(Q, K, V, lab_q, lab_k, kbar, vbar, mask, scale: float, row_chunk: int = 512):
    """Sparse attention output with linear compensation, Eq. (1) + Eq. (6), literally:

        A = softmax(where(M, Q K^T, Q Kbar^T) * scale);  O = (A*M) V + (A*(1-M)) Vbar

    lab_q[i] / lab_k[j] are the cluster (row / column of `mask`) of each query / key;
    kbar, vbar hold one row per key column of `mask` (rows of always-routed columns, e.g.
    the text tail, are never read through M = 0 and may hold anything finite).
    Works on any token order; pass permuted tensors with permuted labels to get the
    permuted output.
    """
    V64 = np.asarray(V, np.float64)
    vbar_rows = np.asarray(vbar, np.float64)[np.asarray(lab_k)]
    out = np.empty((Q.shape[0], V64.shape[1]), dtype=np.float64)
    for s in range(0, Q.shape[0], row_chunk):
        e = min(s + row_chunk, Q.shape[0])
        A, M = attention_map_comp(Q[s:e], K, lab_q[s:e], lab_k, kbar, mask, scale)
        out[s:e] = (A * M) @ V64 + (A * ~M) @ vbar_rows
    return out


# --------------------------------------------------------------------------- whole path


def scale_of(d: int) -> float:
    """1/sqrt(d) (Motivation: logits are q k^T / sqrt(d))."""
    return 1.0 / float(np.sqrt(np.float64(d)))


def hot_path_head(Q, K, V, init_q, init_k, iters: int, budget: int, n_tail: int = 0,
                  value_aware: bool = True, per_row: bool = False, top_p: Optional[float] = None):
    """All stages for one head, in the order the method runs them; returns a dict with
    every intermediate (used by the end-to-end parity test and the cpu_baseline timing).
    Q, K, V are [N, d] arrays (any float dtype holding the exact input values)."""
    Q32, K32, V32 = (np.asarray(t, np.float32) for t in (Q, K, V))
    N, d = Q32.shape
    nv = N - n_tail
    Cq, Ck = init_q.shape[0], init_k.shape[0]
    scale = scale_of(d)
    qbar, lab_q, qcnt, _ = kmeans(Q32[:nv], init_q, iters)
    kbar, lab_k, kcnt, vbar = kmeans(K32[:nv], init_k, iters, X2=V32[:nv])
    perm_q, qoff = permute(lab_q, Cq, n_tail)
    perm_k, koff = permute(lab_k, Ck, n_tail)
    Qp, Kp, Vp = Q32[perm_q], K32[perm_k], V32[perm_k]
    E, scores, m = probe_errors(qbar, kbar, vbar, Kp, Vp, koff, scale, value_aware)
    row_budgets = top_p_row_budgets(qbar, kbar, qcnt, kcnt, top_p, scale)[0] if top_p is not None else None
    mask, row_ptr, col_idx, cost = route(scores, qcnt, kcnt, budget, per_row, n_tail, n_tail, row_budgets)
    lq = np.repeat(np.arange(Cq + 1), np.diff(qoff))
    lk = np.repeat(np.arange(Ck + 1), np.diff(koff))
    kb = np.concatenate([kbar, np.zeros((1, d), np.float32)]) if n_tail else kbar
    vb = np.concatenate([vbar, np.zeros((1, d), np.float32)]) if n_tail else vbar
    Op = attention_comp(Qp, Kp, Vp, lq, lk, kb, vb, mask, scale)
    O = unpermute_rows(Op, perm_q)
    return dict(qbar=qbar, kbar=kbar, vbar=vbar, lab_q=lab_q, lab_k=lab_k, qcnt=qcnt, kcnt=kcnt,
                perm_q=perm_q, perm_k=perm_k, qoff=qoff, koff=koff, E=E, scores=scores, m=m,
                mask=mask, row_ptr=row_ptr, col_idx=col_idx, routed_cost=cost, Op=Op, O=O)
