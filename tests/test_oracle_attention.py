"""Pins for the oracle's compensated attention (Eq. (1), Eq. (6), Algorithm 2,
Proposition 1) -- CPU only."""
import numpy as np
import torch

from oracle import svgear_oracle as orc
from workloads import get_workload, make_qkv, kmeans_init_indices, budget_pairs


def _toy(seed=0, nq=40, nk=70, d=16, Cq=4, Ck=6):
    rng = np.random.default_rng(seed)
    lq = np.sort(rng.integers(0, Cq, nq))
    lk = np.sort(rng.integers(0, Ck, nk))
    ck = rng.standard_normal((Ck, d))
    Q = rng.standard_normal((nq, d))
    K = ck[lk] + 0.4 * rng.standard_normal((nk, d))
    V = rng.standard_normal((nk, d))
    kbar = np.stack([K[lk == b].mean(0) if (lk == b).any() else np.zeros(d) for b in range(Ck)])
    vbar = np.stack([V[lk == b].mean(0) if (lk == b).any() else np.zeros(d) for b in range(Ck)])
    ks = np.bincount(lk, minlength=Ck)
    mask = rng.random((Cq, Ck)) < 0.4
    return Q, K, V, lq, lk, kbar, vbar, ks, mask


def test_all_routed_is_dense_attention():
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy(1)
    scale = 0.25
    O = orc.attention_comp(Q, K, V, lq, lk, kbar, vbar, np.ones_like(mask), scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None], scale=scale)[0].numpy()
    assert np.abs(O - ref).max() < 1e-12
    assert np.abs(orc.dense_attention(Q, K, V, scale) - ref).max() < 1e-12


def test_identical_keys_per_cluster_make_compensation_exact():
    # identical keys inside each cluster give identical attention weights inside the
    # cluster, so sum_j A v_j = |k_b| A vbar_b for ANY mask, values free to differ
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy(2)
    K = kbar[lk].copy()
    dense = orc.dense_attention(Q, K, V, 0.3)
    for m in [mask, np.zeros_like(mask), np.ones_like(mask), ~mask]:
        O = orc.attention_comp(Q, K, V, lq, lk, kbar, vbar, m, 0.3)
        assert np.abs(O - dense).max() < 1e-12
    # and it is NOT exact once the keys differ, so the test above is not vacuous
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy(2)
    O = orc.attention_comp(Q, K, V, lq, lk, kbar, vbar, np.zeros_like(mask), 0.3)
    assert np.abs(O - orc.dense_attention(Q, K, V, 0.3)).max() > 1e-3


def test_map_rows_sum_to_one_and_single_cluster_gives_mean_value():
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy(3)
    A, M = orc.attention_map_comp(Q, K, lq, lk, kbar, mask, 0.3)
    assert np.allclose(A.sum(1), 1.0, atol=1e-14)
    assert M.shape == A.shape and M.dtype == bool
    # block structure of M
    for i in range(Q.shape[0]):
        assert np.array_equal(M[i], mask[lq[i]][lk])
    one = np.zeros(K.shape[0], int)
    O = orc.attention_comp(Q, K, V, lq * 0, one, K.mean(0)[None], V.mean(0)[None], np.zeros((1, 1), bool), 0.3)
    assert np.allclose(O, V.mean(0)[None], atol=1e-13)


def test_compensated_entries_use_centroid_logit_and_mean_value():
    # one query, two clusters, second one skipped: closed form by hand
    q = np.array([[1.0, 2.0]])
    K = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 2.0], [4.0, 0.0]])
    V = np.array([[1.0, 0.0], [0.0, 1.0], [5.0, 5.0], [7.0, 1.0]])
    lk = np.array([0, 0, 1, 1])
    kbar = np.array([[0.5, 0.5], [3.0, 1.0]])
    vbar = np.array([[0.5, 0.5], [6.0, 3.0]])
    mask = np.array([[True, False]])
    s = 0.5
    e = np.exp(np.array([1.0 * s, 2.0 * s, 5.0 * s, 5.0 * s]))  # last two: q.kbar_1 = 5
    want = (e[0] * V[0] + e[1] * V[1] + (e[2] + e[3]) * vbar[1]) / e.sum()
    O = orc.attention_comp(q, K, V, np.array([0]), lk, kbar, vbar, mask, s)
    assert np.allclose(O[0], want, atol=1e-14)


def _toy_with_empty_cluster_and_unrouted_row(seed):
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy(seed)
    mask[2] = False  # a query cluster with nothing routed
    lk2 = lk.copy()
    lk2[lk2 == 3] = 4  # an empty key cluster
    kbar = np.stack([K[lk2 == b].mean(0) if (lk2 == b).any() else np.zeros(K.shape[1]) for b in range(6)])
    vbar = np.stack([V[lk2 == b].mean(0) if (lk2 == b).any() else np.zeros(V.shape[1]) for b in range(6)])
    return Q, K, V, lq, lk2, kbar, vbar, np.bincount(lk2, minlength=6), mask


def test_compensation_equals_dense_attention_over_keys_replaced_by_their_cluster_mean():
    # Eq. (1) + Eq. (6) say: a skipped key behaves as if it sat at its cluster's mean key and
    # carried the cluster's mean value. So plain dense softmax attention over the key/value set
    # in which every key of a skipped block is REPLACED by (kbar_b, vbar_b) -- |k_b| identical
    # copies, which is where the ln|k_b| of the pseudo-key form comes from -- must give the same
    # rows. The replacement depends on the query's cluster, so it is done per query cluster.
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy_with_empty_cluster_and_unrouted_row(4)
    O = orc.attention_comp(Q, K, V, lq, lk, kbar, vbar, mask, 0.3)
    for a in np.unique(lq):
        routed = mask[a][lk]
        K_a = np.where(routed[:, None], K, kbar[lk])
        V_a = np.where(routed[:, None], V, vbar[lk])
        want = orc.dense_attention(Q[lq == a], K_a, V_a, 0.3)
        assert np.abs(O[lq == a] - want).max() < 1e-12


def test_routed_part_and_compensated_part_merge_by_their_log_sum_exp():
    # The two-stage form (Algorithm 2; also what a split into separate kernels relies on): the
    # routed keys alone give (O_r, LSE_r), the skipped non-empty clusters alone -- ONE pseudo-key
    # each, logit q.kbar_b*scale + ln|k_b|, value vbar_b -- give (O_c, LSE_c), and
    #   O = (e^{LSE_r} O_r + e^{LSE_c} O_c) / (e^{LSE_r} + e^{LSE_c}).
    # Written with whole-array softmaxes (no running quantities); a part with no entries has
    # weight zero.
    Q, K, V, lq, lk, kbar, vbar, ks, mask = _toy_with_empty_cluster_and_unrouted_row(4)
    scale = 0.3
    O = orc.attention_comp(Q, K, V, lq, lk, kbar, vbar, mask, scale)

    def part(logits, values):  # softmax-weighted mean and log-sum-exp of one set of entries
        if logits.size == 0:
            return np.zeros(values.shape[1]), -np.inf
        mx = logits.max()
        w = np.exp(logits - mx)
        return (w @ values) / w.sum(), mx + np.log(w.sum())

    for i in range(Q.shape[0]):
        a = lq[i]
        routed = mask[a][lk]
        skipped = np.flatnonzero(~mask[a] & (ks > 0))
        o_r, lse_r = part(K[routed] @ Q[i] * scale, V[routed])
        o_c, lse_c = part(kbar[skipped] @ Q[i] * scale + np.log(ks[skipped]), vbar[skipped])
        top = max(lse_r, lse_c)
        w_r, w_c = np.exp(lse_r - top), np.exp(lse_c - top)
        assert np.abs((w_r * o_r + w_c * o_c) / (w_r + w_c) - O[i]).max() < 1e-12


def test_proposition1_bound_holds_on_tiny_workload():
    wl = get_workload("tiny")
    Q, K, V = make_qkv(wl)
    Q, K, V = Q[0, 0].numpy(), K[0, 0].numpy(), V[0, 0].numpy()
    iq = kmeans_init_indices(0, 0, 0, wl.N, wl.Cq)
    ik = kmeans_init_indices(0, 0, 1, wl.N, wl.Ck)
    r = orc.hot_path_head(Q, K, V, Q[iq], K[ik], 3, budget_pairs(wl.rho, wl.N, wl.N), value_aware=False)
    scale = orc.scale_of(wl.d)
    n = 1024  # a quarter of the query rows keeps the materialised maps small
    rows = np.arange(0, wl.N, wl.N // n)
    Qs, lq = Q[rows].astype(np.float64), r["lab_q"][rows]
    A_sp, M = orc.attention_map_comp(Qs, K, lq, r["lab_k"], r["kbar"], r["mask"], scale)
    L = (Qs @ K.astype(np.float64).T) * scale
    Z = np.exp(L).sum(1)  # softmax normaliser of the full map (logits here stay < 700)
    A_full = np.exp(L) / Z[:, None]
    lhs = ((A_sp - A_full) ** 2).sum() / (n * wl.N)
    qb = r["qbar"].astype(np.float64)[lq]
    kb = r["kbar"].astype(np.float64)[r["lab_k"]]
    eps2 = (np.exp((qb * 1.0) @ r["kbar"].astype(np.float64).T * scale)[:, r["lab_k"]]
            - np.exp((qb @ K.astype(np.float64).T) * scale)) ** 2
    first = 2.0 / (n * wl.N) * ((~M) * eps2 / (Z ** 2)[:, None]).sum()
    delta_q2 = ((Qs - qb) ** 2).sum(1).mean()
    kmax2 = (K.astype(np.float64) ** 2).sum(1).max()
    rhs = first + 8.0 * delta_q2 * kmax2 / (wl.N * wl.d)
    assert lhs <= rhs
    assert kb.shape == K.shape


def test_hot_path_head_runs_and_is_close_to_dense_on_tiny():
    wl = get_workload("tiny")
    Q, K, V = make_qkv(wl)
    Q, K, V = Q[0, 0].numpy(), K[0, 0].numpy(), V[0, 0].numpy()
    iq = kmeans_init_indices(0, 0, 0, wl.N, wl.Cq)
    ik = kmeans_init_indices(0, 0, 1, wl.N, wl.Ck)
    budget = budget_pairs(wl.rho, wl.N, wl.N)
    r = orc.hot_path_head(Q, K, V, Q[iq], K[ik], 4, budget)
    assert r["routed_cost"] <= budget
    dense = orc.dense_attention(Q, K, V, orc.scale_of(wl.d))
    rel = np.linalg.norm(r["O"] - dense) / np.linalg.norm(dense)
    r0 = orc.hot_path_head(Q, K, V, Q[iq], K[ik], 4, 0)
    rel0 = np.linalg.norm(r0["O"] - dense) / np.linalg.norm(dense)
    assert rel <= rel0 + 1e-12  # routing exact blocks cannot hurt here
    rfull = orc.hot_path_head(Q, K, V, Q[iq], K[ik], 4, wl.N * wl.N)
    assert np.abs(rfull["O"] - dense).max() < 1e-10
