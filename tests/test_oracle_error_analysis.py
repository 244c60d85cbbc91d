"""The error-analysis study (oracle/error_analysis.py, CPU only): sanity and the qualitative
findings of the paper's "Error Analysis" section on a small seeded synthetic layer."""
import numpy as np

from oracle import error_analysis as ea
from oracle import svgear_oracle as orc
from workloads.generators import Workload

SMALL = Workload("study_small", 1, 1, 3 * 12 * 16, 0, 32, 12, 36, 6, 0.25, "f32", 27, 1.0, 0.3,
                 (3, 12, 16), (3, 3, 3), 5)


def test_top_p_selects_shortest_prefix_reaching_the_mass():
    qbar = np.array([[1.0, 0.0]])
    kbar = np.array([[2.0, 0.0], [1.0, 0.0], [0.0, 0.0], [5.0, 0.0]])
    sizes = np.array([1, 1, 2, 0])  # the last cluster is empty and must never be chosen
    mass = sizes[:3] * np.exp([2.0, 1.0, 0.0])  # scale = 1
    order = np.argsort(-mass)
    for p in (0.3, 0.6, 0.8, 0.99, 1.0):
        m = ea.top_p_mask(qbar, kbar, sizes, p, 1.0)[0]
        keep = int(m.sum())
        cum = np.cumsum(mass[order])
        assert not m[3]
        assert set(np.flatnonzero(m)) == set(order[:keep])
        assert cum[keep - 1] >= p * cum[-1] - 1e-12 and (keep == 1 or cum[keep - 2] < p * cum[-1])


def test_exact_block_errors_match_entrywise_definition():
    rng = np.random.default_rng(0)
    Q, K = rng.normal(size=(7, 4)), rng.normal(size=(9, 4))
    lab_q = np.array([0, 1, 1, 0, 2, 2, 1])
    lab_k = np.array([0, 0, 1, 2, 2, 2, 1, 0, 3])
    kbar = np.stack([K[lab_k == c].mean(0) for c in range(4)])
    E = ea.exact_block_errors(Q, K, lab_q, lab_k, kbar, 3, 4, 0.5)
    ref = np.zeros((3, 4))
    shift = max(((Q @ K.T) * 0.5).max(), ((Q @ kbar.T) * 0.5).max())
    for i in range(7):
        for j in range(9):
            e = np.exp(Q[i] @ kbar[lab_k[j]] * 0.5 - shift) - np.exp(Q[i] @ K[j] * 0.5 - shift)
            ref[lab_q[i], lab_k[j]] += e * e
    assert np.allclose(E, ref, rtol=1e-10, atol=0)


def test_everything_selected_reproduces_dense_map():
    scale = orc.scale_of(SMALL.d)
    Q, K, V, qbar, lab_q, q_cnt, kbar, vbar, lab_k, k_cnt = ea.cluster(SMALL, 0, SMALL.Cq, SMALL.Ck, 3)
    full = ea.top_p_mask(qbar, kbar, k_cnt, 1.0, scale)
    assert np.array_equal(full, np.broadcast_to(k_cnt[None, :] > 0, full.shape))
    A = ea.dense_map(Q, K, scale)
    assert ea.map_mse(ea.dropped_map(Q, K, lab_q, lab_k, full, scale), A) < 1e-30
    assert ea.map_mse(orc.attention_map_comp(Q, K, lab_q, lab_k, kbar, full, scale)[0], A) < 1e-30


def test_selection_strategies_order_as_in_the_paper():
    # "Strategy of block selection": at equal routed cost, compensation lowers the error of
    # top-p selection by more than an order of magnitude; routing by the exact errors (which
    # needs all logits) is the reference point and beats both practical rules; error-aware
    # routing beats top-p selection with compensation at the two higher densities of this
    # small seeded layer (at p = 0.6 the two are within 10 % of each other, in the other order).
    rows = ea.selection_study(SMALL, ps=(0.6, 0.85, 0.95), iters=6)
    for p, dens, top, top_comp, ear_comp, exact_comp in rows:
        assert 0.0 < dens < 1.0
        assert top > 10 * max(top_comp, ear_comp)
        assert exact_comp < min(top_comp, ear_comp)
        assert ear_comp < 1.1 * top_comp
    for p, dens, top, top_comp, ear_comp, exact_comp in rows[1:]:
        assert ear_comp < top_comp


def test_clustering_error_is_the_mean_over_queries_not_the_maximum():
    # Proposition 1: delta_q^2 = (1/N_q) sum_i |q_i - qbar_i|^2. Two clusters built by hand:
    # cluster 0 = {(0,0), (2,0)} with mean (1,0): squared distances 1, 1;
    # cluster 1 = {(10,0), (10,6), (10,0)} with mean (10,2): squared distances 4, 16, 4.
    # mean = (1 + 1 + 4 + 16 + 4) / 5 = 5.2, whereas the largest is 16 and the sum 26.
    Q = np.array([[0.0, 0.0], [10.0, 0.0], [2.0, 0.0], [10.0, 6.0], [10.0, 0.0]])
    lab = np.array([0, 1, 0, 1, 1])
    qbar = np.array([[1.0, 0.0], [10.0, 2.0]])
    assert ea.clustering_error(Q, qbar, lab) == 5.2
    # one cluster holding everything: the mean squared distance to the grand mean is the
    # trace of the (biased) covariance matrix
    rng = np.random.default_rng(3)
    X = rng.normal(size=(50, 4)) * np.array([1.0, 2.0, 0.5, 3.0])
    got = ea.clustering_error(X, X.mean(0, keepdims=True), np.zeros(50, int))
    assert np.isclose(got, np.trace(np.cov(X.T, bias=True)), rtol=1e-12)
    # the study reports this quantity: its rows equal k-means inertia / N_q
    Qs, _, _, qbar_s, lab_q, _, _, _, _, _ = ea.cluster(SMALL, 0, 16, SMALL.Ck, 6)
    row = ea.clustering_study(SMALL, cqs=(16,), iters=6)[0]
    inertia = sum(float(((Qs[i].astype(np.float64) - qbar_s[lab_q[i]].astype(np.float64)) ** 2).sum())
                  for i in range(Qs.shape[0]))
    assert np.isclose(row[1], inertia / Qs.shape[0], rtol=1e-12)


def test_more_query_clusters_tighten_clustering_error():
    # "Effect of clustering": delta_q^2 falls as the number of query clusters grows, and the
    # attention-map error with it (Proposition 1 ties the two together).
    rows = ea.clustering_study(SMALL, cqs=(4, 16, 64), p=0.85, iters=6)
    dq = [r[1] for r in rows]
    mse = [r[2] for r in rows]
    assert dq[0] > dq[1] > dq[2]
    assert mse[0] > mse[2]


def test_top_p_mask_of_the_study_keeps_as_many_clusters_as_the_row_budget_rule():
    # the float-valued selection used in the study and the integer-unit budget rule of the
    # oracle are two codings of the same reading; on generic data they keep the same prefix
    from oracle import svgear_oracle as orc
    rng = np.random.default_rng(5)
    qbar, kbar = rng.standard_normal((7, 16)), rng.standard_normal((13, 16))
    k_sizes = rng.integers(0, 40, 13)
    q_sizes = rng.integers(1, 9, 7)
    for p in (0.4, 0.7, 0.9):
        mask = ea.top_p_mask(qbar, kbar, k_sizes, p, 0.25)
        budgets, n_keep = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, p, 0.25)
        assert np.array_equal(mask.sum(axis=1), n_keep)
        assert np.array_equal((mask * k_sizes[None, :]).sum(axis=1) * q_sizes, budgets)
