"""Pins for the oracle's probe (Eq. (5), Eq. (7), Algorithm 1) and router
("Error-Aware Routing") -- CPU only."""
import itertools

import numpy as np
import pytest

from oracle import svgear_oracle as orc


def _setup(seed=0, Cq=5, Ck=7, d=8, n=60, empty=None):
    rng = np.random.default_rng(seed)
    qbar = rng.standard_normal((Cq, d))
    lab = np.sort(rng.integers(0, Ck, n))
    if empty is not None:
        lab = lab[lab != empty]
    n = lab.shape[0]
    centers_k = rng.standard_normal((Ck, d))
    centers_v = rng.standard_normal((Ck, d))
    Kp = centers_k[lab] + 0.3 * rng.standard_normal((n, d))
    Vp = centers_v[lab] + 0.3 * rng.standard_normal((n, d))
    off = np.zeros(Ck + 2, np.int32)
    off[1: Ck + 1] = np.cumsum(np.bincount(lab, minlength=Ck))
    off[Ck + 1] = off[Ck]
    kbar = np.zeros((Ck, d))
    vbar = np.zeros((Ck, d))
    for b in range(Ck):
        if off[b + 1] > off[b]:
            kbar[b] = Kp[off[b]: off[b + 1]].mean(0)
            vbar[b] = Vp[off[b]: off[b + 1]].mean(0)
    return qbar, kbar, vbar, Kp, Vp, off, lab


def test_probe_equals_entrywise_eq7_bruteforce():
    # Eq. (7) verbatim for every (query, key) entry with qbar_i per row, summed per block
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(1, empty=3)
    d = qbar.shape[1]
    scale = 1 / np.sqrt(d)
    E, scores, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, scale, True)
    q_sizes = np.array([3, 1, 4, 2, 5])
    row_cluster = np.repeat(np.arange(5), q_sizes)
    tot = np.zeros_like(E)
    for i, a in enumerate(row_cluster):
        for j, b in enumerate(lab):
            lhs = np.exp(qbar[a] @ kbar[b] * scale) * vbar[b]
            rhs = np.exp(qbar[a] @ Kp[j] * scale) * Vp[j]
            tot[a, b] += ((lhs - rhs) ** 2).sum()
    sizes = np.diff(off[:8])
    for a in range(5):
        for b in range(7):
            if sizes[b] == 0:
                assert E[a, b] == 0 and scores[a, b] == 0
                continue
            ratio = tot[a, b] / (q_sizes[a] * sizes[b])  # error-to-cost ratio of the text
            assert np.isclose(ratio * np.exp(-2 * m[a]), scores[a, b], rtol=1e-10)


def test_probe_plain_equals_entrywise_eq5():
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(2)
    scale = 0.37
    E, scores, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, scale, False)
    for a in range(qbar.shape[0]):
        tot = np.zeros(7)
        for j, b in enumerate(lab):
            tot[b] += (np.exp(qbar[a] @ kbar[b] * scale) - np.exp(qbar[a] @ Kp[j] * scale)) ** 2
        assert np.allclose(tot * np.exp(-2 * m[a]), E[a], rtol=1e-10)


def test_probe_zero_when_block_is_constant():
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(3)
    Kp = kbar[lab].copy()
    Vp = vbar[lab].copy()
    E, scores, _ = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, 0.3, True)
    assert np.abs(E).max() < 1e-24
    # only the values constant: error remains (keys still differ from their mean)
    _, _, _, Kp2, _, _, _ = _setup(3)
    E2, _, _ = orc.probe_errors(qbar, kbar, vbar, Kp2, Vp, off, 0.3, True)
    assert E2.max() > 1e-6


def test_probe_row_stabiliser_is_exp_minus_2m():
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(4)
    scale = 0.5
    E, _, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, scale, True)
    S = qbar @ kbar.T * scale
    assert np.allclose(m, S.max(1))
    # un-stabilised Eq. (7) block sums
    for a in range(qbar.shape[0]):
        for b in range(7):
            sl = slice(off[b], off[b + 1])
            raw = ((np.exp(S[a, b]) * vbar[b][None] - np.exp(Kp[sl] @ qbar[a] * scale)[:, None] * Vp[sl]) ** 2).sum()
            assert np.isclose(raw * np.exp(-2 * m[a]), E[a, b], rtol=1e-10)


def test_probe_block_error_merges_from_parts_held_in_other_units():
    # Any streaming evaluation (Algorithm 1) holds partial sums in units of its own running
    # stabiliser and converts at the end. The identity it needs: a sum of Eq. (7) terms held
    # with stabiliser m' is exp(2 (m_a - m')) times the same sum held with m_a, so a part is
    # brought back with exp(2 (m' - m_a)) -- the sign reading of the listing's last line.
    # Check it by cutting every key cluster into two parts, evaluating each part directly with a
    # DIFFERENT stabiliser (its own largest logit), and merging.
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(5, empty=2)
    Kp[::7] *= 4.0  # keys whose logit exceeds every centroid logit: a running maximum would move
    scale = 0.4
    E, _, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, scale, True)
    S = qbar @ kbar.T * scale
    assert ((Kp @ qbar.T * scale).max(0) > m).any()
    for a in range(qbar.shape[0]):
        for b in range(kbar.shape[0]):
            lo, hi = off[b], off[b + 1]
            if hi == lo:
                assert E[a, b] == 0
                continue
            merged = 0.0
            wrong_sign = 0.0
            cut = lo + (hi - lo) // 3
            for sl in (slice(lo, cut), slice(cut, hi)):
                if sl.stop == sl.start:
                    continue
                s = Kp[sl] @ qbar[a] * scale
                m_part = max(s.max(), S[a, b])  # this part's own stabiliser
                part = ((np.exp(S[a, b] - m_part) * vbar[b][None] - np.exp(s - m_part)[:, None] * Vp[sl]) ** 2).sum()
                merged += part * np.exp(2.0 * (m_part - m[a]))
                wrong_sign += part * np.exp(2.0 * (m[a] - m_part))
            assert np.isclose(merged, E[a, b], rtol=1e-11, atol=0)
            if abs(m_part - m[a]) > 1e-3:
                assert not np.isclose(wrong_sign, E[a, b], rtol=1e-6, atol=0)


def test_probe_printed_initial_term_differs_by_exp2S_vbar2():
    # Algorithm 1 as printed starts E at ||Y||^2; that adds exp(2(S-m))||vbar||^2 per block
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(6)
    scale = 0.4
    E, _, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, scale, True)
    S = qbar @ kbar.T * scale
    extra = np.exp(2 * (S - m[:, None])) * (vbar ** 2).sum(1)[None]
    assert extra.min() > 0  # so the two readings are distinguishable
    assert np.all(E + extra > E)


def test_probe_expanded_square_identity():
    qbar, kbar, vbar, Kp, Vp, off, lab = _setup(7)
    scale = 0.4
    E, _, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, off, scale, True)
    S = qbar @ kbar.T * scale
    for a in range(qbar.shape[0]):
        for b in range(7):
            sl = slice(off[b], off[b + 1])
            w = np.exp(Kp[sl] @ qbar[a] * scale - m[a])
            W = np.exp(S[a, b] - m[a])
            ex = (w * w * (Vp[sl] ** 2).sum(1)).sum() - 2 * W * (w * (Vp[sl] @ vbar[b])).sum() \
                + (off[b + 1] - off[b]) * W * W * (vbar[b] ** 2).sum()
            assert np.isclose(ex, E[a, b], rtol=1e-8, atol=1e-12)


# ----------------------------------------------------------------------------- route


def test_route_extremes_and_budget_invariant():
    rng = np.random.default_rng(0)
    Cq, Ck = 6, 9
    scores = rng.random((Cq, Ck))
    qs = rng.integers(1, 20, Cq)
    ks = rng.integers(1, 20, Ck)
    total = int(qs.sum() * ks.sum())
    mask, rp, ci, cost = orc.route(scores, qs, ks, total)
    assert mask.all() and cost == total and rp[-1] == Cq * Ck
    mask, rp, ci, cost = orc.route(scores, qs, ks, 0)
    assert not mask.any() and cost == 0 and rp[-1] == 0
    for budget in [total // 7, total // 3, total // 2]:
        mask, rp, ci, cost = orc.route(scores, qs, ks, budget)
        assert cost == int((np.outer(qs, ks) * mask).sum()) <= budget
        # the best unrouted block is the one the walk stopped at: it must not fit
        un = [(-scores[a, b], a * Ck + b, a, b) for a in range(Cq) for b in range(Ck) if not mask[a, b]]
        _, _, a, b = min(un)
        assert cost + qs[a] * ks[b] > budget
        # every routed block outranks every unrouted one
        worst_routed = max((-scores[a, b], a * Ck + b) for a in range(Cq) for b in range(Ck) if mask[a, b])
        assert worst_routed < min(un)[:2]
        # CSR consistent with the mask, ascending columns
        for a in range(Cq):
            assert ci[rp[a]: rp[a + 1]].tolist() == np.nonzero(mask[a])[0].tolist()


def test_route_ties_lowest_index_and_nan_first():
    scores = np.array([[1.0, 1.0, 1.0], [1.0, np.nan, 0.5]])
    qs, ks = [2, 2], [3, 3, 3]
    mask, _, _, cost = orc.route(scores, qs, ks, 6 * 3)  # room for three blocks
    assert mask.tolist() == [[True, True, False], [False, True, False]]
    assert cost == 18


def test_route_skips_empty_clusters():
    scores = np.full((3, 3), 5.0)
    mask, rp, ci, cost = orc.route(scores, [4, 0, 4], [0, 2, 2], 10 ** 6)
    assert mask.tolist() == [[False, True, True], [False, False, False], [False, True, True]]
    assert cost == 32


def test_route_greedy_vs_bruteforce_knapsack():
    # all 2^16 masks of a 4x4 block grid. Equal costs: greedy by ratio is optimal.
    rng = np.random.default_rng(11)
    scores = rng.random((4, 4))
    qs, ks = [3, 3, 3, 3], [5, 5, 5, 5]
    val = scores * 15 * 3  # block value = |q_a| * E_ab = |q_a||k_b| * score
    for nblocks in [0, 1, 5, 16]:
        budget = 15 * nblocks + 7
        mask, _, _, cost = orc.route(scores, qs, ks, budget)
        got = (val * mask).sum()
        best = 0.0
        for bits in range(1 << 16):
            if bin(bits).count("1") * 15 <= budget:
                sel = np.array([(bits >> t) & 1 for t in range(16)], bool).reshape(4, 4)
                best = max(best, (val * sel).sum())
        assert np.isclose(got, best)
    # unequal costs: the classical greedy guarantee OPT <= greedy + value(first rejected)
    qs, ks = [1, 4, 2, 6], [3, 1, 5, 2]
    cost_m = np.outer(qs, ks)
    val = scores * cost_m
    budget = int(cost_m.sum() * 0.4)
    mask, _, _, cost = orc.route(scores, qs, ks, budget)
    order = sorted(((-scores[a, b], a * 4 + b) for a in range(4) for b in range(4) if not mask[a, b]))
    a, b = divmod(order[0][1], 4)
    best = 0.0
    flat_c, flat_v = cost_m.ravel(), val.ravel()
    for bits in range(1 << 16):
        sel = np.array([(bits >> t) & 1 for t in range(16)], bool)
        if flat_c[sel].sum() <= budget:
            best = max(best, flat_v[sel].sum())
    assert (val * mask).sum() <= best <= (val * mask).sum() + val[a, b] + 1e-12


def test_route_tail_blocks_forced_and_charged():
    rng = np.random.default_rng(12)
    scores = rng.random((3, 4))
    qs, ks = [5, 6, 7], [2, 3, 4, 5]
    tq = tk = 3
    nq, nk = sum(qs) + tq, sum(ks) + tk
    forced = tq * nk + nq * tk - tq * tk
    mask, rp, ci, cost = orc.route(scores, qs, ks, forced + 5 * 2 - 1, n_tail_q=tq, n_tail_k=tk)
    assert mask.shape == (4, 5)
    assert mask[3].all() and mask[:, 4].all()
    assert cost >= forced
    mask2, _, _, cost2 = orc.route(scores, qs, ks, 0, n_tail_q=tq, n_tail_k=tk)
    assert cost2 == forced and mask2[:3, :4].sum() == 0


def test_route_per_row_budgets():
    rng = np.random.default_rng(13)
    scores = rng.random((4, 6))
    qs, ks = [3, 5, 2, 7], [4, 4, 2, 6, 1, 3]
    nq, nk = sum(qs), sum(ks)
    budget = int(0.5 * nq * nk)
    mask, _, _, cost = orc.route(scores, qs, ks, budget, per_row=True)
    for a in range(4):
        row_budget = budget * qs[a] // nq
        row_cost = int((np.array(ks) * mask[a]).sum()) * qs[a]
        assert row_cost <= row_budget
        m1, _, _, c1 = orc.route(scores[a: a + 1], [qs[a]], ks, row_budget)
        assert m1[0].tolist() == mask[a].tolist()
    assert cost == int((np.outer(qs, ks) * mask).sum())


# ------------------------------------------------------------------ top-p row budgets (reading)


def _top_p_case(seed, Cq=6, Ck=11, d=8, empty=(4,)):
    rng = np.random.default_rng(seed)
    qbar = rng.standard_normal((Cq, d)) * 1.5
    kbar = rng.standard_normal((Ck, d)) * 1.5
    q_sizes = rng.integers(1, 9, Cq)
    k_sizes = rng.integers(1, 30, Ck)
    for b in empty:
        k_sizes[b] = 0
    return qbar, kbar, q_sizes, k_sizes


def test_top_p_budget_is_cost_of_softmax_mass_prefix_bruteforce():
    # brute force over every subset size: the kept set is the n heaviest clusters (centroid
    # softmax mass of a key set = sum of |k_b| softmax terms), n the least that reaches p
    scale = 0.4
    for seed in range(6):
        qbar, kbar, q_sizes, k_sizes = _top_p_case(seed)
        for p in (0.3, 0.6, 0.9):
            budgets, n_keep = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, p, scale)
            for a in range(qbar.shape[0]):
                logits = np.repeat(qbar[a] @ kbar.T * scale, k_sizes)  # one pseudo-key per key of a cluster
                owner = np.repeat(np.arange(kbar.shape[0]), k_sizes)
                soft = np.exp(logits - logits.max())
                soft /= soft.sum()
                share = np.bincount(owner, weights=soft, minlength=kbar.shape[0])
                order = np.argsort(-share, kind="stable")
                n = 1
                while share[order[:n]].sum() < p - 1e-9:
                    n += 1
                assert n_keep[a] == n
                assert budgets[a] == q_sizes[a] * k_sizes[order[:n]].sum()


def test_top_p_uniform_logits_closed_form():
    # equal centroids, equal sizes: every cluster has the same mass, n = ceil(p Ck), lowest indices
    Ck, Cq, d = 10, 3, 4
    kbar = np.tile(np.arange(1.0, d + 1), (Ck, 1))
    qbar = np.ones((Cq, d))
    q_sizes = np.array([2, 0, 5])
    k_sizes = np.full(Ck, 7)
    for p, n in ((0.05, 1), (0.09, 1), (0.11, 2), (0.5, 5), (0.95, 10), (1.0, 10)):
        budgets, n_keep = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, p, 0.5)
        assert list(n_keep) == [n, 0, n]
        assert list(budgets) == [2 * 7 * n, 0, 5 * 7 * n]


def test_top_p_limits_monotone_and_empty_clusters():
    qbar, kbar, q_sizes, k_sizes = _top_p_case(3, empty=(0, 7))
    scale = 0.15
    tiny, n_tiny = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, 1e-6, scale)
    mass = k_sizes[None, :] * np.exp(qbar @ kbar.T * scale)
    heaviest = mass.argmax(axis=1)
    assert np.all(n_tiny == 1) and np.array_equal(tiny, q_sizes * k_sizes[heaviest])
    full, n_full = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, 1.0, scale)
    # p = 1 keeps every non-empty cluster
    assert np.all(n_full == (k_sizes > 0).sum()) and np.array_equal(full, q_sizes * k_sizes.sum())
    prev = tiny
    for p in np.linspace(0.05, 1.0, 20):
        cur, _ = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, float(p), scale)
        assert np.all(cur >= prev)
        prev = cur
    # a far-away cluster carries almost no mass: it is the last of the order, dropped for any
    # p below 1 by a hair and kept at p = 1 (the masses are real numbers, nothing is cut off)
    kbar2 = kbar.copy()
    kbar2[5] = -25.0 * qbar[0] / np.linalg.norm(qbar[0])
    share = k_sizes * np.exp(qbar[0] @ kbar2.T * scale)
    assert 1e-12 < share[5] / share.sum() < 2.0 ** -24  # tiny, yet far above the rounding of an fp64 sum
    _, n2 = orc.top_p_row_budgets(qbar[:1], kbar2, q_sizes[:1], k_sizes, 1.0, scale)
    assert n2[0] == (k_sizes > 0).sum()
    _, n3 = orc.top_p_row_budgets(qbar[:1], kbar2, q_sizes[:1], k_sizes, 1.0 - 1e-6, scale)
    assert n3[0] == (k_sizes > 0).sum() - 1


def test_top_p_query_size_scaling_and_key_cluster_relabelling():
    # the kept prefix does not depend on |q_a| (the budget scales with it) nor on how the key
    # clusters are numbered
    qbar, kbar, q_sizes, k_sizes = _top_p_case(5, empty=())
    b1, n1 = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, 0.7, 0.3)
    b2, n2 = orc.top_p_row_budgets(qbar, kbar, 3 * q_sizes, k_sizes, 0.7, 0.3)
    assert np.array_equal(n1, n2) and np.array_equal(3 * b1, b2)
    perm = np.random.default_rng(0).permutation(kbar.shape[0])
    b3, n3 = orc.top_p_row_budgets(qbar, kbar[perm], q_sizes, k_sizes[perm], 0.7, 0.3)
    assert np.array_equal(n1, n3) and np.array_equal(b1, b3)


def test_route_with_row_budgets_spends_each_rows_own_budget():
    rng = np.random.default_rng(9)
    Cq, Ck = 5, 9
    scores = rng.random((Cq, Ck))
    q_sizes = rng.integers(1, 6, Cq)
    k_sizes = rng.integers(1, 12, Ck)
    row_budgets = np.array([0, 10 ** 9, 37, 5, 60]) * 1
    mask, row_ptr, col_idx, cost = orc.route(scores, q_sizes, k_sizes, 0, row_budgets=row_budgets, n_tail_k=4)
    assert mask[:, Ck].all()  # forced tail column, on top of the row budgets
    assert not mask[0, :Ck].any() and mask[1, :Ck].all()
    total = 0
    for a in range(Cq):
        spent = 0
        for b in np.argsort(-scores[a], kind="stable"):
            c = q_sizes[a] * k_sizes[b]
            if spent + c > row_budgets[a]:
                break
            spent += c
            assert mask[a, b]
        assert spent == (mask[a, :Ck] * q_sizes[a] * k_sizes).sum()
        total += spent + q_sizes[a] * 4
    assert cost == total


def test_top_p_then_route_reproduces_top_p_selection_when_scores_are_the_masses():
    # if the error ratio handed to the router is the mass per key, the router's order is the top-p
    # order for equal-size key clusters, so the routed set is exactly the top-p prefix
    rng = np.random.default_rng(11)
    Cq, Ck, d = 4, 12, 6
    qbar, kbar = rng.standard_normal((Cq, d)), rng.standard_normal((Ck, d))
    q_sizes, k_sizes = rng.integers(1, 5, Cq), np.full(Ck, 6)
    budgets, n_keep = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, 0.8, 0.5)
    mass = np.exp(qbar @ kbar.T * 0.5)
    mask = orc.route(mass, q_sizes, k_sizes, 0, row_budgets=budgets)[0]
    for a in range(Cq):
        top = np.argsort(-mass[a], kind="stable")[: n_keep[a]]
        assert set(np.nonzero(mask[a])[0]) == set(top)
