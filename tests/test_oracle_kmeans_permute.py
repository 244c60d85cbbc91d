"""Pins for the oracle's k-means and permutation (CPU only).

The paper (Methodology, "Problem Formulation") fixes only that clusters come from k-means
and that centroids are cluster means; these tests pin the oracle to textbook facts about
Lloyd's algorithm, to brute force and to scipy's implementation.
"""
from fractions import Fraction

import numpy as np
import pytest
from scipy.cluster.vq import kmeans2

from oracle import svgear_oracle as orc
from workloads import get_workload, make_qkv, kmeans_init_indices


def _brute_assign64(X, C):
    d2 = ((X[:, None, :].astype(np.float64) - C[None, :, :].astype(np.float64)) ** 2).sum(-1)
    order = np.sort(d2, axis=1)
    margin = order[:, 1] - order[:, 0] if C.shape[0] > 1 else np.full(X.shape[0], np.inf)
    return d2.argmin(1), margin


def test_assign_matches_bruteforce_distance():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((700, 64)).astype(np.float32)
    C = rng.standard_normal((37, 64)).astype(np.float32)
    lab = orc.kmeans_assign(X, C)
    ref, margin = _brute_assign64(X, C)
    clear = margin > 1e-3  # fp32 evaluation can only differ from fp64 on near-ties
    assert clear.mean() > 0.99
    assert np.array_equal(lab[clear], ref[clear])
    # on near-ties the chosen centroid must still be within rounding of the best
    d2 = ((X[:, None] - C[None]) ** 2).sum(-1)
    assert np.all(d2[np.arange(700), lab] - d2.min(1) <= 1e-3)


def test_assign_is_not_transposed_or_sign_flipped():
    # a point sitting on centroid 3 must get label 3, also when another centroid has a
    # larger dot product with it (catches dropping |c|^2 or flipping the sign of the dot)
    C = np.zeros((5, 8), np.float32)
    C[3] = 1.0
    C[4] = 5.0  # much larger dot product with x, but far away
    X = np.ones((1, 8), np.float32)
    assert orc.kmeans_assign(X, C)[0] == 3
    X2 = -np.ones((1, 8), np.float32)
    C2 = np.stack([np.full(8, -1.0), np.full(8, 1.0)]).astype(np.float32)
    assert orc.kmeans_assign(X2, C2)[0] == 0


def test_assign_ties_go_to_lowest_index():
    rng = np.random.default_rng(1)
    c = rng.standard_normal((4, 16)).astype(np.float32)
    C = np.concatenate([c, c, c])  # every centroid appears three times
    X = rng.standard_normal((200, 16)).astype(np.float32)
    lab = orc.kmeans_assign(X, C)
    assert lab.max() < 4


def _round_to_f32(x: Fraction) -> np.float32:
    """The float32 nearest to the rational x, ties to the even mantissa (IEEE round-to-nearest-even)."""
    f = np.float32(float(x))  # within one float32 step of the answer: pick among it and its neighbours
    cands = sorted({f, np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))}, key=float)
    best = min(abs(Fraction(float(c)) - x) for c in cands)
    near = [c for c in cands if abs(Fraction(float(c)) - x) == best]
    if len(near) == 1:
        return near[0]
    even = [c for c in near if (c.view(np.uint32) & np.uint32(1)) == 0]
    return even[0]


def _fma32(a, b, c) -> np.float32:
    """fmaf(a, b, c): the product and the sum exact (rationals), ONE rounding to float32."""
    return _round_to_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def _fixed_order_scores(x, C, fma=_fma32, order=None, cn_first=False):
    out = []
    ts = list(range(x.shape[0])) if order is None else order
    for j in range(C.shape[0]):
        dot = np.float32(0)
        cn = np.float32(0)
        for t in ts:
            dot = fma(x[t], C[j, t], dot)
        for t in ts:
            cn = fma(C[j, t], C[j, t], cn)
        out.append(fma(np.float32(-2.0), dot, cn))
    return np.array(out, np.float32)


def test_round_to_f32_helper_rounds_ties_to_even():
    one = Fraction(1)
    ulp = Fraction(1, 1 << 23)
    assert _round_to_f32(one + ulp / 2) == np.float32(1.0)                    # tie -> even (1.0)
    assert _round_to_f32(one + ulp + ulp / 2) == np.float32(1.0) + np.float32(2.0 ** -22)  # tie -> even
    assert _round_to_f32(one + ulp / 2 + Fraction(1, 1 << 60)) == np.nextafter(np.float32(1), np.float32(2))
    # a case where rounding to double first and then to single goes wrong: 1 + 2^-24 + 2^-60
    x = one + Fraction(1, 1 << 24) + Fraction(1, 1 << 60)
    assert np.float32(float(x)) == np.float32(1.0) and _round_to_f32(x) != np.float32(1.0)


def test_assign_fixed_fp32_order_bit_for_bit_against_exact_fma_emulation():
    # The documented order -- x.c and |c|^2 each ONE fma chain over t = 0..d-1, then
    # fma(-2, dot, cn), lowest index on ties -- retraced with exactly rounded fused
    # multiply-adds (rational arithmetic, one rounding): scores and labels must be IDENTICAL.
    rng = np.random.default_rng(2)
    X = rng.standard_normal((24, 32)).astype(np.float32)
    C = rng.standard_normal((6, 32)).astype(np.float32)
    C[4] = C[1]  # an exact tie between two centroids: the lower index must win
    lab, best = orc.kmeans_assign(X, C, return_scores=True)
    n_unfused = n_reversed = 0
    for i in range(X.shape[0]):
        scores = _fixed_order_scores(X[i], C)
        assert scores.min().view(np.uint32) == best[i].view(np.uint32)
        assert int(np.flatnonzero(scores == scores.min())[0]) == lab[i]
        assert lab[i] != 4
        # planted mistakes must be visible at this strictness: a separate multiply and add
        # (two roundings), and the chain run in the opposite order, each change some best score
        unfused = _fixed_order_scores(X[i], C, fma=lambda a, b, c: np.float32(np.float32(a * b) + c))
        n_unfused += unfused.min().view(np.uint32) != best[i].view(np.uint32)
        rev = _fixed_order_scores(X[i], C, order=list(range(31, -1, -1)))
        n_reversed += rev.min().view(np.uint32) != best[i].view(np.uint32)
    assert n_unfused > 0 and n_reversed > 0


def test_cluster_means_and_empty_cluster():
    X = np.array([[0, 0], [2, 2], [10, 10], [12, 14]], np.float32)
    labels = np.array([0, 0, 2, 2], np.int32)
    prev = np.full((4, 2), 7.0, np.float32)
    m, cnt = orc.cluster_means(X, labels, 4, prev)
    assert np.array_equal(cnt, [2, 0, 2, 0])
    assert np.allclose(m[0], [1, 1]) and np.allclose(m[2], [11, 12])
    assert np.array_equal(m[1], [7, 7]) and np.array_equal(m[3], [7, 7])


def test_lloyd_inertia_never_increases():
    wl = get_workload("tiny")
    Q, K, V = make_qkv(wl)
    X = K[0, 0].numpy()
    init = X[kmeans_init_indices(0, 0, 1, wl.N, wl.Ck)]
    cent = init.copy()
    prev = np.inf
    for _ in range(6):
        lab = orc.kmeans_assign(X, cent)
        j_assign = orc.inertia(X, cent, lab)
        assert j_assign <= prev * (1 + 1e-12)
        cent, _ = orc.cluster_means(X, lab, wl.Ck, cent)
        j_update = orc.inertia(X, cent, lab)
        assert j_update <= j_assign * (1 + 1e-12)
        prev = j_update


def test_distinct_rows_zero_inertia_after_one_iteration():
    rng = np.random.default_rng(3)
    protos = rng.standard_normal((9, 24)).astype(np.float32)
    z = rng.integers(0, 9, 500)
    z[:9] = np.arange(9)
    X = protos[z]
    cent, lab, cnt, _ = orc.kmeans(X, protos[::-1].copy(), 1)
    assert orc.inertia(X, cent, lab) == 0.0
    assert np.array_equal(lab, 8 - z)
    assert cnt.sum() == 500


def test_matches_scipy_kmeans2():
    wl = get_workload("tiny")
    Q, K, V = make_qkv(wl)
    X = Q[0, 0].numpy()
    init = X[kmeans_init_indices(0, 0, 0, wl.N, wl.Cq)]
    iters = 5
    cent, lab, cnt, _ = orc.kmeans(X, init, iters)
    if (cnt == 0).any():
        pytest.skip("empty cluster: scipy handles it differently")
    # scipy: iter rounds of (assign, update) from the given matrix, labels from the last assign
    c_ref, l_ref = kmeans2(X.astype(np.float64), init.astype(np.float64), iter=iters, minit="matrix")
    agree = (l_ref == lab).mean()
    assert agree > 0.999
    assert np.allclose(c_ref, cent, atol=1e-2)
    if agree == 1.0:
        assert np.allclose(c_ref, cent, rtol=0, atol=2e-6 * max(1.0, np.abs(cent).max()))


def test_values_follow_key_labels():
    rng = np.random.default_rng(4)
    K = rng.standard_normal((300, 16)).astype(np.float32)
    V = rng.standard_normal((300, 16)).astype(np.float32)
    init = K[:7].copy()
    kbar, lab, cnt, vbar = orc.kmeans(K, init, 3, X2=V)
    for c in range(7):
        if cnt[c]:
            assert np.allclose(vbar[c], V[lab == c].astype(np.float64).mean(0), atol=1e-6)
            assert np.allclose(kbar[c], K[lab == c].astype(np.float64).mean(0), atol=1e-6)


def test_permute_is_stable_counting_sort():
    rng = np.random.default_rng(5)
    C, n, tail = 11, 1000, 13
    labels = rng.integers(0, C, n).astype(np.int32)
    labels[labels == 4] = 5  # an empty cluster
    perm, off = orc.permute(labels, C, tail)
    # independent construction: append indices cluster by cluster in increasing order
    ref = []
    for c in range(C):
        ref += [i for i in range(n) if labels[i] == c]
    ref += list(range(n, n + tail))
    assert perm.tolist() == ref
    assert sorted(perm.tolist()) == list(range(n + tail))
    assert off[0] == 0 and off[C] == n and off[C + 1] == n + tail
    assert off[5] - off[4] == 0
    for c in range(C):
        assert np.all(labels[perm[off[c]: off[c + 1]]] == c)
    X = rng.standard_normal((n + tail, 3))
    assert np.array_equal(orc.unpermute_rows(X[perm], perm), X)
