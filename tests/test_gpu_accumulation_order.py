"""The k-means assignment promises labels of ONE fixed fp32 order (x.c a single fma chain over
t = 0..d-1). The library runs those dot products as chains of fp32 matrix-core instructions
(v_mfma_f32_32x32x2_f32, two k-steps per instruction), relying on the hardware to accumulate each
output element as that sequential chain. This file builds inputs on which OTHER accumulation
orders (the two k-steps of an instruction swapped or summed exactly before rounding, groups of
four, an unfused multiply and add, a fully reversed or an exactly rounded dot product) decide
many labels differently, and checks the library against the fixed-order oracle on them: a
toolchain, firmware or kernel change that alters the order fails here, and the message says which
order the labels now follow.

Construction: every row x is an exact real-arithmetic TIE between two centroids c0, c1 (they differ
in one coordinate t, with x_t their midpoint), so only the roundings of the fp32 evaluation decide
the label; all other centroids are far away.
"""
import numpy as np
import pytest
import torch

import paper_2603_08982_amd as sv
from oracle import svgear_oracle as orc

ORDERS = ("pair swapped", "pair fused", "unfused", "quad fused", "quad reversed", "fully reversed", "exact")


def _f32(x):
    return np.asarray(x, np.float64).astype(np.float32).astype(np.float64)


def _dots_in_other_orders(X, C):
    """x.c for every (row, centroid) in the alternative orders, emulated in fp64 (a product of two
    fp32 numbers is exact there; each '_f32' is one rounding to fp32). [order][n, C] float32."""
    X64, C64 = X.astype(np.float64), C.astype(np.float64)
    n, d = X.shape
    P = X64[:, None, :] * C64[None, :, :]  # exact products [n, C, d]
    out = {}
    acc = np.zeros(P.shape[:2])
    for s in range(d // 2):  # the two k-steps of one instruction in the other order
        acc = _f32(P[:, :, 2 * s] + _f32(P[:, :, 2 * s + 1] + acc))
    out["pair swapped"] = acc
    acc = np.zeros(P.shape[:2])
    for s in range(d // 2):  # both products added exactly, one rounding per instruction
        acc = _f32(acc + P[:, :, 2 * s] + P[:, :, 2 * s + 1])
    out["pair fused"] = acc
    acc = np.zeros(P.shape[:2])
    for t in range(d):  # separate multiply and add: two roundings per term
        acc = _f32(acc + _f32(P[:, :, t]))
    out["unfused"] = acc
    acc = np.zeros(P.shape[:2])
    for s in range(d // 4):
        acc = _f32(acc + P[:, :, 4 * s] + P[:, :, 4 * s + 1] + P[:, :, 4 * s + 2] + P[:, :, 4 * s + 3])
    out["quad fused"] = acc
    acc = np.zeros(P.shape[:2])
    for s in range(d // 4):
        for u in (3, 2, 1, 0):
            acc = _f32(P[:, :, 4 * s + u] + acc)
    out["quad reversed"] = acc
    acc = np.zeros(P.shape[:2])
    for t in range(d - 1, -1, -1):
        acc = _f32(P[:, :, t] + acc)
    out["fully reversed"] = acc
    out["exact"] = _f32(P.sum(axis=2))
    return {k: v.astype(np.float32) for k, v in out.items()}


def _labels_from_dots(dots, C):
    cn = np.zeros(C.shape[0], np.float32)
    for t in range(C.shape[1]):  # |c|^2 in the documented order (this part is not under test)
        cn = _f32(C[:, t].astype(np.float64) ** 2 + cn).astype(np.float32)
    score = _f32(-2.0 * dots.astype(np.float64) + cn.astype(np.float64)[None, :])
    return score.argmin(axis=1).astype(np.int32)  # argmin takes the lowest index on ties


def tie_case(d, n_pairs=24, rows_per_pair=40, seed=0, bf16_rows=False):
    """(X [n,d] f32, C [2*n_pairs, d] f32): every row ties exactly, in real arithmetic, between
    the two centroids of its pair."""
    rng = np.random.default_rng(seed)
    base = (3.0 * rng.standard_normal((n_pairs, d))).astype(np.float32)
    X, C = [], np.repeat(base, 2, axis=0).copy()
    t_of = rng.integers(0, d, n_pairs)
    for p in range(n_pairs):
        t = int(t_of[p])
        # c0_t a multiple of 2^-10 and c1 = c0 + 2^-6 e_t: c1_t and the midpoint c0_t + 2^-7 are exact
        C[2 * p, t] = np.float32(np.round(np.float64(C[2 * p, t]) * 1024.0) / 1024.0)
        delta = np.float32(2.0 ** -6)
        C[2 * p + 1, t] = np.float32(C[2 * p, t] + delta)
        mid = np.float64(C[2 * p, t]) + np.float64(C[2 * p + 1, t])
        assert np.float64(np.float32(mid / 2)) == mid / 2
        x = base[p][None, :] + (0.25 * rng.standard_normal((rows_per_pair, d))).astype(np.float32)
        if bf16_rows:
            x = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
            # the midpoint must be a bf16 number too: put both centroid coordinates around a bf16 value
            xt = torch.tensor(float(base[p, t])).to(torch.bfloat16).float().item()
            # ... at a distance with many significant bits (an odd multiple of xt's last fp32 place), so
            # that the two dot products do not differ by a multiple of the accumulators' spacing
            eta = float(2 * rng.integers(1 << 13, 1 << 14) + 1) * float(np.spacing(np.float32(abs(xt))))
            C[2 * p, t] = np.float32(xt - eta)
            C[2 * p + 1, t] = np.float32(xt + eta)
            assert np.float64(C[2 * p, t]) + np.float64(C[2 * p + 1, t]) == 2.0 * xt
            x[:, t] = xt
        else:
            x[:, t] = np.float32(mid / 2)
        X.append(x.astype(np.float32))
    X = np.concatenate(X)
    # exact tie in real arithmetic: |c0|^2 - 2 x.c0 == |c1|^2 - 2 x.c1 (integer-exact check via fractions)
    from fractions import Fraction
    for i in (0, len(X) - 1):
        p = i // rows_per_pair
        s = [sum(Fraction(float(c)) ** 2 - 2 * Fraction(float(a)) * Fraction(float(c)) for a, c in zip(X[i], C[2 * p + k]))
             for k in (0, 1)]
        assert s[0] == s[1]
    return X, C


@pytest.mark.parametrize("d", [64, 128])
def test_tie_cases_separate_the_fixed_order_from_other_orders(d):
    """CPU: on the constructed ties, every alternative order disagrees with the fixed order on many rows."""
    X, C = tie_case(d)
    ref = orc.kmeans_assign(X, C)
    assert np.all(ref // 2 == np.arange(len(X)) // 40)  # the far centroids never win
    assert 0.2 < (ref % 2).mean() < 0.8  # rounding noise sends rows both ways
    for name, dots in _dots_in_other_orders(X, C).items():
        differ = int((_labels_from_dots(dots, C) != ref).sum())
        assert differ >= 20, (name, differ)


@pytest.mark.gpu
@pytest.mark.parametrize("d,dtype", [(64, torch.float32), (128, torch.float32), (128, torch.bfloat16), (64, torch.bfloat16)])
def test_kmeans_labels_follow_the_sequential_fma_chain_on_exact_ties(d, dtype):
    X, C = tie_case(d, seed=1 + d, bf16_rows=dtype == torch.bfloat16)
    ref = orc.kmeans_assign(X, C)
    others = {k: _labels_from_dots(v, C) for k, v in _dots_in_other_orders(X, C).items()}
    for name in ORDERS:
        assert int((others[name] != ref).sum()) >= 10, name  # the case can tell that order apart
    x = torch.from_numpy(X).to(dtype)[None, None].cuda().contiguous()
    assert torch.equal(x.float().cpu()[0, 0], torch.from_numpy(X))  # the rows are exact in this dtype
    cent = torch.from_numpy(C)[None, None].cuda().contiguous()
    print(f"tie case d={d} {dtype} rows={len(X)} centroids={len(C)}", flush=True)
    labels, counts, _ = sv.kmeans(x, cent, 1)
    torch.cuda.synchronize()
    got = labels[0, 0].cpu().numpy()
    if not np.array_equal(got, ref):
        match = {k: int((got == v).sum()) for k, v in others.items()}
        best = max(match, key=match.get)
        raise AssertionError(
            f"{int((got != ref).sum())} of {len(ref)} labels differ from the fixed-order fma chain; they agree best "
            f"with the '{best}' order ({match[best]} rows): the fp32 matrix-core chain no longer accumulates as the "
            f"sequential chain the k-means kernels assume (all orders: {match})")
    assert np.array_equal(counts[0, 0].cpu().numpy(), np.bincount(ref, minlength=len(C)))
