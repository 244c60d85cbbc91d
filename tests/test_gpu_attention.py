"""GPU parity: svgear_sparse_attn_comp (fp32 and bf16 MFMA kernels) and the chained path."""
import numpy as np
import pytest
import torch

import paper_2603_08982_amd as sv
from oracle import svgear_oracle as orc
from workloads import get_workload, make_qkv, budget_pairs
from helpers import (dev, to_np, oracle_head, mask_to_bits, csr_from_mask, full_mask, rel_l2, init_centroids,
                     check_top_p_row_budgets)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 1e-2}  # relative L2 error of the attention output


def _run_stage(wl, Q, K, V, refs, masks, two_stage=False):
    """Feeds the oracle's clustering and the given masks to the GPU attention stage."""
    B, H = Q.shape[:2]
    Cq, Ck = wl.Cq, wl.Ck

    def stack(fn, dtype):
        return torch.stack([torch.stack([torch.from_numpy(np.ascontiguousarray(fn(b, h))) for h in range(H)])
                            for b in range(B)]).to(dtype).to(dev())

    kbar = stack(lambda b, h: refs[b][h]["kbar"], torch.float32)
    vbar = stack(lambda b, h: refs[b][h]["vbar"], torch.float32)
    qoff = stack(lambda b, h: refs[b][h]["qoff"], torch.int32)
    koff = stack(lambda b, h: refs[b][h]["koff"], torch.int32)
    bits = stack(lambda b, h: mask_to_bits(masks[b][h], Cq, Ck).view(np.int32), torch.int32)
    csr = [[csr_from_mask(full_mask(masks[b][h], Cq, Ck)) for h in range(H)] for b in range(B)]
    row_ptr = stack(lambda b, h: csr[b][h][0], torch.int32)
    col_idx = stack(lambda b, h: csr[b][h][1], torch.int32)
    gather = lambda X, key: torch.stack([torch.stack([X[b, h][torch.from_numpy(refs[b][h][key]).long()]
                                                      for h in range(H)]) for b in range(B)]).to(dev())
    Qp, Kp, Vp = gather(Q, "perm_q"), gather(K, "perm_k"), gather(V, "perm_k")
    op, lse = sv.sparse_attn_comp(Qp, Kp, Vp, kbar, vbar, qoff, koff, bits, row_ptr, col_idx, orc.scale_of(wl.d),
                                  want_lse=True, two_stage=two_stage)
    torch.cuda.synchronize()
    return Qp, Kp, Vp, op, lse


def _oracle_stage(wl, ref, Qp, Kp, Vp, mask):
    Cq, Ck, d = wl.Cq, wl.Ck, wl.d
    lq = np.repeat(np.arange(Cq + 1), np.diff(ref["qoff"]))
    lk = np.repeat(np.arange(Ck + 1), np.diff(ref["koff"]))
    kb = np.concatenate([ref["kbar"], np.zeros((1, d), np.float32)])
    vb = np.concatenate([ref["vbar"], np.zeros((1, d), np.float32)])
    return orc.attention_comp(Qp, Kp, Vp, lq, lk, kb, vb, full_mask(mask, Cq, Ck), orc.scale_of(d))


@pytest.mark.parametrize("name", ["tiny", "mini_video", "mini_video_tail", "mini_d64", "mini_manyq", "mini_manyk", "mini_f32_d128"])
@pytest.mark.parametrize("mode", ["routed", "all", "none", "random"])
def test_attention_stage_matches_oracle(name, mode):
    wl = get_workload(name)
    Q, K, V = make_qkv(wl, "cpu")
    B, H = Q.shape[:2]
    refs = [[oracle_head(Q, K, V, b, h, wl, iters=3) for h in range(H)] for b in range(B)]
    rng = np.random.default_rng(5)
    masks = [[None] * H for _ in range(B)]
    for b in range(B):
        for h in range(H):
            base = full_mask(refs[b][h]["mask"], wl.Cq, wl.Ck)
            forced = np.zeros_like(base)
            forced[wl.Cq, :] = True
            forced[:, wl.Ck] = True
            nonempty = np.outer(np.diff(refs[b][h]["qoff"]) > 0, np.diff(refs[b][h]["koff"]) > 0)
            if mode == "all":
                m = np.ones_like(base)
            elif mode == "none":
                m = forced.copy()
            elif mode == "random":
                m = (rng.random(base.shape) < 0.3) | forced
            else:
                m = base
            masks[b][h] = m & nonempty
    Qp, Kp, Vp, op, lse = _run_stage(wl, Q, K, V, refs, masks)
    for b in range(B):
        for h in range(H):
            o_ref = _oracle_stage(wl, refs[b][h], to_np(Qp[b, h]), to_np(Kp[b, h]), to_np(Vp[b, h]), masks[b][h])
            err = rel_l2(to_np(op[b, h]), o_ref)
            assert err <= TOL[wl.dtype], f"{name}/{mode} head {b},{h}: rel-L2 {err}"
            if mode == "all":
                dense = orc.dense_attention(to_np(Qp[b, h]), to_np(Kp[b, h]), to_np(Vp[b, h]), orc.scale_of(wl.d))
                assert rel_l2(to_np(op[b, h]), dense) <= TOL[wl.dtype]
                L = (to_np(Qp[b, h]).astype(np.float64) @ to_np(Kp[b, h]).astype(np.float64).T) * orc.scale_of(wl.d)
                lse_ref = np.log(np.exp(L - L.max(1, keepdims=True)).sum(1)) + L.max(1)
                assert np.allclose(to_np(lse[b, h]), lse_ref, atol=2e-2 if wl.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("name", ["mini_video", "mini_video_tail", "mini_manyq", "mini_manyk"])
@pytest.mark.parametrize("mode", ["routed", "none", "all"])
def test_two_stage_form_matches_oracle_and_fused_kernel(name, mode):
    """Algorithm 2's form on the GPU (routed pass, compensation pass, merge; bf16, d = 128)
    against the oracle's literal evaluation and against the fused kernel, output and LSE."""
    wl = get_workload(name)
    Q, K, V = make_qkv(wl, "cpu")
    B, H = Q.shape[:2]
    refs = [[oracle_head(Q, K, V, b, h, wl, iters=3) for h in range(H)] for b in range(B)]
    masks = [[None] * H for _ in range(B)]
    for b in range(B):
        for h in range(H):
            base = full_mask(refs[b][h]["mask"], wl.Cq, wl.Ck)
            forced = np.zeros_like(base)
            forced[wl.Cq, :] = True
            forced[:, wl.Ck] = True
            nonempty = np.outer(np.diff(refs[b][h]["qoff"]) > 0, np.diff(refs[b][h]["koff"]) > 0)
            m = np.ones_like(base) if mode == "all" else (forced.copy() if mode == "none" else base)
            masks[b][h] = m & nonempty
    Qp, Kp, Vp, op2, lse2 = _run_stage(wl, Q, K, V, refs, masks, two_stage=True)
    _, _, _, op1, lse1 = _run_stage(wl, Q, K, V, refs, masks)
    for b in range(B):
        for h in range(H):
            o_ref = _oracle_stage(wl, refs[b][h], to_np(Qp[b, h]), to_np(Kp[b, h]), to_np(Vp[b, h]), masks[b][h])
            assert rel_l2(to_np(op2[b, h]), o_ref) <= TOL[wl.dtype], f"{name}/{mode} head {b},{h}"
            assert rel_l2(to_np(op2[b, h]), to_np(op1[b, h])) <= TOL[wl.dtype]
            l1, l2 = to_np(lse1[b, h]), to_np(lse2[b, h])
            fin = np.isfinite(l1)
            assert np.array_equal(fin, np.isfinite(l2)) and np.allclose(l1[fin], l2[fin], atol=2e-2)


def test_identical_keys_per_cluster_compensation_exact_on_gpu():
    # keys identical inside every cluster: compensated output equals dense for any mask
    wl = get_workload("mini_video")
    Q, K, V = make_qkv(wl, "cpu")
    B, H = Q.shape[:2]
    refs = [[oracle_head(Q, K, V, b, h, wl, iters=2) for h in range(H)] for b in range(B)]
    K2 = K.clone()
    for b in range(B):
        for h in range(H):
            kb16 = torch.from_numpy(refs[b][h]["kbar"]).to(torch.bfloat16)
            K2[b, h] = kb16[torch.from_numpy(refs[b][h]["lab_k"]).long()]
            refs[b][h]["kbar"] = kb16.float().numpy()
    masks = [[np.zeros((wl.Cq, wl.Ck), bool) for _ in range(H)] for _ in range(B)]
    Qp, Kp, Vp, op, _ = _run_stage(wl, Q, K2, V, refs, masks)
    for b in range(B):
        for h in range(H):
            dense = orc.dense_attention(to_np(Qp[b, h]), to_np(Kp[b, h]), to_np(Vp[b, h]), orc.scale_of(wl.d))
            assert rel_l2(to_np(op[b, h]), dense) <= TOL["bf16"]


@pytest.mark.parametrize("name", ["tiny", "mini_video", "mini_video_tail", "mini_d64", "mini_manyq", "mini_manyk", "mini_f32_d128"])
def test_end_to_end_chain_matches_oracle(name):
    wl = get_workload(name)
    Q, K, V = make_qkv(wl, dev())
    B, H = Q.shape[:2]
    nv = wl.N - wl.n_tail
    cq = init_centroids(Q, wl.Cq, wl.seed, 0, wl.n_tail)
    ck = init_centroids(K, wl.Ck, wl.seed, 1, wl.n_tail)
    budget = budget_pairs(wl.rho, wl.N, wl.N)
    O, r = sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget, wl.n_tail)
    torch.cuda.synchronize()
    assert int(r["routed_cost"].max()) <= budget
    for b in range(B):
        for h in range(H):
            ref = oracle_head(Q, K, V, b, h, wl)
            same_clusters = np.array_equal(to_np(r["lab_q"][b, h]), ref["lab_q"]) and \
                np.array_equal(to_np(r["lab_k"][b, h]), ref["lab_k"])
            if same_clusters:
                assert np.array_equal(to_np(r["perm_q"][b, h]), ref["perm_q"])
                assert np.array_equal(to_np(r["perm_k"][b, h]), ref["perm_k"])
            # free-running comparison: the two paths may part on fp32 near-ties in k-means or
            # on near-equal probe scores, so the output is compared against the oracle's
            # output AND against the oracle evaluated on the GPU's own clustering/mask
            lq = np.repeat(np.arange(wl.Cq + 1), np.diff(to_np(r["qoff"][b, h])))
            lk = np.repeat(np.arange(wl.Ck + 1), np.diff(to_np(r["koff"][b, h])))
            from helpers import bits_to_mask
            m = bits_to_mask(to_np(r["mask_bits"][b, h]), wl.Ck)
            kb = np.concatenate([to_np(r["kbar"][b, h]), np.zeros((1, wl.d), np.float32)])
            vb = np.concatenate([to_np(r["vbar"][b, h]), np.zeros((1, wl.d), np.float32)])
            op_ref = orc.attention_comp(to_np(Q[b, h])[to_np(r["perm_q"][b, h])], to_np(r["Kp"][b, h]), to_np(r["Vp"][b, h]), lq, lk, kb,
                                        vb, m, orc.scale_of(wl.d))
            o_ref = orc.unpermute_rows(op_ref, to_np(r["perm_q"][b, h]))
            assert rel_l2(to_np(O[b, h]), o_ref) <= TOL[wl.dtype]
            if same_clusters and np.array_equal(m, full_mask(ref["mask"], wl.Cq, wl.Ck)):
                assert rel_l2(to_np(O[b, h]), ref["O"]) <= TOL[wl.dtype]


def test_attention_is_deterministic():
    wl = get_workload("mini_video")
    Q, K, V = make_qkv(wl, dev())
    outs = []
    for _ in range(2):
        cq = init_centroids(Q, wl.Cq, wl.seed, 0)
        ck = init_centroids(K, wl.Ck, wl.seed, 1)
        O, r = sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget_pairs(wl.rho, wl.N, wl.N))
        torch.cuda.synchronize()
        outs.append((O.clone(), r["lab_k"].clone(), r["mask_bits"].clone(), ck.clone()))
    for x, y in zip(*outs):
        assert torch.equal(x, y)


@pytest.mark.parametrize("name", ["mini_video", "mini_video_tail", "mini_manyk"])
def test_end_to_end_chain_with_adaptive_row_budgets_matches_oracle(name):
    """The whole path with the per-query-cluster adaptive budgets (the top-p reading) in place of
    one budget per head: budgets valid against the oracle's, mask an exact function of the GPU's
    scores and budgets, output within tolerance of Eq. (1) + Eq. (6) on that mask."""
    wl = get_workload(name)
    p = 0.85
    Q, K, V = make_qkv(wl, dev())
    B, H = Q.shape[:2]
    cq = init_centroids(Q, wl.Cq, wl.seed, 0, wl.n_tail)
    ck = init_centroids(K, wl.Ck, wl.seed, 1, wl.n_tail)
    O, r = sv.attention_layer(Q, K, V, cq, ck, wl.iters, 0, wl.n_tail, top_p=p)
    torch.cuda.synchronize()
    scale = orc.scale_of(wl.d)
    from helpers import bits_to_mask
    for b in range(B):
        for h in range(H):
            qcnt, kcnt = to_np(r["qcnt"][b, h]), to_np(r["kcnt"][b, h])
            got = to_np(r["row_budget"][b, h])
            check_top_p_row_budgets(got, to_np(r["qbar"][b, h]), to_np(r["kbar"][b, h]), qcnt, kcnt, p, scale)
            m_ref = orc.route(to_np(r["scores"][b, h]), qcnt, kcnt, 0, n_tail_q=wl.n_tail, n_tail_k=wl.n_tail,
                              row_budgets=got)[0]
            m = bits_to_mask(to_np(r["mask_bits"][b, h]), wl.Ck)
            assert np.array_equal(m, full_mask(m_ref, wl.Cq, wl.Ck))
            lq = np.repeat(np.arange(wl.Cq + 1), np.diff(to_np(r["qoff"][b, h])))
            lk = np.repeat(np.arange(wl.Ck + 1), np.diff(to_np(r["koff"][b, h])))
            kb = np.concatenate([to_np(r["kbar"][b, h]), np.zeros((1, wl.d), np.float32)])
            vb = np.concatenate([to_np(r["vbar"][b, h]), np.zeros((1, wl.d), np.float32)])
            op_ref = orc.attention_comp(to_np(Q[b, h])[to_np(r["perm_q"][b, h])], to_np(r["Kp"][b, h]), to_np(r["Vp"][b, h]), lq, lk, kb,
                                        vb, m, scale)
            assert rel_l2(to_np(O[b, h]), orc.unpermute_rows(op_ref, to_np(r["perm_q"][b, h]))) <= TOL[wl.dtype]


@pytest.mark.parametrize("name", ["tiny", "mini_video", "mini_video_tail", "mini_d64", "mini_manyq", "mini_f32_d128"])
def test_token_order_entry_equals_permuted_entry_plus_unpermute(name):
    """svgear_sparse_attn_comp_token_order reads the queries and writes the rows
    svgear_sparse_attn_comp computes (parity with the oracle is tested above) through the
    queries' permutation: bitwise equal to gathering Q, that call and svgear_unpermute, also from
    and into strided [B, N, H, d] buffers, lse in token order; and the whole layer gives the
    same output either way."""
    wl = get_workload(name)
    Q, K, V = make_qkv(wl, dev())
    B, H, N, d = Q.shape
    cq = init_centroids(Q, wl.Cq, wl.seed, 0, wl.n_tail)
    ck = init_centroids(K, wl.Ck, wl.seed, 1, wl.n_tail)
    budget = budget_pairs(wl.rho, wl.N, wl.N)
    O_sep, r = sv.attention_layer(Q, K, V, cq.clone(), ck.clone(), wl.iters, budget, wl.n_tail, token_order=False)
    O_tok, r2 = sv.attention_layer(Q, K, V, cq.clone(), ck.clone(), wl.iters, budget, wl.n_tail)
    torch.cuda.synchronize()
    assert "Op" in r and "Qp" in r and "Op" not in r2 and "Qp" not in r2
    assert torch.equal(O_sep, O_tok)
    assert torch.equal(O_sep, sv.unpermute(r["Op"], r["perm_q"]))
    rest = (r["Kp"], r["Vp"], r["kbar"], r["vbar"], r["qoff"], r["koff"], r["mask_bits"], r["row_ptr"], r["col_idx"],
            orc.scale_of(wl.d))
    op, lse_p = sv.sparse_attn_comp(r["Qp"], *rest, want_lse=True)
    Q_strided = Q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    buf = torch.zeros(B, N, H, d, dtype=Q.dtype, device=dev())
    o, lse_t = sv.sparse_attn_comp(Q_strided, *rest, want_lse=True, q_perm=r["perm_q"], out=buf.permute(0, 2, 1, 3))
    torch.cuda.synchronize()
    assert torch.equal(buf.permute(0, 2, 1, 3), O_sep)
    idx = r["perm_q"].long()
    assert torch.equal(torch.gather(lse_t, 2, idx), lse_p)
    with pytest.raises(RuntimeError):  # rows of the output must be 16-byte aligned
        bad = torch.zeros(B, H, N, d + 1, dtype=Q.dtype, device=dev())[..., :d]
        sv.sparse_attn_comp(Q, *rest, q_perm=r["perm_q"], out=bad)
