#!/usr/bin/env python3
"""Benchmark of the SVG-EAR attention hot path on one MI355X.

A "step" is one pass of the whole hot path (k-means of Q and K, permutation, probe + route,
fused sparse attention with compensation, un-permutation) over one synthetic attention layer
with Q/K/V already resident in HBM. The default workload is the Wan2.2-shaped layer
(H=40, N=75600, d=128, bf16, C_q=100, C_k=500, 10 cold k-means iterations, 25% routed budget).

Prints ONE JSON line with the whole-layer figure (dense-equivalent TFLOP/s = 4 H N^2 d / t),
per-stage times, the roofline of the dominant kernel (fused attention, bf16 MFMA), the rel-L2
error of sampled output rows against the CPU oracle, the dense brackets, and the CPU oracle
timed on a bounded sample on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
HBM_PEAK_GBS = 8000.0
FP32_VECTOR_PEAK_TFLOPS = 157.3  # 256 CUs x 4 SIMDs x 64 lanes x 2 flop x 2.4 GHz
# HBM bytes per launch of the fused attention kernel come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled
# by a 1 GiB copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0). They are kept in a tracked text file together with the
# hash of the kernel sources they were measured on; a figure measured on other sources is not reported.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attention_hbm_traffic.txt")
ATTENTION_SOURCES = ["attention_bf16.hip", "attention.hip", "attention.h", "common.h"]


def attention_source_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in ATTENTION_SOURCES:
        with open(os.path.join(ROOT, "paper_2603_08982_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def vendor_gemm_rate():
    """What the vendor's own bf16 GEMM (torch.matmul, 8192^3, 100 calls back to back) sustains on this
    GPU: context for `roofline.frac`, whose peak is the published one."""
    import torch
    try:
        n = 8192
        a = torch.randn(n, n, device="cuda", dtype=torch.bfloat16)
        b = torch.randn(n, n, device="cuda", dtype=torch.bfloat16)
        for _ in range(5):
            a @ b
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(100):
            a @ b
        e1.record()
        torch.cuda.synchronize()
        return {"torch_matmul_bf16_8192_tflops": 2.0 * n ** 3 * 100 / (e0.elapsed_time(e1) * 1e-3) / 1e12}
    except Exception as ex:  # noqa: BLE001
        return {"torch_matmul_error": str(ex)[:200]}


def measured_attention_traffic(workload: str, rho: float, heads: int):
    """Bytes per launch from the tracked file, or None if no line matches this workload, budget, head
    count and the current kernel sources. Line format: workload rho heads source_hash bytes."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    cur = attention_source_hash()
    for line in open(TRAFFIC_FILE):
        f = line.split("#")[0].split()
        if len(f) == 5 and f[0] == workload and abs(float(f[1]) - rho) < 1e-9 and int(f[2]) == heads and f[3] == cur:
            return float(f[4])
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="wan", help="wan | hunyuan | tiny | mini_video ...")
    ap.add_argument("--heads", type=int, default=0, help="override head count (debug)")
    ap.add_argument("--rho", type=float, default=-1.0, help="override routed budget fraction")
    ap.add_argument("--iters", type=int, default=-1, help="override k-means iterations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense brackets")
    ap.add_argument("--sample-rows", type=int, default=64,
                    help="random output rows per sampled head checked against the oracle (structural rows come on top)")
    ap.add_argument("--mode", default="layer", choices=["layer", "sweep", "trajectory", "attention-steps"],
                    help="layer: one JSON line for the whole hot path (default); sweep: routed-budget sweep with "
                         "per-stage times and the compensation-only / dense brackets; trajectory: warm-started "
                         "k-means over denoising steps; attention-steps: the fused attention kernel on synthetic "
                         "block layouts (equal query clusters of k x 32 rows, equal key clusters), which separates "
                         "its time per 64-key step from its fixed time per query tile and shows how the step time "
                         "depends on the number of active waves")
    ap.add_argument("--one-stream", action="store_true",
                    help="profiling aid: run the Q and the K/V call of a stage one after the other on one stream, so "
                         "that a kernel trace shows each kernel's duration when it has the GPU to itself")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) so that a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run can be scaled against it")
    ap.add_argument("--layers", type=int, default=40, help="trajectory mode: attention layers per step")
    ap.add_argument("--traj-steps", type=int, default=10, help="trajectory mode: denoising steps")
    return ap.parse_args()


def bits_to_mask(bits: np.ndarray, Ck: int) -> np.ndarray:
    bits = bits.astype(np.uint32)
    R, W = bits.shape
    out = np.zeros((R, W * 32), dtype=bool)
    for j in range(32):
        out[:, j::32] = (bits >> np.uint32(j)) & 1
    return out[:, : Ck + 1]


class StageTimer:
    """HIP events on torch's current stream (the stream every library call is enqueued on)."""

    def __init__(self):
        self.marks = []

    def mark(self, name):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        self.marks.append((name, ev))

    def stages_ms(self):
        out = {}
        for (n0, e0), (n1, e1) in zip(self.marks[:-1], self.marks[1:]):
            out[n1] = out.get(n1, 0.0) + e0.elapsed_time(e1)
        return out


ONE_STREAM = False


def run_layer(sv, Q, K, V, cq0, ck0, cq, ck, wl, budget, timer=None):
    """One pass of the whole path (cold k-means start: centroids reset from the seeded init): the
    binding's attention_layer, which runs Q's k-means and permutation index beside those of K/V on
    a second stream and lets the attention kernel read the queries and write the output in token
    order through that index (no permuted copy of Q, no separate un-permutation pass)."""
    cq.copy_(cq0)
    ck.copy_(ck0)
    if timer: timer.mark("start")
    O, r = sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget, wl.n_tail, overlap=not ONE_STREAM,
                              mark=timer.mark if timer else None)
    r["Q"] = Q
    return r


def permuted_queries(sv, r):
    """The layer never materialises the permuted queries (the attention kernel reads Q through the
    permutation); the sweeps and brackets that call the plain entry point gather them here."""
    if "Qp" not in r:
        r["Qp"] = sv.permute_rows(r["perm_q"], [r["Q"]])[0]
    return r["Qp"]


def oracle_rows_rel_l2(orc, wl, r, cq, ck, head, n_rows, rng):
    """Sampled output rows of one head against the oracle's literal evaluation of Eq. (1)+(6) on the
    GPU's own clustering and mask: rows at the edges of clusters and row tiles, of the smallest and
    the largest cluster, with nothing / the most routed, text rows, plus random ones.
    Returns (pooled rel-L2, worst single-row rel-L2, its name)."""
    from workloads import structural_rows
    f = lambda t: t.float().cpu().numpy()
    qoff = r["qoff"][0, head].cpu().numpy()
    koff = r["koff"][0, head].cpu().numpy()
    named = structural_rows(qoff, r["row_ptr"][0, head].cpu().numpy(), wl.Cq, rng, n_random=n_rows)
    names = list(named)
    rows = np.array([named[k] for k in names], np.int64)
    lq_all = np.repeat(np.arange(wl.Cq + 1), np.diff(qoff))
    lk = np.repeat(np.arange(wl.Ck + 1), np.diff(koff))
    mask = bits_to_mask(r["mask_bits"][0, head].cpu().numpy(), wl.Ck)
    kb = np.concatenate([f(ck[0, head]), np.zeros((1, wl.d), np.float32)])
    vb = np.concatenate([f(r["vbar"][0, head]), np.zeros((1, wl.d), np.float32)])
    tok = r["perm_q"][0, head][torch.from_numpy(rows).to(r["O"].device)].long()
    Qs = f(r["Q"][0, head][tok])
    ref = orc.attention_comp(Qs, f(r["Kp"][0, head]), f(r["Vp"][0, head]), lq_all[rows], lk, kb, vb, mask,
                             orc.scale_of(wl.d), row_chunk=32)
    # permuted row p of the output sits at token perm_q[p] (the kernel writes token order)
    got = f(r["O"][0, head][tok])
    per_row = np.linalg.norm(got - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-30)
    worst = int(np.argmax(per_row))
    return float(np.linalg.norm(got - ref) / np.linalg.norm(ref)), float(per_row[worst]), names[worst]


def probe_exponent_excess(orc, wl, r, cq, ck, head):
    """max over (query cluster a, clustered key j) of qbar_a.k_j*scale - m_a on one head, in fp64 from
    the oracle's stabiliser: how far a key's logit rises above every centroid logit of its row. The
    library caps that exponent at 40; below the cap its scores are those of Eq. (7)."""
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    koff = r["koff"][0, head].cpu().numpy()
    scale = orc.scale_of(wl.d)
    qbar, kbar = f(cq[0, head]), f(ck[0, head])
    sizes = np.diff(koff[: wl.Ck + 1])
    m = np.where(sizes[None, :] > 0, (qbar @ kbar.T) * scale, -np.inf).max(axis=1)
    nv = int(koff[wl.Ck])
    Kp = r["Kp"][0, head][:nv]
    worst = -np.inf
    for j0 in range(0, nv, 16384):
        s = (f(Kp[j0: j0 + 16384]) @ qbar.T) * scale
        worst = max(worst, float((s - m[None, :]).max()))
    return worst


def cpu_baseline(orc, wl, Q, K, V, cq0, ck0, budget, n_rows=48):
    """The oracle as it stands on this machine's host cores, on a bounded sample of the workload:
    head 0, ONE k-means iteration of Q and of K (scaled by the iteration count), the probe,
    the router, and the attention definition on `n_rows` query rows (scaled to all rows);
    the head time is scaled by the head count. Extrapolated, labelled as such."""
    f = lambda t: t.float().cpu().numpy()
    q, k, v = f(Q[0, 0]), f(K[0, 0]), f(V[0, 0])
    nv = wl.N - wl.n_tail
    t0 = time.perf_counter()
    qbar, lab_q, qcnt, _ = orc.kmeans(q[:nv], f(cq0[0, 0]), 1)
    kbar, lab_k, kcnt, vbar = orc.kmeans(k[:nv], f(ck0[0, 0]), 1, X2=v[:nv])
    t_km = (time.perf_counter() - t0) * wl.iters
    t0 = time.perf_counter()
    perm_q, qoff = orc.permute(lab_q, wl.Cq, wl.n_tail)
    perm_k, koff = orc.permute(lab_k, wl.Ck, wl.n_tail)
    Qp, Kp, Vp = q[perm_q], k[perm_k], v[perm_k]
    t_perm = time.perf_counter() - t0
    t0 = time.perf_counter()
    E, scores, m = orc.probe_errors(qbar, kbar, vbar, Kp, Vp, koff, orc.scale_of(wl.d))
    mask, rp, ci, cost = orc.route(scores, qcnt, kcnt, budget, n_tail_q=wl.n_tail, n_tail_k=wl.n_tail)
    t_pr = time.perf_counter() - t0
    lq = np.repeat(np.arange(wl.Cq + 1), np.diff(qoff))
    lk = np.repeat(np.arange(wl.Ck + 1), np.diff(koff))
    fm = np.zeros((wl.Cq + 1, wl.Ck + 1), bool)
    fm[: mask.shape[0], : mask.shape[1]] = mask
    kb = np.concatenate([kbar, np.zeros((1, wl.d), np.float32)])
    vb = np.concatenate([vbar, np.zeros((1, wl.d), np.float32)])
    rows = np.linspace(0, wl.N - 1, n_rows).astype(np.int64)
    t0 = time.perf_counter()
    orc.attention_comp(Qp[rows], Kp, Vp, lq[rows], lk, kb, vb, fm, orc.scale_of(wl.d), row_chunk=16)
    t_att = (time.perf_counter() - t0) * (wl.N / n_rows)
    t_head = t_km + t_perm + t_pr + t_att
    t_layer = t_head * wl.H * wl.B
    dense_flops = 4.0 * wl.B * wl.H * float(wl.N) ** 2 * wl.d
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas_threads = 1
    return {
        "value": dense_flops / t_layer / 1e12, "unit": "TFLOP/s", "cores": max(orc.host_threads(), blas_threads),
        "kind": "oracle",
        "sample": (f"head 0 of {wl.H}: 1 of {wl.iters} k-means iterations (Q and K), permute, probe, route in full; "
                   f"attention on {n_rows} of {wl.N} query rows; scaled linearly to the layer (extrapolated)"),
        "s_per_layer_extrapolated": t_layer,
        "stage_s_per_head": {"kmeans": t_km, "permute": t_perm, "probe_route": t_pr, "attention": t_att},
    }


def _time_ms(fn, reps=3):
    best = None
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn()
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1)
        best = t if best is None else min(best, t)
    return best, out


def run_sweep(sv, args, wl, Q, K, V, cq0, ck0):
    """Budget sweep on one clustering: per-stage times, compensation-only and dense brackets."""
    cq, ck = cq0.clone(), ck0.clone()
    scale = float(wl.d) ** -0.5
    tm = StageTimer()
    r = run_layer(sv, Q, K, V, cq0, ck0, cq, ck, wl, 0, tm)  # warm-up
    tm = StageTimer()
    r = run_layer(sv, Q, K, V, cq0, ck0, cq, ck, wl, 0, tm)
    torch.cuda.synchronize()
    base = tm.stages_ms()
    dense_flops = 4.0 * wl.B * wl.H * float(wl.N) ** 2 * wl.d
    from workloads import budget_pairs

    def attend(budget, flags=0):
        pr = sv.probe_route(cq, ck, r["vbar"], r["Kp"], r["Vp"], r["qoff"], r["koff"], budget, scale, flags=flags)
        return sv.sparse_attn_comp(permuted_queries(sv, r), r["Kp"], r["Vp"], ck, r["vbar"], r["qoff"], r["koff"], pr["mask_bits"],
                                   pr["row_ptr"], pr["col_idx"], scale)[0]

    def rel_l2(o, ref):  # per head, then averaged (fp32 on the GPU)
        num = (o.float() - ref.float()).flatten(2).norm(dim=2)
        return float((num / ref.float().flatten(2).norm(dim=2)).mean().item())

    # quality axis on the synthetic data: distance of the layer's output from exact attention
    # (this kernel with every block routed), for the value-aware probe (Eq. (7), default), the
    # plain probe (Eq. (5)) and per-query-cluster budgets (the paper's implementation)
    o_dense = attend(budget_pairs(1.0, wl.N, wl.N))
    rows = []
    for rho in [0.0, 0.05, 0.10, 0.15, 0.25, 0.50, 1.0]:
        budget = budget_pairs(rho, wl.N, wl.N)
        t_pr, pr = _time_ms(lambda: sv.probe_route(cq, ck, r["vbar"], r["Kp"], r["Vp"], r["qoff"], r["koff"], budget,
                                                   scale))
        t_at, at = _time_ms(lambda: sv.sparse_attn_comp(permuted_queries(sv, r), r["Kp"], r["Vp"], ck, r["vbar"], r["qoff"], r["koff"],
                                                        pr["mask_bits"], pr["row_ptr"], pr["col_idx"], scale))
        dens = float(pr["routed_cost"].sum().item()) / (wl.B * wl.H * float(wl.N) ** 2)
        row = {"rho": rho, "achieved_density": dens, "probe_route_ms": t_pr, "attention_ms": t_at,
               "layer_ms": base["kmeans"] + base["permute"] + base["unpermute"] + t_pr + t_at,
               "attention_routed_tflops": 4.0 * wl.d * float(pr["routed_cost"].sum().item()) / (t_at * 1e-3) / 1e12,
               "rel_l2_vs_all_routed": rel_l2(at[0], o_dense)}
        del at
        if 0.0 < rho < 1.0:
            # Algorithm 2's two-stage form (routed pass, compensation pass, merge) on the same mask
            t_2s, _ = _time_ms(lambda: sv.sparse_attn_comp(permuted_queries(sv, r), r["Kp"], r["Vp"], ck, r["vbar"], r["qoff"],
                                                           r["koff"], pr["mask_bits"], pr["row_ptr"], pr["col_idx"],
                                                           scale, two_stage=True))
            row["attention_two_stage_ms"] = t_2s
            row["rel_l2_vs_all_routed_plain_probe"] = rel_l2(attend(budget, sv.PROBE_PLAIN), o_dense)
            row["rel_l2_vs_all_routed_per_row_budget"] = rel_l2(attend(budget, sv.ROUTE_PER_ROW), o_dense)
        rows.append(row)
    # adaptive per-query-cluster budgets (the top-p reading of the paper's implementation), with
    # the one-budget-per-head rule at the same mean cost beside it
    top_p_rows = []
    for p in [0.3, 0.5, 0.7, 0.85]:
        def probe_p():
            return sv.probe_route(cq, ck, r["vbar"], r["Kp"], r["Vp"], r["qoff"], r["koff"], 0, scale, top_p=p)
        t_pr, pr = _time_ms(probe_p)
        t_at, at = _time_ms(lambda: sv.sparse_attn_comp(permuted_queries(sv, r), r["Kp"], r["Vp"], ck, r["vbar"], r["qoff"], r["koff"],
                                                        pr["mask_bits"], pr["row_ptr"], pr["col_idx"], scale))
        mean_cost = int(pr["routed_cost"].double().mean().item())
        top_p_rows.append({"top_p": p, "achieved_density": mean_cost / float(wl.N) ** 2, "probe_route_ms": t_pr,
                           "attention_ms": t_at,
                           "layer_ms": base["kmeans"] + base["permute"] + base["unpermute"] + t_pr + t_at,
                           "rel_l2_vs_all_routed": rel_l2(at[0], o_dense),
                           "rel_l2_vs_all_routed_one_budget_same_cost": rel_l2(attend(mean_cost), o_dense)})
        del at
    del o_dense
    out = {"mode": "sweep", "workload": wl.name, "kmeans_ms": base["kmeans"], "permute_ms": base["permute"],
           "unpermute_ms": base["unpermute"], "sweep": rows, "top_p_sweep": top_p_rows}
    try:
        t_sd, _ = _time_ms(lambda: torch.nn.functional.scaled_dot_product_attention(Q, K, V), reps=2)
        out["torch_sdpa_dense_ms"] = t_sd
        out["torch_sdpa_dense_tflops"] = dense_flops / (t_sd * 1e-3) / 1e12
    except Exception as ex:  # noqa: BLE001
        out["torch_sdpa_error"] = str(ex)[:200]
    print(json.dumps(out))


def run_attention_steps(sv):
    """Kernel-level timing of attn_bf16_d128_kernel on synthetic layouts (bf16, d = 128, 16 heads): every query
    cluster has 32 k rows (k active waves per tile), every key cluster the same size, each query cluster routes
    `routed` random key clusters. (1) k = 12, exactly 12 tiles per CU, the routed count varied: a least-squares fit
    of time per tile against the steps per tile T gives the fixed time per tile and the time per step. (2) a quarter
    of the key clusters routed, k varied: time per tile-step against the active waves."""
    dev = torch.device("cuda:0")
    H, d, Ck = 16, 128, 512
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def run_case(k, Cq, routed):
        N = Cq * 32 * k
        Q, K, V = (torch.randn(1, H, N, d, generator=gen, device=dev).to(torch.bfloat16) for _ in range(3))
        kbar, vbar = torch.randn(1, H, Ck, d, device=dev), torch.randn(1, H, Ck, d, device=dev)
        ks = np.full(Ck, N // Ck)
        ks[: N - ks.sum()] += 1
        koff = np.concatenate([[0], np.cumsum(ks), [N]]).astype(np.int32)
        qoff = np.concatenate([np.arange(Cq + 1) * 32 * k, [N]]).astype(np.int32)
        rng = np.random.default_rng(1000 * k + routed)
        W = (Ck + 1 + 31) // 32
        mask = np.zeros((Cq + 1, W * 32), bool)
        for a in range(Cq):
            mask[a, rng.choice(Ck, routed, replace=False)] = True
        bits = np.zeros((Cq + 1, W), np.uint32)
        for j in range(32):
            bits |= mask[:, j::32].astype(np.uint32) << np.uint32(j)
        rp = np.zeros(Cq + 2, np.int32)
        rp[1:] = np.cumsum(mask[:, : Ck + 1].sum(1))
        ci = np.zeros((Cq + 1) * (Ck + 1), np.int32)
        nz = np.concatenate([np.nonzero(mask[a, : Ck + 1])[0] for a in range(Cq + 1)])
        ci[: len(nz)] = nz
        rep = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(torch.int32).to(dev)[None, None].expand(
            1, H, *x.shape).contiguous()
        meta = [rep(qoff), rep(koff), rep(bits.view(np.int32)), rep(rp), rep(ci)]
        call = lambda: sv.sparse_attn_comp(Q, K, V, kbar, vbar, *meta, d ** -0.5)
        call()
        ms = min(_time_ms(call, reps=1)[0] for _ in range(4))
        steps = float(np.mean([(int(ks[np.nonzero(mask[a, :Ck])[0]].sum()) + 63) // 64 for a in range(Cq)])) + Ck // 64
        tiles = H * Cq * ((32 * k + 383) // 384)
        return {"active_waves": k, "query_clusters": Cq, "routed_key_clusters": routed, "steps_per_tile": steps,
                "tiles_per_cu": tiles / 256.0, "kernel_ms": ms, "us_per_tile": ms * 1e3 / (tiles / 256.0),
                "ns_per_tile_step": ms * 1e6 / (tiles / 256.0 * steps)}

    fit_rows = [run_case(12, 192, r) for r in (0, 16, 32, 64, 128, 256)]
    A = np.array([[1.0, r["steps_per_tile"]] for r in fit_rows])
    y = np.array([r["us_per_tile"] for r in fit_rows])
    (a, b), *_ = np.linalg.lstsq(A, y, rcond=None)
    wave_rows = [run_case(k, 2304 // k, 128) for k in (12, 9, 8, 6, 4, 3, 2, 1)]
    print(json.dumps({"mode": "attention-steps", "kernel": "attn_bf16_d128_kernel", "heads": H, "key_clusters": Ck,
                      "fit_us_per_tile": a, "fit_ns_per_step": b * 1e3, "fit_cases": fit_rows, "wave_cases": wave_rows}))


def run_trajectory(sv, args, wl):
    """Denoising-trajectory stack: `layers` attention layers x `traj_steps` steps; each step's
    Q/K/V = previous + N(0, 0.05^2) drift (re-rounded to bf16); k-means warm-started from the
    previous step's centroids with 2 iterations (step 0: seeded cold start, also 2 iterations);
    routed budget 20 %. Reports the summed all-stage time of the layers per step."""
    from workloads import make_qkv, kmeans_init_indices, budget_pairs
    dev = torch.device("cuda:0")
    wl = wl.with_(rho=0.20 if args.rho < 0 else args.rho, iters=2 if args.iters < 0 else args.iters)
    budget = budget_pairs(wl.rho, wl.N, wl.N)
    nv = wl.N - wl.n_tail
    layers = []
    for ell in range(args.layers):
        w_l = wl.with_(seed=wl.seed + 1000 + ell)
        Q, K, V = make_qkv(w_l, dev)
        cq = torch.empty(wl.B, wl.H, wl.Cq, wl.d, device=dev)
        ck = torch.empty(wl.B, wl.H, wl.Ck, wl.d, device=dev)
        for h in range(wl.H):
            cq[0, h] = Q[0, h][torch.from_numpy(kmeans_init_indices(w_l.seed, h, 0, nv, wl.Cq)).to(dev)].float()
            ck[0, h] = K[0, h][torch.from_numpy(kmeans_init_indices(w_l.seed, h, 1, nv, wl.Ck)).to(dev)].float()
        layers.append([Q, K, V, cq, ck])
    gen = torch.Generator(device=dev)
    gen.manual_seed(12345)
    per_step = []
    for step in range(args.traj_steps):
        if step > 0:
            for Lr in layers:
                for X in Lr[:3]:
                    for h in range(wl.H):  # per head to bound temporaries
                        X[0, h] = (X[0, h].float() + 0.05 * torch.randn(X[0, h].shape, generator=gen, device=dev)).to(X.dtype)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for Q, K, V, cq, ck in layers:
            sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget, wl.n_tail)  # centroids updated in place
        e1.record()
        torch.cuda.synchronize()
        per_step.append(e0.elapsed_time(e1))
    dense_flops = 4.0 * wl.B * wl.H * float(wl.N) ** 2 * wl.d * args.layers
    warm = per_step[1:] if len(per_step) > 1 else per_step
    print(json.dumps({"mode": "trajectory", "workload": wl.name, "layers": args.layers, "steps": args.traj_steps,
                      "kmeans_iters_per_step": wl.iters, "rho": wl.rho, "attention_ms_per_step": per_step,
                      "mean_ms_per_warm_step": sum(warm) / len(warm),
                      "dense_equiv_tflops_warm": dense_flops / (sum(warm) / len(warm) * 1e-3) / 1e12}))


def main():
    global ONE_STREAM
    args = parse()
    ONE_STREAM = args.one_stream
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (heads are independent and would shard over GPUs with no "
              "communication inside the layer, but no multi-GPU path is built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        sys.exit(2)
    import paper_2603_08982_amd as sv
    from workloads import get_workload, make_qkv, kmeans_init_indices, budget_pairs

    sv.load_library()
    dev = torch.device("cuda:0")
    wl = get_workload(args.workload)
    if args.heads > 0: wl = wl.with_(H=args.heads)
    if args.rho >= 0: wl = wl.with_(rho=args.rho)
    if args.iters > 0: wl = wl.with_(iters=args.iters)
    budget = budget_pairs(wl.rho, wl.N, wl.N)

    if args.mode == "trajectory":
        run_trajectory(sv, args, wl)
        return
    if args.mode == "attention-steps":
        run_attention_steps(sv)
        return
    Q, K, V = make_qkv(wl, dev)
    nv = wl.N - wl.n_tail
    cq0 = torch.empty(wl.B, wl.H, wl.Cq, wl.d, device=dev)
    ck0 = torch.empty(wl.B, wl.H, wl.Ck, wl.d, device=dev)
    for b in range(wl.B):
        for h in range(wl.H):
            iq = torch.from_numpy(kmeans_init_indices(wl.seed, b * wl.H + h, 0, nv, wl.Cq)).to(dev)
            ik = torch.from_numpy(kmeans_init_indices(wl.seed, b * wl.H + h, 1, nv, wl.Ck)).to(dev)
            cq0[b, h] = Q[b, h][iq].float()
            ck0[b, h] = K[b, h][ik].float()
    if args.mode == "sweep":
        run_sweep(sv, args, wl, Q, K, V, cq0, ck0)
        return
    cq, ck = cq0.clone(), ck0.clone()

    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        run_layer(sv, Q, K, V, cq0, ck0, cq, ck, wl, budget)
    torch.cuda.synchronize()
    timers = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tm = StageTimer()
        r = run_layer(sv, Q, K, V, cq0, ck0, cq, ck, wl, budget, tm)
        timers.append(tm)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stages = {}
    for tm in timers:
        for k, v in tm.stages_ms().items():
            stages[k] = stages.get(k, 0.0) + v / args.steps

    dense_flops = 4.0 * wl.B * wl.H * float(wl.N) ** 2 * wl.d
    value = dense_flops / (ms_per_step * 1e-3) / 1e12

    # algorithmic flops of the fused attention kernel: routed pairs + one pseudo-key per skipped cluster
    routed_pairs = float(r["routed_cost"].sum().item())
    mask_all = r["mask_bits"].cpu().numpy()
    qoff_all = r["qoff"].cpu().numpy()
    koff_all = r["koff"].cpu().numpy()
    comp_pairs = 0.0
    for b in range(wl.B):
        for h in range(wl.H):
            m = bits_to_mask(mask_all[b, h], wl.Ck)[: wl.Cq, : wl.Ck]
            qs = np.diff(qoff_all[b, h])[: wl.Cq]
            ks = np.diff(koff_all[b, h])[: wl.Ck]
            comp_pairs += float((qs[:, None] * ((~m) & (ks[None, :] > 0))).sum())
    attn_flops = 4.0 * wl.d * (routed_pairs + comp_pairs)
    attn_ms = stages["attention"]
    # bf16: matrix cores; fp32 (one query row per lane on the vector ALUs): the fp32 vector peak
    peak_tflops = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS
    achieved = attn_flops / (attn_ms * 1e-3) / 1e12
    density = routed_pairs / (wl.B * wl.H * float(wl.N) ** 2)

    from oracle import svgear_oracle as orc
    rng = np.random.default_rng(0)
    checks = [oracle_rows_rel_l2(orc, wl, r, cq, ck, h, args.sample_rows, rng) for h in sorted({0, wl.H - 1})]
    rel = max(c[0] for c in checks)
    worst_row = max(checks, key=lambda c: c[1])
    excess = max(probe_exponent_excess(orc, wl, r, cq, ck, h) for h in sorted({0, wl.H - 1}))

    out = {
        "metric": "dense-equivalent TFLOP/s of one attention layer, whole hot path "
                  "(k-means + permute + probe/route + fused sparse attention with compensation + unpermute)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} H={wl.H} N={wl.N} (tail {wl.n_tail}) d={wl.d} Cq={wl.Cq} "
                               f"Ck={wl.Ck} kmeans_iters={wl.iters} (cold start) rho={wl.rho}",
                   "budget_pairs_per_head": budget},
        "stages_ms": stages,
        "achieved_density": density,
        "rel_l2_vs_oracle_sampled_rows": rel,
        "worst_sampled_row": {"rel_l2": worst_row[1], "row": worst_row[2]},
        "probe_max_exponent_above_row_stabiliser": {"value": excess, "cap": 40.0, "cap_reached": bool(excess > 40.0)},
        "attention_stage": {"ms": attn_ms, "dense_equiv_tflops": dense_flops / (attn_ms * 1e-3) / 1e12},
        "roofline": {"bound": "mfma" if wl.dtype == "bf16" else "alu",
                     "kernel": ("attn_bf16_d128_kernel" if wl.d == 128 else "attn_bf16_kernel") if wl.dtype == "bf16"
                     else "attn_f32_kernel",
                     "achieved": achieved, "peak": peak_tflops, "unit": "TFLOP/s",
                     "frac": achieved / peak_tflops,
                     "traffic": measured_attention_traffic(wl.name, wl.rho, wl.H),
                     "kernel_source_hash": attention_source_hash(),
                     "algorithmic_flops_per_launch": attn_flops},
    }

    if not args.no_dense and wl.dtype == "bf16":
        # dense brackets on the same tensors: this library at 100% budget, and torch SDPA
        full = sv.probe_route(cq, ck, r["vbar"], r["Kp"], r["Vp"], r["qoff"], r["koff"], wl.N * wl.N,
                              float(wl.d) ** -0.5, flags=sv.USE_GIVEN_SCORES, scores=r["scores"])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        sv.sparse_attn_comp(permuted_queries(sv, r), r["Kp"], r["Vp"], ck, r["vbar"], r["qoff"], r["koff"], full["mask_bits"],
                            full["row_ptr"], full["col_idx"], float(wl.d) ** -0.5)
        e1.record()
        torch.cuda.synchronize()
        own_ms = e0.elapsed_time(e1)
        sd = {}
        try:
            torch.nn.functional.scaled_dot_product_attention(Q[:, :2], K[:, :2], V[:, :2])
            torch.cuda.synchronize()
            e0.record()
            torch.nn.functional.scaled_dot_product_attention(Q, K, V)
            e1.record()
            torch.cuda.synchronize()
            sd = {"torch_sdpa_ms": e0.elapsed_time(e1),
                  "torch_sdpa_tflops": dense_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12}
        except Exception as ex:  # noqa: BLE001
            sd = {"torch_sdpa_error": str(ex)[:200]}
        out["dense_bracket"] = {"own_kernel_all_routed_ms": own_ms,
                                "own_kernel_all_routed_tflops": dense_flops / (own_ms * 1e-3) / 1e12, **sd,
                                **vendor_gemm_rate()}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(orc, wl, Q, K, V, cq0, ck0, budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
