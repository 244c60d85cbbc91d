/*
 * svgear.h -- C ABI of the MI355X (gfx950) implementation of the SVG-EAR attention hot path.
 *
 * The path, per attention head (batch and head are independent; paper, Appendix "Kernel
 * Implementation Details"):
 *
 *   svgear_kmeans            semantic k-means of the queries and of the keys; the values
 *                            are averaged under the keys' labels
 *   svgear_permute           tokens of a cluster laid out contiguously
 *   svgear_probe_route       error probe (value-aware, Eq. (7); plain, Eq. (5)) and greedy
 *                            error-to-cost routing under a budget
 *   svgear_sparse_attn_comp  block-sparse exact attention over the routed blocks fused with
 *                            centroid compensation of every skipped block (Eq. (1), Eq. (6))
 *   svgear_unpermute         rows of the output put back in token order
 *
 * Conventions that hold for every call
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps device memory, and never synchronises the host.
 *   - `stream` is a hipStream_t passed as void*; all work is enqueued on it, in order.
 *   - `ws` is caller-provided device scratch of `ws_bytes` bytes, 256-byte aligned; its
 *     required size comes from the matching svgear_*_workspace() host function. Calls that
 *     overlap in time need distinct workspaces.
 *   - B*H heads are processed; "BH" below means B*H, heads stored b-major.
 *   - Token tensors are [B, H, N, d] with d contiguous; unpermuted inputs/outputs take
 *     element strides {stride_b, stride_h, stride_n}; permuted tensors are dense.
 *   - d is 64 or 128. dtype is fp32 or bf16 (raw 16-bit pattern, upper half of an fp32).
 *   - The last n_tail tokens of a head (text tokens) are not clustered: they form
 *     pseudo-cluster C (after clusters 0..C-1), keep their order, and their blocks are always
 *     routed exactly. n_tail may be 0; the tail slot still exists and is then empty.
 *   - offsets arrays have C + 2 int32 entries per head: cluster c is rows
 *     [offsets[c], offsets[c+1]) of the permuted tensor, the tail is [offsets[C], offsets[C+1]).
 *   - Return value: SVGEAR_OK or a negative svgear_status. On error nothing useful has been
 *     written. No exceptions, no errno, no global state except the last HIP error code.
 */
#ifndef SVGEAR_H
#define SVGEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The last enumerator only widens the enum's value range to that of int, so that a caller's
 * out-of-range value reaches the argument checks as a defined value (and is rejected there). */
typedef enum { SVGEAR_F32 = 0, SVGEAR_BF16 = 1, SVGEAR_DTYPE_INT_RANGE = 0x7fffffff } svgear_dtype;

typedef enum {
  SVGEAR_OK = 0,
  SVGEAR_ERR_INVALID = -1,     /* null pointer, non-positive size, C > N, bad d/dtype/flags */
  SVGEAR_ERR_WORKSPACE = -2,   /* ws_bytes smaller than svgear_*_workspace() */
  SVGEAR_ERR_HIP = -3,         /* a HIP runtime call failed: see svgear_last_hip_error() */
  SVGEAR_ERR_UNSUPPORTED = -4  /* valid request this build has no kernel for */
} svgear_status;

/* svgear_probe_route flags */
#define SVGEAR_PROBE_VALUE_AWARE 0u   /* Eq. (7), default */
#define SVGEAR_PROBE_PLAIN 1u         /* Eq. (5): value vectors ignored */
#define SVGEAR_ROUTE_GLOBAL 0u        /* one budget per head ("Error-Aware Routing") */
#define SVGEAR_ROUTE_PER_ROW 2u       /* one budget per query cluster (Experiments, "Implementation") */
#define SVGEAR_USE_GIVEN_SCORES 4u    /* skip the probe; route from scores[] as supplied */

/* Library/ABI version (host only). */
int svgear_version(void);

/* Code of the last HIP error seen by this thread's calls (0 if none). Host only. */
int svgear_last_hip_error(void);

/* ---------------------------------------------------------------------------------------
 * k-means (Methodology, "Problem Formulation": Q and K are clustered, the centroid of a
 * cluster is the mean of its tokens; "Linear Compensation": V follows K's assignment).
 *
 * Runs `iters` >= 1 Lloyd iterations -- assign every row to the nearest centroid, then
 * recompute every centroid as the mean of its rows -- starting from centroids[] (in: the
 * initial or previous step's centroids; out: the exact means of the final labels).
 * Assignment is squared Euclidean in fp32 in one fixed order: score(c) = fma(-2, x.c, |c|^2)
 * with x.c and |c|^2 each a single fma chain over t = 0..d-1; the lowest index wins ties.
 * A cluster left without rows keeps its previous centroid and gets count 0.
 * If x2 != NULL, centroids2 receives the means of x2 under the final labels (rows of empty
 * clusters untouched).
 *
 *   x, x2        [B,H,N,d] dtype `dt`, strides xstride (shared by x and x2); read only
 *   centroids    [BH,C,d] fp32 in/out;  centroids2 [BH,C,d] fp32 out (may be NULL iff x2 is)
 *   labels       [BH,N-n_tail] int32 out;  counts [BH,C] int32 out
 * Requires 1 <= C <= N - n_tail.
 */
size_t svgear_kmeans_workspace(int B, int H, int64_t N, int d, int C);
int svgear_kmeans(const void* x, const void* x2, svgear_dtype dt, int B, int H, int64_t N,
                  int64_t n_tail, int d, const int64_t xstride[3], int C, int iters,
                  float* centroids, float* centroids2, int32_t* labels, int32_t* counts,
                  void* ws, size_t ws_bytes, void* stream);

/* Tuning (host only; results never depend on it). From the second iteration on, a bf16 call
 * re-assigns only the rows whose distance bounds do not prove that their label stays. With
 * C >= the value set here each such row is tested against the centroids near its cluster only
 * (candidate lists from centroid-to-centroid distances); with fewer centroids against all of
 * them. min_centroids >= 1 sets the threshold for later calls of this process (INT_MAX: never
 * use lists); min_centroids <= 0 only queries. Returns the previous value (default 400). */
int svgear_kmeans_list_threshold(int min_centroids);

/* ---------------------------------------------------------------------------------------
 * permute (Motivation, "Structured Redundancy": tokens within each cluster are laid out
 * contiguously so the attention map becomes a grid of blocks).
 *
 * perm = stable sort of token indices by label (equal labels keep ascending token order; tail
 * tokens come last in their own order): perm[p] is the token at permuted position p.
 * Then gathers n_tensors (0..4) tensors: dst[k][bh][p][:] = src[k][bh][perm[p]][:].
 *
 *   labels  [BH,N-n_tail] int32 in, values in [0,C);  perm [BH,N] int32 out
 *   offsets [BH,C+2] int32 out
 *   src[k]  [B,H,N,d] dtype dt with strides sstride[k];  dst[k] [BH,N,d] dense
 *   src/dst/sstride are HOST arrays of n_tensors entries (of device pointers / strides).
 */
size_t svgear_permute_workspace(int B, int H, int64_t N, int C);
int svgear_permute(const int32_t* labels, int B, int H, int64_t N, int64_t n_tail, int C,
                   int32_t* perm, int32_t* offsets, int n_tensors, const void* const* src,
                   const int64_t (*sstride)[3], void* const* dst, svgear_dtype dt, int d,
                   void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * svgear_permute for callers that cannot allocate device memory and so have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc. The sort's scratch (per-chunk label histograms) is a fixed array inside the
 * library's device image (svgear_permute_static_capacity() bytes, 8 MiB, held on every GPU
 * the library runs on until the process ends) instead of `ws`; the call allocates and frees
 * nothing. Arguments and results are exactly those of svgear_permute.
 *   - SVGEAR_ERR_WORKSPACE if svgear_permute_workspace(B, H, N, C) exceeds the capacity
 *     (e.g. B*H*ceil(N/2048)*(C+1) counters of 4 bytes: 40 heads x 75,600 tokens x C <= 1416).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (different streams or threads) race. Calls on one stream are ordered and safe; nothing
 *     has to be cleared between them (every counter is written before it is read).
 */
size_t svgear_permute_static_capacity(void);
int svgear_permute_static(const int32_t* labels, int B, int H, int64_t N, int64_t n_tail, int C,
                          int32_t* perm, int32_t* offsets, int n_tensors, const void* const* src,
                          const int64_t (*sstride)[3], void* const* dst, svgear_dtype dt, int d,
                          void* stream);

/* ---------------------------------------------------------------------------------------
 * The row movement of svgear_permute alone: dst[k][bh][p][:] = src[k][b,h,perm[p],:] for a
 * permutation already computed (svgear_permute with n_tensors = 0 returns perm and offsets
 * only). For callers that overlap the two halves with other work: the probe needs the
 * queries' offsets but not the permuted queries, so their rows can move on a second stream
 * while the probe runs. 1 <= n_tensors <= 4; arguments as in svgear_permute. No workspace.
 */
int svgear_permute_rows(const int32_t* perm, int B, int H, int64_t N, int n_tensors,
                        const void* const* src, const int64_t (*sstride)[3], void* const* dst,
                        svgear_dtype dt, int d, void* stream);

/* ---------------------------------------------------------------------------------------
 * probe + route ("Error-Aware Routing"; Eq. (5), Eq. (7); Algorithm 1).
 *
 * Probe: for query cluster a and non-empty key cluster b,
 *   E[a,b] = sum_{j in b} || e^{Sbar_ab - m_a} vbar_b - e^{qbar_a.k_j*scale - m_a} v_j ||^2,
 *   Sbar_ab = qbar_a.kbar_b*scale,  m_a = max over non-empty b of Sbar_ab
 * (PLAIN: the same with the value vectors dropped), and scores[a,b] = E[a,b]/|k_b| -- the
 * block's error-to-cost ratio, |q_a| cancelling. Empty key clusters score 0.
 * The exponents Sbar_ab - m_a (<= 0 by construction) and qbar_a.k_j*scale - m_a are capped at 40
 * before the exponential so that the squares stay inside fp32: a key whose logit exceeds EVERY
 * centroid logit of its row by more than 40 (e^40 ~ 2e17 times the weight of the row's best
 * centroid) is scored as if the excess were 40, i.e. such a score is a lower bound of Eq. (7), not
 * its value. Up to that excess the scores follow Eq. (7) / Eq. (5) to fp32 accuracy.
 * Route: blocks with both sizes non-zero are ordered by score descending (NaN as +inf),
 * ties by ascending a*Ck+b; cost of a block is |q_a||k_b|; walking that order, blocks are
 * routed while the summed cost stays <= the budget, stopping at the first that does not fit.
 * Tail row (index Cq) and tail column (index Ck) blocks are always routed and charged first.
 * PER_ROW: the same rule per query cluster a with budget floor(budget_cost*|q_a|/Nq).
 *
 *   qbar [BH,Cq,d], kbar, vbar [BH,Ck,d] fp32;  kp, vp [BH,Nk,d] dt, permuted (dense)
 *   q_offsets [BH,Cq+2], k_offsets [BH,Ck+2] int32
 *   budget_cost   number of (query,key) pairs per head, e.g. floor(rho*Nq*Nk), >= 0
 *   scores        [BH,Cq,Ck] fp32: out, or in with SVGEAR_USE_GIVEN_SCORES
 *   mask_bits     [BH,Cq+1,W] uint32 out, W = (Ck+1+31)/32; bit b of row a = block routed
 *   row_ptr       [BH,Cq+2] int32 out;  col_idx [BH,(Cq+1)*(Ck+1)] int32 out: routed key
 *                 clusters of row a, ascending, at col_idx[bh*(Cq+1)*(Ck+1) + row_ptr[a] ...]
 *   routed_cost   [BH] int64 out: summed cost of routed blocks (forced ones included)
 */
size_t svgear_probe_route_workspace(int B, int H, int64_t Nk, int d, int Cq, int Ck);
int svgear_probe_route(const float* qbar, const float* kbar, const float* vbar, const void* kp,
                       const void* vp, svgear_dtype dt, const int32_t* q_offsets,
                       const int32_t* k_offsets, int B, int H, int64_t Nq, int64_t Nk, int d,
                       int Cq, int Ck, int64_t budget_cost, float scale, unsigned flags,
                       float* scores, uint32_t* mask_bits, int32_t* row_ptr, int32_t* col_idx,
                       int64_t* routed_cost, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * probe + route with one ADAPTIVE budget per query cluster (Experiments, "Implementation":
 * the method inherits a top-p budget allocation, hyper-parameter "TopP", and routes per query
 * cluster). The paper does not define that allocation; this entry point implements a stated
 * reading of it, not a rule the paper prints:
 *   for query cluster a, every non-empty key cluster b carries the centroid attention mass
 *     mass_b = |k_b| exp(Sbar_ab - m_a)       (Sbar, m_a as in the probe above),
 *   counted in integer units w_b = floor(mass_b * 2^20) (fp32 evaluation); clusters are ordered
 *   by w_b descending, equal ones by ascending b; the shortest prefix whose summed weight
 *   reaches ceil(top_p * sum_b w_b) (double arithmetic) is kept, and
 *     row_budget[a] = |q_a| * sum over the kept b of |k_b|
 *   query-key pairs. Row a then routes its clustered blocks by descending score exactly as
 *   with SVGEAR_ROUTE_PER_ROW, up to row_budget[a]; the tail column and tail row are routed
 *   in addition and are not charged to it.
 * Arguments as svgear_probe_route, except: top_p in (0, 1] replaces budget_cost;
 * row_budget [BH,Cq] int64 out. flags: SVGEAR_PROBE_PLAIN and SVGEAR_USE_GIVEN_SCORES are
 * accepted (with given scores qbar and kbar are still read, for the masses);
 * SVGEAR_ROUTE_PER_ROW is implied and must not be set. Workspace: svgear_probe_route_workspace.
 */
int svgear_probe_route_top_p(const float* qbar, const float* kbar, const float* vbar, const void* kp,
                             const void* vp, svgear_dtype dt, const int32_t* q_offsets,
                             const int32_t* k_offsets, int B, int H, int64_t Nq, int64_t Nk, int d,
                             int Cq, int Ck, float top_p, float scale, unsigned flags, float* scores,
                             uint32_t* mask_bits, int32_t* row_ptr, int32_t* col_idx,
                             int64_t* routed_cost, int64_t* row_budget, void* ws, size_t ws_bytes,
                             void* stream);

/* ---------------------------------------------------------------------------------------
 * fused block-sparse attention + centroid compensation (Eq. (1), Eq. (6); Algorithm 2).
 *
 * For every query row i of query cluster a, one softmax over
 *   (i) every key j of every routed key cluster of row a: logit q_i.k_j*scale, value v_j;
 *  (ii) every non-routed, non-empty key cluster b as ONE pseudo-key: logit
 *       q_i.kbar_b*scale + ln|k_b|, value vbar_b
 * and op_i = sum(weights * values). This equals Eq. (6) with the map of Eq. (1).
 * bf16: QK^T and PV run on bf16 MFMA with fp32 accumulation, softmax in fp32, centroids are
 * rounded to bf16. fp32: everything in fp32.
 *
 *   qp [BH,Nq,d], kp, vp [BH,Nk,d] dt permuted;  kbar, vbar [BH,Ck,d] fp32
 *   q_offsets, k_offsets, mask_bits, row_ptr, col_idx as produced by svgear_probe_route
 *   op  [BH,Nq,d] dt out (permuted order);  lse [BH,Nq] fp32 out or NULL: natural log of the
 *   softmax denominator of each row.
 * Limits of the bf16 kernels (SVGEAR_ERR_UNSUPPORTED beyond them; fp32 has neither): the
 * per-key-cluster tables sit in LDS beside the K/V tile buffers (12 bytes per key cluster), which
 * allows Ck up to about 2500 for d = 128 and 8192 for d = 64; for d = 128 the K/V rows of a head are
 * addressed by 32-bit byte offsets, so Nk <= 16,777,215 keys per head.
 */
size_t svgear_sparse_attn_comp_workspace(int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                                         int Ck);
int svgear_sparse_attn_comp(const void* qp, const void* kp, const void* vp, svgear_dtype dt,
                            const float* kbar, const float* vbar, const int32_t* q_offsets,
                            const int32_t* k_offsets, const uint32_t* mask_bits,
                            const int32_t* row_ptr, const int32_t* col_idx, int B, int H,
                            int64_t Nq, int64_t Nk, int d, int Cq, int Ck, float scale, void* op,
                            float* lse, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * svgear_sparse_attn_comp with the queries' permutation folded into the kernel at both ends:
 * every lane of the kernel reads one whole query row and writes one whole output row, so
 * taking row p of head bh from token q_perm[bh*Nq + p] of the unpermuted queries, and sending
 * its result to that token of the output, costs no extra pass (neither the permuted copy of Q
 * nor svgear_unpermute is then needed; K and V are still streamed from their permuted copies).
 *   q [B,H,Nq,d] dt, token order, element strides qstride = {stride_b, stride_h, stride_n}
 *   q_perm [BH,Nq] int32 as produced by svgear_permute for the queries (n_tensors = 0 suffices)
 *   o [B,H,Nq,d] dt out, token order, element strides ostride
 *     (stride_n >= d and all strides multiples of 16 bytes, for q and for o)
 *   lse [BH,Nq] fp32 out or NULL, token order
 * Everything else as svgear_sparse_attn_comp (same workspace size).
 */
int svgear_sparse_attn_comp_token_order(const void* q, const int64_t qstride[3], const void* kp,
                                        const void* vp, svgear_dtype dt, const float* kbar,
                                        const float* vbar, const int32_t* q_offsets,
                                        const int32_t* k_offsets, const uint32_t* mask_bits,
                                        const int32_t* row_ptr, const int32_t* col_idx,
                                        const int32_t* q_perm, int B, int H, int64_t Nq, int64_t Nk,
                                        int d, int Cq, int Ck, float scale, void* o,
                                        const int64_t ostride[3], float* lse, void* ws,
                                        size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * The same result in the two-stage form of Algorithm 2, for comparison with the fused kernel:
 * (1) block-sparse exact attention over the routed blocks alone -> (O_r, LSE_r); (2) the
 * pseudo-keys of the skipped clusters alone -> (O_c, LSE_c); (3) merge:
 * op = (e^{LSE_r} O_r + e^{LSE_c} O_c) / (e^{LSE_r} + e^{LSE_c}), lse = log of that
 * denominator. Arguments as svgear_sparse_attn_comp; only dt = SVGEAR_BF16 with d = 128
 * (SVGEAR_ERR_UNSUPPORTED otherwise). The workspace also holds the two partial results.
 */
size_t svgear_sparse_attn_two_stage_workspace(int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                                              int Ck);
int svgear_sparse_attn_two_stage(const void* qp, const void* kp, const void* vp, svgear_dtype dt,
                                 const float* kbar, const float* vbar, const int32_t* q_offsets,
                                 const int32_t* k_offsets, const uint32_t* mask_bits,
                                 const int32_t* row_ptr, const int32_t* col_idx, int B, int H,
                                 int64_t Nq, int64_t Nk, int d, int Cq, int Ck, float scale,
                                 void* op, float* lse, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * unpermute: o[bh][perm[p]][:] = op[bh][p][:]  (inverse of the layout of "Structured
 * Redundancy").  op [BH,N,d] dense, perm [BH,N], o [B,H,N,d] with strides ostride.
 */
int svgear_unpermute(const void* op, const int32_t* perm, svgear_dtype dt, int B, int H,
                     int64_t N, int d, void* o, const int64_t ostride[3], void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVGEAR_H */
