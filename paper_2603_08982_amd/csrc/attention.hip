// Fused block-sparse exact attention + centroid compensation.
// Paper: Eq. (1) (compensated attention map), Eq. (6) (output), Algorithm 2 (a skipped key
// cluster enters the online softmax as one pseudo-key with logit q.kbar*scale + ln|k_c| and
// value vbar), "Linear Compensation" (cost O((Nq Ck + rho Nk Nq) d)).
//
// Work decomposition: the query rows of one query cluster are cut into tiles of BM rows; a
// tile never straddles two query clusters because the routing mask is per query cluster.
// The routed key clusters of that query cluster are concatenated into one virtual key
// sequence (cluster-contiguous K/V rows make every piece a contiguous row range), consumed
// in tiles of 64 keys regardless of cluster boundaries; the centroids of the skipped
// clusters follow as extra 64-key tiles with a per-key bias log2|k_b| (-inf for routed or
// empty clusters). One online softmax (base-2 exponent domain) runs over both phases.
//
// bf16 kernel (gfx950 MFMA, v_mfma_f32_32x32x16_bf16): each wave owns 32 query rows and
// computes the TRANSPOSED score tile S^T = K Q^T, so that every lane holds scores of a
// single query (lane%32) and row max / row sum need one cross-lane exchange (with lane^32)
// instead of a butterfly; exp2'd scores are then already in B-operand layout for
// O^T += V^T P^T. V tiles are transposed on their way into LDS.
// fp32 kernel: one query row per lane, plain fp32 FMAs (the fp32 reference-quality path).
#include "attention.h"

namespace svgear {
namespace {

// ------------------------------------------------------------------------------ plan
// Tile list of every head: tile -> (query cluster, first row). One workgroup per head.
__global__ void __launch_bounds__(256)
plan_kernel(const int32_t* __restrict__ q_offsets, int Cq, int BM, int max_tiles, int32_t* __restrict__ tile_a,
            int32_t* __restrict__ tile_row0, int32_t* __restrict__ n_tiles) {
  extern __shared__ int32_t first[];  // Cq+2
  const int bh = blockIdx.x, R = Cq + 1;
  const int32_t* qo = q_offsets + (int64_t)bh * (Cq + 2);
  for (int a = threadIdx.x; a < R; a += 256) first[a] = (qo[a + 1] - qo[a] + BM - 1) / BM;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int a = 0; a < R; ++a) {
      const int c = first[a];
      first[a] = run;
      run += c;
    }
    first[R] = run;
    n_tiles[bh] = run < max_tiles ? run : max_tiles;
  }
  __syncthreads();
  for (int a = threadIdx.x; a < R; a += 256) {
    const int lo = first[a], hi = first[a + 1];
    for (int t = lo; t < hi && t < max_tiles; ++t) {
      tile_a[(int64_t)bh * max_tiles + t] = a;
      tile_row0[(int64_t)bh * max_tiles + t] = qo[a] + (t - lo) * BM;
    }
  }
}

// Both centroid tables to bf16 in one launch (blockIdx.y picks the table).
__global__ void to_bf16_kernel(const float* __restrict__ src0, const float* __restrict__ src1, int64_t n,
                               bf16_t* __restrict__ dst0, bf16_t* __restrict__ dst1) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  if (blockIdx.y == 0) dst0[i] = f32_to_bf16(src0[i]);
  else dst1[i] = f32_to_bf16(src1[i]);
}

// ------------------------------------------------------------------------------ fp32
template <int D>
__global__ void __launch_bounds__(64)
attn_f32_kernel(AttnArgs p) {
  constexpr int TK = 16;
  __shared__ float4 ks[TK * D / 4];
  __shared__ float4 vs[TK * D / 4];
  const int bh = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
  if (tile >= p.n_tiles[bh]) return;
  const int Cq = p.Cq, Ck = p.Ck, R = Cq + 1, Cc = Ck + 1, W = (Cc + 31) / 32;
  const int a = p.tile_a[(int64_t)bh * p.max_tiles + tile];
  const int row0 = p.tile_row0[(int64_t)bh * p.max_tiles + tile];
  const int32_t* qo = p.q_offsets + (int64_t)bh * (Cq + 2);
  const int32_t* ko = p.k_offsets + (int64_t)bh * (Ck + 2);
  const int row_end = qo[a + 1];
  const int row = row0 + tid;
  const bool valid = row < row_end;
  const float* kh = static_cast<const float*>(p.kp) + (int64_t)bh * p.Nk * D;
  const float* vh = static_cast<const float*>(p.vp) + (int64_t)bh * p.Nk * D;
  const float c = p.scale * kLog2e;
  float q[D], acc[D];
  {
    const float4* qr = reinterpret_cast<const float4*>(static_cast<const float*>(p.qp) +
                                                       q_row_offset(p, bh, valid ? row : row_end - 1, D));
#pragma unroll
    for (int t = 0; t < D / 4; ++t) {
      const float4 v = qr[t];
      q[4 * t] = v.x; q[4 * t + 1] = v.y; q[4 * t + 2] = v.z; q[4 * t + 3] = v.w;
      acc[4 * t] = acc[4 * t + 1] = acc[4 * t + 2] = acc[4 * t + 3] = 0.f;
    }
  }
  float m = -INFINITY, l = 0.f;
  const int32_t* rp = p.row_ptr + (int64_t)bh * (R + 1);
  const int32_t* ci = p.col_idx + (int64_t)bh * R * Cc + rp[a];
  const int ne = rp[a + 1] - rp[a];
  for (int e = 0; e < ne; ++e) {
    const int b = ci[e];
    const int kend = ko[b + 1];
    for (int j0 = ko[b]; j0 < kend; j0 += TK) {
      const int nk = min(TK, kend - j0);
      __syncthreads();
      const float4* ksrc = reinterpret_cast<const float4*>(kh + (int64_t)j0 * D);
      const float4* vsrc = reinterpret_cast<const float4*>(vh + (int64_t)j0 * D);
      for (int i = tid; i < nk * D / 4; i += 64) {
        ks[i] = ksrc[i];
        vs[i] = vsrc[i];
      }
      __syncthreads();
      float s[TK];
      float mx = m;
#pragma unroll
      for (int kk = 0; kk < TK; ++kk) {
        s[kk] = -INFINITY;
        if (kk < nk) {
          float dot = 0.f;
#pragma unroll
          for (int t = 0; t < D / 4; ++t) {
            const float4 v = ks[kk * (D / 4) + t];
            dot = __builtin_fmaf(q[4 * t], v.x, dot);
            dot = __builtin_fmaf(q[4 * t + 1], v.y, dot);
            dot = __builtin_fmaf(q[4 * t + 2], v.z, dot);
            dot = __builtin_fmaf(q[4 * t + 3], v.w, dot);
          }
          s[kk] = dot * c;
          mx = fmaxf(mx, s[kk]);
        }
      }
      if (mx > m) {
        const float alpha = exp2f(m - mx);
        l *= alpha;
#pragma unroll
        for (int t = 0; t < D; ++t) acc[t] *= alpha;
        m = mx;
      }
#pragma unroll
      for (int kk = 0; kk < TK; ++kk) {
        if (kk < nk) {
          const float pr = exp2f(s[kk] - m);
          l += pr;
#pragma unroll
          for (int t = 0; t < D / 4; ++t) {
            const float4 v = vs[kk * (D / 4) + t];
            acc[4 * t] = __builtin_fmaf(pr, v.x, acc[4 * t]);
            acc[4 * t + 1] = __builtin_fmaf(pr, v.y, acc[4 * t + 1]);
            acc[4 * t + 2] = __builtin_fmaf(pr, v.z, acc[4 * t + 2]);
            acc[4 * t + 3] = __builtin_fmaf(pr, v.w, acc[4 * t + 3]);
          }
        }
      }
    }
  }
  // compensation: every non-routed, non-empty key cluster as one pseudo-key
  if (a < Cq) {
    const uint32_t* mrow = p.mask_bits + ((int64_t)bh * R + a) * W;
    for (int b = 0; b < Ck; ++b) {
      const int sz = ko[b + 1] - ko[b];
      if (sz <= 0 || mask_bit(mrow, b)) continue;
      const float4* kb = reinterpret_cast<const float4*>(p.kbar + ((int64_t)bh * Ck + b) * D);
      const float4* vb = reinterpret_cast<const float4*>(p.vbar + ((int64_t)bh * Ck + b) * D);
      float dot = 0.f;
#pragma unroll
      for (int t = 0; t < D / 4; ++t) {
        const float4 v = kb[t];
        dot = __builtin_fmaf(q[4 * t], v.x, dot);
        dot = __builtin_fmaf(q[4 * t + 1], v.y, dot);
        dot = __builtin_fmaf(q[4 * t + 2], v.z, dot);
        dot = __builtin_fmaf(q[4 * t + 3], v.w, dot);
      }
      const float s = __builtin_fmaf(dot, c, log2f((float)sz));
      if (s > m) {
        const float alpha = exp2f(m - s);
        l *= alpha;
#pragma unroll
        for (int t = 0; t < D; ++t) acc[t] *= alpha;
        m = s;
      }
      const float pr = exp2f(s - m);
      l += pr;
#pragma unroll
      for (int t = 0; t < D / 4; ++t) {
        const float4 v = vb[t];
        acc[4 * t] = __builtin_fmaf(pr, v.x, acc[4 * t]);
        acc[4 * t + 1] = __builtin_fmaf(pr, v.y, acc[4 * t + 1]);
        acc[4 * t + 2] = __builtin_fmaf(pr, v.z, acc[4 * t + 2]);
        acc[4 * t + 3] = __builtin_fmaf(pr, v.w, acc[4 * t + 3]);
      }
    }
  }
  if (valid) {
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    int64_t lse_idx;
    float4* o = reinterpret_cast<float4*>(static_cast<float*>(p.op) + out_row_offset(p, bh, row, D, lse_idx));
#pragma unroll
    for (int t = 0; t < D / 4; ++t)
      o[t] = make_float4(acc[4 * t] * inv, acc[4 * t + 1] * inv, acc[4 * t + 2] * inv, acc[4 * t + 3] * inv);
    if (p.lse) p.lse[lse_idx] = (m + log2f(l)) * kLn2;
  }
}


}  // namespace
}  // namespace svgear

using namespace svgear;

static int attn_bm(svgear_dtype dt, int d) { return dt == SVGEAR_F32 ? 64 : attn_bf16_bm(d); }

extern "C" size_t svgear_sparse_attn_comp_workspace(int B, int H, int64_t Nq, int64_t Nk, int d, int Cq, int Ck) {
  (void)Nk;
  if (B <= 0 || H <= 0 || Nq <= 0 || Cq <= 0 || Ck <= 0 || d <= 0) return 0;
  const size_t BH = (size_t)B * H;
  const size_t max_tiles = (size_t)ceil_div(Nq, 64) + Cq + 1;  // bound for either tile height
  return 2 * align_up(BH * max_tiles * 4, 256) + align_up(BH * 4, 256) + 2 * align_up(BH * Ck * d * 2, 256) +
         plan_d128_workspace((int)BH, Cq, Nq);
}

static int attn_run(const void* qp, const void* kp, const void* vp, svgear_dtype dt, const float* kbar,
                    const float* vbar, const int32_t* q_offsets, const int32_t* k_offsets, const uint32_t* mask_bits,
                    const int32_t* row_ptr, const int32_t* col_idx, int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                    int Ck, float scale, void* op, float* lse, void* ws, size_t ws_bytes, void* stream, int part,
                    const int32_t* tok_perm = nullptr, const int64_t* qstride = nullptr,
                    const int64_t* ostride = nullptr) {
  if (!qp || !kp || !vp || !kbar || !vbar || !q_offsets || !k_offsets || !mask_bits || !row_ptr || !col_idx || !op ||
      B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || Cq <= 0 || Ck <= 0 || Cq > 8192 || Ck > 8192 ||
      Nq > INT32_MAX / 2 || Nk > INT32_MAX / 2 || (d != 64 && d != 128) || (dt != SVGEAR_F32 && dt != SVGEAR_BF16) ||
      !(scale > 0.f))
    return SVGEAR_ERR_INVALID;
  const void* ptrs[] = {qp, kp, vp, kbar, vbar, op};
  for (const void* q : ptrs)
    if (reinterpret_cast<uintptr_t>(q) % 16) return SVGEAR_ERR_INVALID;
  Strides q_st{0, 0, 0}, out_st{0, 0, 0};
  if (tok_perm) {  // token order at both ends: strides in elements, rows 16-byte aligned
    const int64_t es = dt == SVGEAR_F32 ? 4 : 2;
    if (!qstride || !ostride) return SVGEAR_ERR_INVALID;
    for (int i = 0; i < 3; ++i)
      if (qstride[i] < 0 || (qstride[i] * es) % 16 || ostride[i] < 0 || (ostride[i] * es) % 16)
        return SVGEAR_ERR_INVALID;
    if (qstride[2] < d || ostride[2] < d) return SVGEAR_ERR_INVALID;
    q_st = Strides{qstride[0], qstride[1], qstride[2]};
    out_st = Strides{ostride[0], ostride[1], ostride[2]};
  }
  if (!ws || ws_bytes < svgear_sparse_attn_comp_workspace(B, H, Nq, Nk, d, Cq, Ck)) return SVGEAR_ERR_WORKSPACE;
  const int BH = B * H;
  if ((int64_t)BH * ((int64_t)ceil_div(Nq, 64) + Cq + 1) > INT32_MAX / 2) return SVGEAR_ERR_UNSUPPORTED;
  if (part != 0 && !(dt == SVGEAR_BF16 && d == 128)) return SVGEAR_ERR_UNSUPPORTED;
  if (dt == SVGEAR_BF16 && attn_bf16_lds_bytes(d, Ck) > 160 * 1024) return SVGEAR_ERR_UNSUPPORTED;
  // the d = 128 bf16 kernel addresses K/V rows of a head by 32-bit byte offsets (256 bytes a row)
  if (dt == SVGEAR_BF16 && d == 128 && Nk > (int64_t)(UINT32_MAX / 256)) return SVGEAR_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  Workspace w(ws, ws_bytes);
  const int BM = attn_bm(dt, d);
  const int max_tiles = (int)(ceil_div(Nq, BM) + Cq + 1);
  const size_t cap = (size_t)ceil_div(Nq, 64) + Cq + 1;
  int32_t* tile_a = w.take<int32_t>((size_t)BH * cap);
  int32_t* tile_row0 = w.take<int32_t>((size_t)BH * cap);
  int32_t* n_tiles = w.take<int32_t>(BH);
  bf16_t* kbar16 = w.take<bf16_t>((size_t)BH * Ck * d);
  bf16_t* vbar16 = w.take<bf16_t>((size_t)BH * Ck * d);
  if (!w.ok()) return SVGEAR_ERR_WORKSPACE;
  if (!(dt == SVGEAR_BF16 && d == 128)) {  // the d = 128 bf16 kernel has work lists of its own (plan_d128)
    plan_kernel<<<BH, 256, (Cq + 2) * sizeof(int32_t), s>>>(q_offsets, Cq, BM, max_tiles, tile_a, tile_row0, n_tiles);
    SVGEAR_LAUNCH_CHECK();
  }
  AttnArgs a{qp, kp, vp, kbar, vbar, kbar16, vbar16, q_offsets, k_offsets, mask_bits, row_ptr, col_idx,
             tile_a, tile_row0, n_tiles, nullptr, nullptr, nullptr, nullptr, nullptr,
             Nq, Nk, BH, Cq, Ck, max_tiles, scale, op, lse, part, tok_perm, q_st, out_st, H};
  if (dt == SVGEAR_F32) {
    dim3 grid(max_tiles, BH);
    if (d == 64)
      attn_f32_kernel<64><<<grid, 64, 0, s>>>(a);
    else
      attn_f32_kernel<128><<<grid, 64, 0, s>>>(a);
    SVGEAR_LAUNCH_CHECK();
    return SVGEAR_OK;
  }
  const int64_t n = (int64_t)BH * Ck * d;
  to_bf16_kernel<<<dim3((unsigned)ceil_div(n, 256), 2), 256, 0, s>>>(kbar, vbar, n, kbar16, vbar16);
  SVGEAR_LAUNCH_CHECK();
  if (d == 128) {
    const int rc = plan_d128(a, static_cast<char*>(ws) + w.used, ws_bytes - w.used, s);
    if (rc != SVGEAR_OK) return rc;
  }
  const unsigned total = (unsigned)align_up((size_t)BH * max_tiles, 8);
  return launch_attn_bf16(a, d, total, s);
}

extern "C" int svgear_sparse_attn_comp(const void* qp, const void* kp, const void* vp, svgear_dtype dt,
                                       const float* kbar, const float* vbar, const int32_t* q_offsets,
                                       const int32_t* k_offsets, const uint32_t* mask_bits, const int32_t* row_ptr,
                                       const int32_t* col_idx, int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                                       int Ck, float scale, void* op, float* lse, void* ws, size_t ws_bytes,
                                       void* stream) {
  return attn_run(qp, kp, vp, dt, kbar, vbar, q_offsets, k_offsets, mask_bits, row_ptr, col_idx, B, H, Nq, Nk, d, Cq,
                  Ck, scale, op, lse, ws, ws_bytes, stream, 0);
}

extern "C" int svgear_sparse_attn_comp_token_order(const void* q, const int64_t qstride[3], const void* kp,
                                                   const void* vp, svgear_dtype dt, const float* kbar,
                                                   const float* vbar, const int32_t* q_offsets,
                                                   const int32_t* k_offsets, const uint32_t* mask_bits,
                                                   const int32_t* row_ptr, const int32_t* col_idx,
                                                   const int32_t* q_perm, int B, int H, int64_t Nq, int64_t Nk, int d,
                                                   int Cq, int Ck, float scale, void* o, const int64_t ostride[3],
                                                   float* lse, void* ws, size_t ws_bytes, void* stream) {
  if (!q_perm || !qstride || !ostride) return SVGEAR_ERR_INVALID;
  return attn_run(q, kp, vp, dt, kbar, vbar, q_offsets, k_offsets, mask_bits, row_ptr, col_idx, B, H, Nq, Nk, d, Cq,
                  Ck, scale, o, lse, ws, ws_bytes, stream, 0, q_perm, qstride, ostride);
}

extern "C" size_t svgear_sparse_attn_two_stage_workspace(int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                                                         int Ck) {
  const size_t base = svgear_sparse_attn_comp_workspace(B, H, Nq, Nk, d, Cq, Ck);
  if (base == 0) return 0;
  const size_t BH = (size_t)B * H;
  return align_up(base, 256) + 2 * align_up(BH * Nq * d * 2, 256) + 2 * align_up(BH * Nq * 4, 256);
}

extern "C" int svgear_sparse_attn_two_stage(const void* qp, const void* kp, const void* vp, svgear_dtype dt,
                                            const float* kbar, const float* vbar, const int32_t* q_offsets,
                                            const int32_t* k_offsets, const uint32_t* mask_bits,
                                            const int32_t* row_ptr, const int32_t* col_idx, int B, int H, int64_t Nq,
                                            int64_t Nk, int d, int Cq, int Ck, float scale, void* op, float* lse,
                                            void* ws, size_t ws_bytes, void* stream) {
  if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || Cq <= 0 || Ck <= 0 || !op) return SVGEAR_ERR_INVALID;
  if (!(dt == SVGEAR_BF16 && d == 128)) return SVGEAR_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < svgear_sparse_attn_two_stage_workspace(B, H, Nq, Nk, d, Cq, Ck)) return SVGEAR_ERR_WORKSPACE;
  const size_t base = align_up(svgear_sparse_attn_comp_workspace(B, H, Nq, Nk, d, Cq, Ck), 256);
  const size_t BH = (size_t)B * H;
  Workspace w(static_cast<char*>(ws) + base, ws_bytes - base);
  bf16_t* o_r = w.take<bf16_t>(BH * Nq * d);
  bf16_t* o_c = w.take<bf16_t>(BH * Nq * d);
  float* lse_r = w.take<float>(BH * Nq);
  float* lse_c = w.take<float>(BH * Nq);
  if (!w.ok()) return SVGEAR_ERR_WORKSPACE;
  int rc = attn_run(qp, kp, vp, dt, kbar, vbar, q_offsets, k_offsets, mask_bits, row_ptr, col_idx, B, H, Nq, Nk, d,
                    Cq, Ck, scale, o_r, lse_r, ws, base, stream, 1);
  if (rc != SVGEAR_OK) return rc;
  rc = attn_run(qp, kp, vp, dt, kbar, vbar, q_offsets, k_offsets, mask_bits, row_ptr, col_idx, B, H, Nq, Nk, d, Cq,
                Ck, scale, o_c, lse_c, ws, base, stream, 2);
  if (rc != SVGEAR_OK) return rc;
  return launch_merge(o_r, lse_r, o_c, lse_c, (int64_t)BH * Nq, d, static_cast<bf16_t*>(op), lse,
                      static_cast<hipStream_t>(stream));
}
