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
#include "common.h"

namespace svgear {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int BN = 64;  // keys per tile

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

__global__ void to_bf16_kernel(const float* __restrict__ src, int64_t n, bf16_t* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = f32_to_bf16(src[i]);
}

struct AttnArgs {
  const void* qp;
  const void* kp;
  const void* vp;
  const float* kbar;
  const float* vbar;
  const bf16_t* kbar16;
  const bf16_t* vbar16;
  const int32_t* q_offsets;
  const int32_t* k_offsets;
  const uint32_t* mask_bits;
  const int32_t* row_ptr;
  const int32_t* col_idx;
  const int32_t* tile_a;
  const int32_t* tile_row0;
  const int32_t* n_tiles;
  int64_t Nq, Nk;
  int BH, Cq, Ck, max_tiles;
  float scale;
  void* op;
  float* lse;
};

__device__ __forceinline__ bool mask_bit(const uint32_t* mrow, int b) { return (mrow[b >> 5] >> (b & 31)) & 1u; }

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
  const float* qh = static_cast<const float*>(p.qp) + (int64_t)bh * p.Nq * D;
  const float* kh = static_cast<const float*>(p.kp) + (int64_t)bh * p.Nk * D;
  const float* vh = static_cast<const float*>(p.vp) + (int64_t)bh * p.Nk * D;
  const float c = p.scale * kLog2e;
  float q[D], acc[D];
  {
    const float4* qr = reinterpret_cast<const float4*>(qh + (int64_t)(valid ? row : row_end - 1) * D);
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
    float4* o = reinterpret_cast<float4*>(static_cast<float*>(p.op) + ((int64_t)bh * p.Nq + row) * D);
#pragma unroll
    for (int t = 0; t < D / 4; ++t)
      o[t] = make_float4(acc[4 * t] * inv, acc[4 * t + 1] * inv, acc[4 * t + 2] * inv, acc[4 * t + 3] * inv);
    if (p.lse) p.lse[(int64_t)bh * p.Nq + row] = (m + log2f(l)) * kLn2;
  }
}

// ------------------------------------------------------------------------------ bf16 MFMA
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  union { bf16x2 b; uint32_t u; } c;
  c.b = b;
  return c.u;
}

template <int D>
struct Bf16Tile {
  static constexpr int KROW = D + 8;         // bf16 per K row in LDS (16-byte pad: conflict-free b128 reads)
  static constexpr int VROW = BN + 8;        // bf16 per V^T row in LDS
  static constexpr int K_ELEMS = BN * KROW;  // per buffer
  static constexpr int V_ELEMS = D * VROW;
};

static inline size_t attn_bf16_lds_bytes(int D, int Ck) {
  const size_t kv = 2 * ((size_t)BN * (D + 8) + (size_t)D * (BN + 8)) * 2;
  const size_t lw = (size_t)align_up(Ck, 64) * 4;
  const size_t seg = (size_t)(2 * (Ck + 1) + 1) * 4;
  return kv + 2 * BN * 4 + lw + align_up(seg, 16);
}

// NW waves of 32 query rows each.
template <int D, int NW>
__global__ void __launch_bounds__(64 * NW)
attn_bf16_kernel(AttnArgs p) {
  constexpr int NT = 64 * NW;
  constexpr int BM = 32 * NW;
  constexpr int KS = D / 16;           // k-steps of the QK^T product
  constexpr int DB = D / 32;           // 32-row blocks of O^T
  constexpr int CPR = D / 8;           // 16-byte chunks per K/V row
  constexpr int KCH = BN * CPR / NT;   // K chunks per thread
  constexpr int VUNITS = 16 * CPR;     // (4-key group) x (8-dim group) units per V tile
  constexpr int VCH = (VUNITS + NT - 1) / NT;
  using TL = Bf16Tile<D>;
  static_assert(BN * CPR % NT == 0, "tile/threads mismatch");
  (void)BM;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem);                       // [2][BN][KROW]
  bf16_t* Vs = Ks + 2 * TL::K_ELEMS;                                  // [2][D][VROW]
  int32_t* rowmap = reinterpret_cast<int32_t*>(Vs + 2 * TL::V_ELEMS);  // [2][BN]
  float* lw = reinterpret_cast<float*>(rowmap + 2 * BN);              // [align64(Ck)]
  int32_t* vstart = reinterpret_cast<int32_t*>(lw + ((p.Ck + 63) & ~63));  // [ne+1]
  int32_t* pstart = vstart + (p.Ck + 2);                                    // [ne]

  // XCD-aware tile order: workgroup ids go round-robin over the 8 XCDs; give each XCD one
  // contiguous range of logical tiles so tiles that share routed K/V share an L2.
  const int total = gridDim.x;
  const int wg = blockIdx.x;
  const int logical = (wg & 7) * (total >> 3) + (wg >> 3);
  const int bh = logical / p.max_tiles, tile = logical % p.max_tiles;
  if (bh >= p.BH || tile >= p.n_tiles[bh]) return;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int Cq = p.Cq, Ck = p.Ck, R = Cq + 1, Cc = Ck + 1, W = (Cc + 31) / 32;
  const int a = p.tile_a[(int64_t)bh * p.max_tiles + tile];
  const int row0 = p.tile_row0[(int64_t)bh * p.max_tiles + tile];
  const int32_t* qo = p.q_offsets + (int64_t)bh * (Cq + 2);
  const int32_t* ko = p.k_offsets + (int64_t)bh * (Ck + 2);
  const int row_end = qo[a + 1];
  const int32_t* rp = p.row_ptr + (int64_t)bh * (R + 1);
  const int32_t* ci = p.col_idx + (int64_t)bh * R * Cc + rp[a];
  const int ne = rp[a + 1] - rp[a];
  const uint32_t* mrow = p.mask_bits + ((int64_t)bh * R + a) * W;

  // ---- prologue: virtual key sequence of the routed clusters, compensation biases
  if (wave == 0) {
    int carry = 0;
    for (int e0 = 0; e0 < ne; e0 += 64) {
      const int e = e0 + lane;
      int sz = 0;
      if (e < ne) {
        const int b = ci[e];
        const int ps = ko[b];
        sz = ko[b + 1] - ps;
        sz = sz > 0 ? sz : 0;
        pstart[e] = ps;
      }
      int incl = sz;
      for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      if (e < ne) vstart[e] = carry + incl - sz;
      carry += __shfl(incl, 63);
    }
    if (lane == 0) vstart[ne] = carry;
  }
  for (int b = tid; b < ((Ck + 63) & ~63); b += NT) {
    float v = -INFINITY;
    if (b < Ck && a < Cq) {
      const int sz = ko[b + 1] - ko[b];
      if (sz > 0 && !mask_bit(mrow, b)) v = log2f((float)sz);
    }
    lw[b] = v;
  }
  __syncthreads();
  const int n_r = vstart[ne];
  const int nt_r = (n_r + BN - 1) / BN;
  const int nt_c = (a < Cq) ? (Ck + BN - 1) / BN : 0;
  const int T = nt_r + nt_c;

  const bf16_t* kh = static_cast<const bf16_t*>(p.kp) + (int64_t)bh * p.Nk * D;
  const bf16_t* vh = static_cast<const bf16_t*>(p.vp) + (int64_t)bh * p.Nk * D;
  const bf16_t* kc = p.kbar16 + (int64_t)bh * Ck * D;
  const bf16_t* vc = p.vbar16 + (int64_t)bh * Ck * D;

  int cur = 0;  // segment cursor of threads 0..63 (virtual position -> permuted K/V row)
  auto map_tile = [&](int t) {
    if (tid < BN) {
      int phys;
      if (t < nt_r) {
        const int pos = t * BN + tid;
        if (pos < n_r) {
          while (pos >= vstart[cur + 1]) ++cur;
          phys = pstart[cur] + (pos - vstart[cur]);
        } else {
          phys = 0;  // masked below; any valid row
        }
      } else {
        const int b = (t - nt_r) * BN + tid;
        phys = b < Ck ? b : Ck - 1;
      }
      rowmap[(t & 1) * BN + tid] = phys;
    }
  };

  uint4 kreg[KCH], vreg[VCH][4];
  auto issue_loads = [&](int t) {
    const bf16_t* kb = t < nt_r ? kh : kc;
    const bf16_t* vb = t < nt_r ? vh : vc;
    const int32_t* rm = rowmap + (t & 1) * BN;
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int chunk = tid + i * NT;
      const int r = chunk / CPR, c16 = chunk % CPR;
      kreg[i] = *reinterpret_cast<const uint4*>(kb + (int64_t)rm[r] * D + c16 * 8);
    }
#pragma unroll
    for (int i = 0; i < VCH; ++i) {
      const int unit = tid + i * NT;
      if (unit < VUNITS) {
        const int kg = unit / CPR, dg = unit % CPR;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
          vreg[i][qd] = *reinterpret_cast<const uint4*>(vb + (int64_t)rm[4 * kg + qd] * D + dg * 8);
      }
    }
  };
  auto store_tiles = [&](int buf) {
    bf16_t* Kb = Ks + buf * TL::K_ELEMS;
    bf16_t* Vb = Vs + buf * TL::V_ELEMS;
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int chunk = tid + i * NT;
      const int r = chunk / CPR, c16 = chunk % CPR;
      *reinterpret_cast<uint4*>(Kb + r * TL::KROW + c16 * 8) = kreg[i];
    }
#pragma unroll
    for (int i = 0; i < VCH; ++i) {
      const int unit = tid + i * NT;
      if (unit < VUNITS) {
        const int kg = unit / CPR, dg = unit % CPR;
        // column of key 4*kg inside its 16-key group: keys are stored so that the 8 keys a
        // lane needs for one MFMA B/A operand pair are contiguous
        const int g4 = kg & 3;
        const int pos0 = 16 * (kg >> 2) + 8 * (g4 & 1) + 4 * (g4 >> 1);
        const uint32_t w0[4] = {vreg[i][0].x, vreg[i][0].y, vreg[i][0].z, vreg[i][0].w};
        const uint32_t w1[4] = {vreg[i][1].x, vreg[i][1].y, vreg[i][1].z, vreg[i][1].w};
        const uint32_t w2[4] = {vreg[i][2].x, vreg[i][2].y, vreg[i][2].z, vreg[i][2].w};
        const uint32_t w3[4] = {vreg[i][3].x, vreg[i][3].y, vreg[i][3].z, vreg[i][3].w};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int wd = u >> 1;
          uint2 o;
          if (u & 1) {
            o.x = (w0[wd] >> 16) | (w1[wd] & 0xffff0000u);
            o.y = (w2[wd] >> 16) | (w3[wd] & 0xffff0000u);
          } else {
            o.x = (w0[wd] & 0xffffu) | (w1[wd] << 16);
            o.y = (w2[wd] & 0xffffu) | (w3[wd] << 16);
          }
          *reinterpret_cast<uint2*>(Vb + (8 * dg + u) * TL::VROW + pos0) = o;
        }
      }
    }
  };

  // ---- Q fragments (B operand of S^T = K Q^T): lane holds query li, dims 16s + 8*lh + 0..7
  const int qrow = row0 + 32 * wave + li;
  const bool qvalid = qrow < row_end;
  const bool wave_active = (row0 + 32 * wave) < row_end;
  bf16x8 bq[KS];
  {
    const bf16_t* qr = static_cast<const bf16_t*>(p.qp) + ((int64_t)bh * p.Nq + (qvalid ? qrow : row_end - 1)) * D;
#pragma unroll
    for (int s = 0; s < KS; ++s) bq[s] = as_bf16x8(*reinterpret_cast<const uint4*>(qr + 16 * s + 8 * lh));
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float c = p.scale * kLog2e;

  if (T > 0) {
    map_tile(0);
    if (T > 1) map_tile(1);
    __syncthreads();
    issue_loads(0);
    store_tiles(0);
    __syncthreads();
  }

  for (int t = 0; t < T; ++t) {
    const int buf = t & 1;
    if (t + 1 < T) issue_loads(t + 1);
    if (wave_active) {
      const bf16_t* Kb = Ks + buf * TL::K_ELEMS;
      const bf16_t* Vb = Vs + buf * TL::V_ELEMS;
      // ---- S^T tile: 64 keys x 32 queries
      f32x16 sacc[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const bf16x8 ak =
              as_bf16x8(*reinterpret_cast<const uint4*>(Kb + (32 * kb + li) * TL::KROW + 16 * s + 8 * lh));
          sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[s], sacc[kb], 0, 0, 0);
        }
      }
      // register r of block kb is key 32*kb + 8*(r/4) + 4*lh + r%4 of this tile
      float mx = -INFINITY;
      if (t < nt_r) {
        const int left = n_r - t * BN;  // valid keys in this tile
        if (left < BN) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (32 * kb + 8 * (r >> 2) + 4 * lh + (r & 3) >= left) sacc[kb][r] = -INFINITY;
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            sacc[kb][r] *= c;
            mx = fmaxf(mx, sacc[kb][r]);
          }
      } else {
        const float* lwt = lw + (t - nt_r) * BN;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float4 bias = *reinterpret_cast<const float4*>(lwt + 32 * kb + 8 * g + 4 * lh);
            sacc[kb][4 * g + 0] = __builtin_fmaf(sacc[kb][4 * g + 0], c, bias.x);
            sacc[kb][4 * g + 1] = __builtin_fmaf(sacc[kb][4 * g + 1], c, bias.y);
            sacc[kb][4 * g + 2] = __builtin_fmaf(sacc[kb][4 * g + 2], c, bias.z);
            sacc[kb][4 * g + 3] = __builtin_fmaf(sacc[kb][4 * g + 3], c, bias.w);
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, sacc[kb][4 * g + r]);
          }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx);
      if (__any(m_new > m)) {
        const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - m_new);
        l *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        m = m_new;
      }
      const float m_use = (m == -INFINITY) ? 0.f : m;
      uint32_t pk[2][8];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(sacc[kb][r] - m_use);
          const float p1 = __builtin_amdgcn_exp2f(sacc[kb][r + 1] - m_use);
          l += p0 + p1;
          pk[kb][r >> 1] = pack_bf16(p0, p1);
        }
      // ---- O^T += V^T P^T : k-step ks covers keys 16*ks .. 16*ks+15
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kb = ks >> 1, u4 = (ks & 1) * 4;
        uint4 pw = make_uint4(pk[kb][u4], pk[kb][u4 + 1], pk[kb][u4 + 2], pk[kb][u4 + 3]);
        const bf16x8 bp = as_bf16x8(pw);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 av =
              as_bf16x8(*reinterpret_cast<const uint4*>(Vb + (32 * db + li) * TL::VROW + 16 * ks + 8 * lh));
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bp, oacc[db], 0, 0, 0);
        }
      }
    }
    if (t + 2 < T) map_tile(t + 2);
    if (t + 1 < T) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: normalise and write (lane holds query li, dims 32db + 8g + 4lh + 0..3)
  if (wave_active) {
    const float lt = l + __shfl_xor(l, 32);
    if (qvalid) {
      const float inv = lt > 0.f ? 1.0f / lt : 0.f;
      bf16_t* o = static_cast<bf16_t*>(p.op) + ((int64_t)bh * p.Nq + qrow) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = pack_bf16(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
          w.y = pack_bf16(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
          *reinterpret_cast<uint2*>(o + 32 * db + 8 * g + 4 * lh) = w;
        }
      if (p.lse && lh == 0) p.lse[(int64_t)bh * p.Nq + qrow] = (m + log2f(lt)) * kLn2;
    }
  }
}

constexpr int kBf16Waves = 4;

}  // namespace
}  // namespace svgear

using namespace svgear;

static int attn_bm(svgear_dtype dt) { return dt == SVGEAR_F32 ? 64 : 32 * kBf16Waves; }

extern "C" size_t svgear_sparse_attn_comp_workspace(int B, int H, int64_t Nq, int64_t Nk, int d, int Cq, int Ck) {
  (void)Nk;
  if (B <= 0 || H <= 0 || Nq <= 0 || Cq <= 0 || Ck <= 0 || d <= 0) return 0;
  const size_t BH = (size_t)B * H;
  const size_t max_tiles = (size_t)ceil_div(Nq, 64) + Cq + 1;  // bound for either tile height
  return 2 * align_up(BH * max_tiles * 4, 256) + align_up(BH * 4, 256) + 2 * align_up(BH * Ck * d * 2, 256);
}

extern "C" int svgear_sparse_attn_comp(const void* qp, const void* kp, const void* vp, svgear_dtype dt,
                                       const float* kbar, const float* vbar, const int32_t* q_offsets,
                                       const int32_t* k_offsets, const uint32_t* mask_bits, const int32_t* row_ptr,
                                       const int32_t* col_idx, int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                                       int Ck, float scale, void* op, float* lse, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (!qp || !kp || !vp || !kbar || !vbar || !q_offsets || !k_offsets || !mask_bits || !row_ptr || !col_idx || !op ||
      B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || Cq <= 0 || Ck <= 0 || Cq > 8192 || Ck > 8192 ||
      Nq > INT32_MAX / 2 || Nk > INT32_MAX / 2 || (d != 64 && d != 128) || (dt != SVGEAR_F32 && dt != SVGEAR_BF16) ||
      !(scale > 0.f))
    return SVGEAR_ERR_INVALID;
  const void* ptrs[] = {qp, kp, vp, kbar, vbar, op};
  for (const void* q : ptrs)
    if (reinterpret_cast<uintptr_t>(q) % 16) return SVGEAR_ERR_INVALID;
  if (!ws || ws_bytes < svgear_sparse_attn_comp_workspace(B, H, Nq, Nk, d, Cq, Ck)) return SVGEAR_ERR_WORKSPACE;
  const int BH = B * H;
  if ((int64_t)BH * ((int64_t)ceil_div(Nq, 64) + Cq + 1) > INT32_MAX / 2) return SVGEAR_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  Workspace w(ws, ws_bytes);
  const int BM = attn_bm(dt);
  const int max_tiles = (int)(ceil_div(Nq, BM) + Cq + 1);
  const size_t cap = (size_t)ceil_div(Nq, 64) + Cq + 1;
  int32_t* tile_a = w.take<int32_t>((size_t)BH * cap);
  int32_t* tile_row0 = w.take<int32_t>((size_t)BH * cap);
  int32_t* n_tiles = w.take<int32_t>(BH);
  bf16_t* kbar16 = w.take<bf16_t>((size_t)BH * Ck * d);
  bf16_t* vbar16 = w.take<bf16_t>((size_t)BH * Ck * d);
  if (!w.ok()) return SVGEAR_ERR_WORKSPACE;
  plan_kernel<<<BH, 256, (Cq + 2) * sizeof(int32_t), s>>>(q_offsets, Cq, BM, max_tiles, tile_a, tile_row0, n_tiles);
  SVGEAR_LAUNCH_CHECK();
  AttnArgs a{qp, kp, vp, kbar, vbar, kbar16, vbar16, q_offsets, k_offsets, mask_bits, row_ptr, col_idx,
             tile_a, tile_row0, n_tiles, Nq, Nk, BH, Cq, Ck, max_tiles, scale, op, lse};
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
  to_bf16_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(kbar, n, kbar16);
  SVGEAR_LAUNCH_CHECK();
  to_bf16_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(vbar, n, vbar16);
  SVGEAR_LAUNCH_CHECK();
  const size_t lds = attn_bf16_lds_bytes(d, Ck);
  if (lds > 160 * 1024) return SVGEAR_ERR_UNSUPPORTED;
  const unsigned total = (unsigned)align_up((size_t)BH * max_tiles, 8);
  if (d == 64) {
    auto kern = attn_bf16_kernel<64, kBf16Waves>;
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<total, 64 * kBf16Waves, lds, s>>>(a);
  } else {
    auto kern = attn_bf16_kernel<128, kBf16Waves>;
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<total, 64 * kBf16Waves, lds, s>>>(a);
  }
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}
