// bf16 MFMA kernels of the fused block-sparse attention + centroid compensation.
// Paper: Eq. (1), Eq. (6), Algorithm 2 (see attention.hip for the decomposition).
#include "attention.h"

#include <type_traits>

namespace svgear {
namespace {

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

static inline size_t lds_bytes_generic(int D, int Ck) {
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
    const bf16_t* qr = static_cast<const bf16_t*>(p.qp) + q_row_offset(p, bh, qvalid ? qrow : row_end - 1, D);
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
      int64_t lse_idx;
      bf16_t* o = static_cast<bf16_t*>(p.op) + out_row_offset(p, bh, qrow, D, lse_idx);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = pack_bf16(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
          w.y = pack_bf16(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
          *reinterpret_cast<uint2*>(o + 32 * db + 8 * g + 4 * lh) = w;
        }
      if (p.lse && lh == 0) p.lse[lse_idx] = (m + log2f(lt)) * kLn2;
    }
  }
}


// ------------------------------------------------------------------------------ d = 128
// Same algorithm, data path built on two gfx950 features:
//  * K and V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per
//    lane, a wave fills 1 KB = 4 rows of 256 B contiguously), so no VGPRs stage the tiles
//    and the loads of tile t+1 fly while tile t is computed;
//  * V stays row-major [key][dim] in LDS and the A operand of O^T += V^T P^T is fetched
//    with the LDS transpose read (ds_read_b64_tr_b16): within a group of 16 lanes, lane j
//    receives element j%4 of the four 8-byte rows addressed by lanes j/4, j/4+4, j/4+8,
//    j/4+12 of the group. Lanes r of a group address V[key0 + r/4][dim0 + 4*(r%4) ..+3],
//    so lane j gets dims dim0+j of keys key0..key0+3.
// Bank conflicts are avoided by XOR-swizzling the 16-byte chunk index inside each 256 B
// row (K: chunk ^ (row % 16); V: chunk ^ 4*(row % 4)); the swizzle is applied on the
// global side of the copy (a lane picks which global chunk lands in its LDS slot).
constexpr float kLazyRescale = 8.0f;  // log2 headroom before the running maximum is refreshed

typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
// acc + lo(p) + hi(p) for a packed bf16 pair (v_dot2c_f32_bf16 against (1, 1))
__device__ __forceinline__ float dot2_ones(uint32_t pair, float acc) {
  union { uint32_t u; bf16x2v b; } x, one;
  x.u = pair;
  one.u = 0x3f803f80u;
  return __builtin_amdgcn_fdot2_f32_bf16(x.b, one.b, acc, false);
}

// value held by lane ^ 32 (v_permlane32_swap: a VALU exchange of the two wave halves, no LDS)
__device__ __forceinline__ float swap32(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16* lds_v4i16_ptr;

__device__ __forceinline__ bf16x8 tr_pair(const unsigned char* lds_base, int off_bytes) {
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(lds_base + off_bytes));
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(lds_base + off_bytes + 8 * 256));
  union { struct { v4i16 a, b; } s; bf16x8 v; } c;
  c.s.a = lo;
  c.s.b = hi;
  return c.v;
}

// A wave-uniform pointer the compiler could not prove uniform, moved to scalar registers.
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)(p);
}

static inline size_t lds_bytes_d128(int Ck, int stages) {
  const size_t kv = (size_t)stages * 2 * BN * 128 * 2;  // K and V, `stages` buffers each
  const size_t lw = (size_t)align_up(Ck, 64) * 4;
  const size_t seg = (size_t)(2 * (Ck + 2) + 1) * 4;  // vstart, pstart, claimed tile slot
  return kv + (size_t)(stages + 2) * BN * 4 + lw + align_up(seg, 16);
}


// NW waves of 32 query rows (three per SIMD); NSTAGE K/V tile buffers. The first CW waves of
// the workgroup (the oldest wave of every SIMD, which finishes its step first) issue the tile
// copies, after their compute of the step (just before the tile barrier): measured faster
// than issuing them behind the score MFMAs or from more waves.
template <int NW, int NSTAGE, int CW>
__global__ void __launch_bounds__(64 * NW, 1)
attn_bf16_d128_kernel(AttnArgs p) {
  constexpr int D = 128;
  constexpr int NT = 64 * NW;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int TILE_BYTES = BN * D * 2;            // 16 KB
  constexpr int INST_PER_TILE = TILE_BYTES / 1024;  // wave-wide 1 KB copies per tensor tile
  constexpr int LOADS_PER_TILE = 2 * INST_PER_TILE / CW;  // copy instructions per copying wave per tile
  constexpr int RS = NSTAGE + 1;                    // row-map ring
  static_assert(INST_PER_TILE % CW == 0 && CW <= NW, "copies must split evenly over the copying waves");

  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  unsigned char* Ks = smem;                        // [NSTAGE][64 rows][256 B], chunk-swizzled
  unsigned char* Vs = smem + NSTAGE * TILE_BYTES;  // [NSTAGE][64 rows][256 B], chunk-swizzled
  int32_t* rowmap = reinterpret_cast<int32_t*>(smem + 2 * NSTAGE * TILE_BYTES);  // [RS][BN]
  float* lw = reinterpret_cast<float*>(rowmap + RS * BN);  // [align64(Ck)] compensation biases
  float* rag_bias = lw + ((p.Ck + 63) & ~63);              // [BN] bias of the ragged routed tile
  int32_t* vstart = reinterpret_cast<int32_t*>(rag_bias + BN);
  int32_t* pstart = vstart + (p.Ck + 2);

  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // Every workgroup claims one tile: the next of the work list of the XCD it runs on (tiles
  // of one query cluster are neighbours in a list, so the CUs of an XCD work on the same
  // routed K/V at the same time and share it in their L2), or, once that list is used up, of
  // the other XCDs' lists. Lists are sorted longest tile first and workgroups start in
  // order, so the long tiles start early and the short ones fill the end of the launch. The
  // grid covers the tile-count bound; workgroups that find every list used up exit.
  int32_t* slot_s = pstart + (p.Ck + 2);
  if (tid == 0) {
    const int my_xcd = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 7;  // XCC_ID
    int found = -1;
    for (int xk = 0; xk < 8 && found < 0; ++xk) {
      const int xl = (my_xcd + xk) & 7;
      if (p.sched_x[16 + xl] >= p.sched_x[8 + xl]) continue;  // used up (the counter only grows)
      const int slot = atomicAdd(p.sched_x + 16 + xl, 1);
      if (slot < p.sched_x[8 + xl]) found = p.sched_x[xl] + slot;
    }
    *slot_s = found;
  }
  __syncthreads();
  const int claimed = __builtin_amdgcn_readfirstlane(*slot_s);
  if (claimed < 0) return;
  const int bh = p.sched_bh[claimed], a = p.sched_a[claimed], row0 = p.sched_row0[claimed];
  const int Cq = p.Cq, Ck = p.Ck, R = Cq + 1, Cc = Ck + 1, W = (Cc + 31) / 32;
  const int32_t* ko = p.k_offsets + (int64_t)bh * (Ck + 2);
  const int row_end = p.sched_rend[claimed];  // the tile's rows are [row0, row_end), all of query cluster a
  const int32_t* rp = p.row_ptr + (int64_t)bh * (R + 1);
  const int32_t* ci = p.col_idx + (int64_t)bh * R * Cc + rp[a];
  const int ne = rp[a + 1] - rp[a];
  const uint32_t* mrow = p.mask_bits + ((int64_t)bh * R + a) * W;

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
  // (part 2 leaves the routed keys out, part 1 the centroid tiles: the two-stage form)
  const int n_r = p.part == 2 ? 0 : __builtin_amdgcn_readfirstlane(vstart[ne]);  // wave-uniform
  const int nt_r = (n_r + BN - 1) / BN;
  const int nt_c = (a < Cq && p.part != 1) ? (Ck + BN - 1) / BN : 0;
  const int T = nt_r + nt_c;
  const int nt_full = n_r / BN;  // routed tiles with all 64 keys valid
  if (tid < BN) rag_bias[tid] = (nt_full * BN + tid < n_r) ? 0.f : -INFINITY;

  const bf16_t* kh = static_cast<const bf16_t*>(p.kp) + (int64_t)bh * p.Nk * D;
  const bf16_t* vh = static_cast<const bf16_t*>(p.vp) + (int64_t)bh * p.Nk * D;
  const bf16_t* kc = p.kbar16 + (int64_t)bh * Ck * D;
  const bf16_t* vc = p.vbar16 + (int64_t)bh * Ck * D;

  int cur = 0;  // segment cursor of threads 0..63 (virtual key position -> permuted row)
  auto map_tile = [&](int t) __attribute__((always_inline)) {
    if (tid < BN) {
      int phys;
      if (t < nt_r) {
        const int pos = t * BN + tid;
        if (pos < n_r) {
          while (pos >= vstart[cur + 1]) ++cur;
          phys = pstart[cur] + (pos - vstart[cur]);
        } else {
          phys = 0;  // masked by rag_bias; any valid row
        }
      } else {
        const int b = (t - nt_r) * BN + tid;
        phys = b < Ck ? b : Ck - 1;
      }
      rowmap[(t % RS) * BN + tid] = phys;
    }
  };

  // one wave-wide copy moves rows 4*inst .. 4*inst+3 of a tile; lane -> (row, LDS chunk slot).
  // Copy i of this wave is instruction inst = wave + i*CW of the tile: tile row cp_rr + 4*i*CW.
  // CW is a multiple of 4, so the row's swizzle phases (row % 16, row % 4), and with them the
  // 16-byte chunk a lane fetches, are the same for every i.
  static_assert(CW % 4 == 0, "copy rows of one lane must share their swizzle phase");
  constexpr int CPW = INST_PER_TILE / CW;  // copies per tensor per wave per tile
  const uint32_t lds_k0 = lds_address(Ks), lds_v0 = lds_address(Vs);
  const int cp_rr = 4 * (wave % CW) + (lane >> 4);
  const uint32_t cp_koff = (uint32_t)(((lane & 15) ^ (cp_rr & 15)) << 4);
  const uint32_t cp_voff = (uint32_t)(((lane & 15) ^ ((cp_rr & 3) << 2)) << 4);
  // permuted rows (of K/V or of the centroid tables) this lane copies for tile t
  auto fetch_rows = [&](int t, int (&rows)[CPW]) __attribute__((always_inline)) {
    const int32_t* rm = rowmap + (t % RS) * BN + cp_rr;
#pragma unroll
    for (int i = 0; i < CPW; ++i) rows[i] = rm[4 * i * CW];
  };
  auto issue_copies = [&](int t) __attribute__((always_inline)) {
    if (CW < NW && wave >= CW) return;
    int rows[CPW];
    fetch_rows(t, rows);
    const void* kb = uniform_ptr(t < nt_r ? kh : kc);
    const void* vb = uniform_ptr(t < nt_r ? vh : vc);
    const uint32_t kdst = lds_k0 + (t % NSTAGE) * TILE_BYTES + wave * 1024;
    const uint32_t vdst = lds_v0 + (t % NSTAGE) * TILE_BYTES + wave * 1024;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
      const uint32_t rowoff = (uint32_t)rows[i] * (D * 2);
      async_copy_16B(kb, rowoff + cp_koff, __builtin_amdgcn_readfirstlane(kdst + i * CW * 1024));
      async_copy_16B(vb, rowoff + cp_voff, __builtin_amdgcn_readfirstlane(vdst + i * CW * 1024));
    }
  };

  // per-lane LDS byte offsets of the MFMA operands
  // K row li of a 32-row block, dims 16s + 8lh .. +7: chunk (2s + lh) ^ (li % 16)
  // (the swizzles are XORs of disjoint bit fields, so operand s / block db is the offset of
  // operand 0 with s << 5 / db << 6 XORed in: one register each instead of a table)
  const int koff0 = li * 256 + ((lh ^ (li & 15)) << 4);
  auto koff = [&](int s) { return koff0 ^ (s << 5); };
  int voff0;  // transpose read: group = lane/16 -> (dim half, key half); r = lane%16
  {
    const int r = lane & 15, g = lane >> 4, ddhalf = g & 1, khalf = g >> 1;
    voff0 = (4 * khalf + (r >> 2)) * 256 + ((4 * (r >> 2) + 2 * ddhalf + ((r & 3) >> 1)) << 4) + (r & 1) * 8;
  }
  auto voff = [&](int db) { return voff0 ^ (db << 6); };

  const bool wave_active = (row0 + 32 * wave) < row_end;
  bf16x8 bq[KS];
  {
    const int qrow = row0 + 32 * wave + li;
    const bf16_t* qr = static_cast<const bf16_t*>(p.qp) + q_row_offset(p, bh, qrow < row_end ? qrow : row_end - 1, D);
#pragma unroll
    for (int s = 0; s < KS; ++s) bq[s] = as_bf16x8(*reinterpret_cast<const uint4*>(qr + 16 * s + 8 * lh));
  }
  // Q must be in registers before the asynchronous tile copies start: the compiler does not
  // see those copies and would otherwise wait for "its" loads inside the main loop
  SVGEAR_WAIT_VMCNT(0);

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float c = p.scale * kLog2e;

  auto rescale = [&](float m_new) __attribute__((always_inline)) {
    const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - m_new);
    l *= alpha;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    m = m_new;
  };

  // ---- S^T = K Q^T of tile t: 64 keys x 32 queries; register r of block kb is key
  // 32kb + 8(r/4) + 4lh + r%4, query li. The scores of tile t+1 are computed at the end of
  // pipeline step t (see below), so they live in registers across the tile barrier.
  f32x16 sacc[2];
  auto scores = [&](int t) __attribute__((always_inline)) {
    const unsigned char* Kb = Ks + (t % NSTAGE) * TILE_BYTES;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
    // the two 32-key blocks alternate so that consecutive MFMAs are independent; operand
    // reads run four fragments ahead of the MFMAs that consume them
    bf16x8 ak[2 * KS];
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i)
      ak[i] = as_bf16x8(*reinterpret_cast<const uint4*>(Kb + (i & 1) * 32 * 256 + koff(i >> 1)));
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i)
      sacc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[i], bq[i >> 1], sacc[i & 1], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
    for (int i = 0; i < 2 * KS - 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  };

  // ---- online softmax of tile t in the base-2 domain, from its scores in sacc to the packed
  // bf16 probabilities pk; the running maximum m is refreshed lazily (only when a score
  // exceeds it by more than 2^kLazyRescale), so O is rarely rescaled. BIASED = false: a full
  // routed tile. BIASED = true: per-key additive bias (ragged routed tile: 0 / -inf;
  // compensation tile: log2|k_b| or -inf).
  uint32_t pk[2][8];
  auto softmax = [&](int t, auto biased_tag) __attribute__((always_inline)) {
    constexpr bool BIASED = decltype(biased_tag)::value;
    if constexpr (!BIASED) {
      // four independent max chains (a single chain of 16 dependent ops stalls the wave)
      float mxa = fmaxf(sacc[0][0], sacc[1][0]), mxb = fmaxf(sacc[0][1], sacc[1][1]);
      float mxc = fmaxf(sacc[0][2], sacc[1][2]), mxd = fmaxf(sacc[0][3], sacc[1][3]);
#pragma unroll
      for (int r = 4; r < 16; r += 4) {
        mxa = fmaxf(fmaxf(mxa, sacc[0][r]), sacc[1][r]);
        mxb = fmaxf(fmaxf(mxb, sacc[0][r + 1]), sacc[1][r + 1]);
        mxc = fmaxf(fmaxf(mxc, sacc[0][r + 2]), sacc[1][r + 2]);
        mxd = fmaxf(fmaxf(mxd, sacc[0][r + 3]), sacc[1][r + 3]);
      }
      float mx = fmaxf(fmaxf(mxa, mxb), fmaxf(mxc, mxd));
      mx = fmaxf(mx, swap32(mx));
      const float ms = mx * c;
      if (__any(ms > m + kLazyRescale)) rescale(fmaxf(m, ms));
      const float neg_m = -m;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r], c, neg_m));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][r + 1], c, neg_m));
          pk[kb][r >> 1] = pack_bf16(p0, p1);
        }
    } else {
      const float* lwt = t < nt_r ? rag_bias : lw + (t - nt_r) * BN;
      float mx = -INFINITY;
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
      mx = fmaxf(mx, swap32(mx));
      if (__any(mx > m + kLazyRescale)) rescale(fmaxf(m, mx));
      const float m_use = (m == -INFINITY) ? 0.f : m;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(sacc[kb][r] - m_use);
          const float p1 = __builtin_amdgcn_exp2f(sacc[kb][r + 1] - m_use);
          pk[kb][r >> 1] = pack_bf16(p0, p1);
        }
    }
    // row sums from the bf16-rounded probabilities (the values the PV product uses), in
    // four independent partial sums
    {
      float l0 = 0.f, l1 = 0.f, l2 = 0.f, l3 = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int u = 0; u < 8; u += 4) {
          l0 = dot2_ones(pk[kb][u], l0);
          l1 = dot2_ones(pk[kb][u + 1], l1);
          l2 = dot2_ones(pk[kb][u + 2], l2);
          l3 = dot2_ones(pk[kb][u + 3], l3);
        }
      l += (l0 + l1) + (l2 + l3);
    }
  };
  // ---- O^T += V^T P^T of tile t: k-step ks covers keys 16ks .. 16ks+15; the transpose reads
  // of k-step ks+1 are issued before the MFMAs of k-step ks
  auto pv = [&](int t) __attribute__((always_inline)) {
    const unsigned char* Vb = Vs + (t % NSTAGE) * TILE_BYTES;
    {
      bf16x8 av[4][DB];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int db = 0; db < DB; ++db) av[ks][db] = tr_pair(Vb, ks * 16 * 256 + voff(db));
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kb = ks >> 1, u4 = (ks & 1) * 4;
        const bf16x8 bp = as_bf16x8(make_uint4(pk[kb][u4], pk[kb][u4 + 1], pk[kb][u4 + 2], pk[kb][u4 + 3]));
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ks][db], bp, oacc[db], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 1);  // reads of k-step 0
#pragma unroll
      for (int ks = 0; ks < 3; ++ks)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);  // MFMA (ks, db)
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);  // the two reads of operand (ks+1, db)
        }
      __builtin_amdgcn_sched_group_barrier(0x008, DB, 1);
    }
  };

  // Pipeline step t (between two workgroup barriers). The three waves of a SIMD (wave / 4 =
  // phase group) run the same three phases per step - scores, softmax, PV - but each group
  // starts at a different one, so that while one wave is in its softmax (vector ALU) the other
  // two have matrix work queued:
  //   group 0:  S(t)   softmax(t)  PV(t)
  //   group 1:  softmax(t)  PV(t)  S(t+1)            (prologue: S(0))
  //   group 2:  PV(t)  S(t+1)  softmax(t+1)          (prologue: S(0), softmax(0))
  // (of the six ways to give the three orders to the oldest, middle and youngest wave of a
  // SIMD this one measured fastest, the others 3-6 % slower)
  // Step t therefore reads K(t), K(t+1) and V(t): both must have landed before it starts, and
  // the buffers of tile t are free after its barrier; the copies of tile t+NSTAGE-1 are
  // issued during step t.
  static_assert(NW == 12, "three phase groups of four waves");
  const int group = wave >> 2;
  auto run_step = [&](int t, auto group_tag, auto biased_tag) __attribute__((always_inline)) {
    constexpr int G = decltype(group_tag)::value;
    const bool more = t + NSTAGE - 1 < T;
    if (wave_active) {
      if constexpr (G == 0) {
        scores(t);
        softmax(t, biased_tag);
        pv(t);
      } else if constexpr (G == 1) {
        softmax(t, biased_tag);
        pv(t);
        __builtin_amdgcn_sched_barrier(0);  // keep the two MFMA pipelines in separate scheduling regions
        // (unconditional, so the old and the new scores never have to be live together: the
        // last step recomputes its own tile's scores, which nobody reads)
        scores(t + 1 < T ? t + 1 : t);
      } else {
        pv(t);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < T) {
          scores(t + 1);
          softmax(t + 1, biased_tag);
        } else {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int u = 0; u < 8; ++u) pk[kb][u] = 0u;
        }
      }
    }
    if (more) issue_copies(t + NSTAGE - 1);
    if (t + NSTAGE < T) map_tile(t + NSTAGE);
    // this wave's copies of tile t+2 must have landed (step t+1 reads K(t+2)); one younger
    // tile may stay in flight
    if (more) SVGEAR_WAIT_VMCNT((NSTAGE - 3) * LOADS_PER_TILE);
    else SVGEAR_WAIT_VMCNT(0);
    __syncthreads();
  };

  // prologue: tiles 0 .. NSTAGE-2 in flight, tiles 0 and 1 landed
#pragma unroll
  for (int t = 0; t < NSTAGE; ++t)
    if (t < T) map_tile(t);
  __syncthreads();
#pragma unroll
  for (int t = 0; t < NSTAGE - 1; ++t)
    if (t < T) issue_copies(t);
  if (T >= NSTAGE - 1) SVGEAR_WAIT_VMCNT((NSTAGE - 3) * LOADS_PER_TILE);
  else SVGEAR_WAIT_VMCNT(0);
  __syncthreads();

  // Every group runs T steps (T barriers). The bias tag belongs to the tile whose softmax the
  // step contains: tile t for groups 0 and 1, tile t+1 for group 2.
  if (group == 0) {
    for (int t = 0; t < nt_full; ++t) run_step(t, std::integral_constant<int, 0>{}, std::false_type{});
    for (int t = nt_full; t < T; ++t) run_step(t, std::integral_constant<int, 0>{}, std::true_type{});
  } else if (group == 1) {
    if (wave_active && T > 0) scores(0);
    for (int t = 0; t < nt_full; ++t) run_step(t, std::integral_constant<int, 1>{}, std::false_type{});
    for (int t = nt_full; t < T; ++t) run_step(t, std::integral_constant<int, 1>{}, std::true_type{});
  } else {
    if (wave_active && T > 0) {
      scores(0);
      if (nt_full > 0) softmax(0, std::false_type{});
      else softmax(0, std::true_type{});
    }
    int t = 0;
    for (; t + 1 < nt_full; ++t) run_step(t, std::integral_constant<int, 2>{}, std::false_type{});
    for (; t < T; ++t) run_step(t, std::integral_constant<int, 2>{}, std::true_type{});
  }

  // ---- epilogue: lane holds query li, dims 32db + 8g + 4lh + 0..3
  if (wave_active) {
    const float lt = l + swap32(l);
    const int qrow = row0 + 32 * wave + li;
    if (qrow < row_end) {
      const float inv = lt > 0.f ? 1.0f / lt : 0.f;
      int64_t lse_idx;
      bf16_t* o = static_cast<bf16_t*>(p.op) + out_row_offset(p, bh, qrow, D, lse_idx);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = pack_bf16(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
          w.y = pack_bf16(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
          *reinterpret_cast<uint2*>(o + 32 * db + 8 * g + 4 * lh) = w;
        }
      if (p.lse && lh == 0) p.lse[lse_idx] = (m + log2f(lt)) * kLn2;
    }
  }
}

// ------------------------------------------------------------------------ work lists
// Item = (head, query cluster); its tiles all run T = #routed key tiles + #centroid tiles
// pipeline steps. Items are ranked by T, longest first (ties by index), and dealt to the 8
// lists in boustrophedon order, which keeps the lists' totals close; inside a list the
// longest come first, so a list's tail consists of its shortest tiles.
__global__ void __launch_bounds__(256)
plan_items_kernel(const int32_t* __restrict__ q_offsets, const int32_t* __restrict__ k_offsets,
                  const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx, int Cq, int Ck, int BM,
                  int32_t* __restrict__ item_T, int32_t* __restrict__ item_nt) {
  const int bh = blockIdx.x, R = Cq + 1, Cc = Ck + 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t* qo = q_offsets + (int64_t)bh * (Cq + 2);
  const int32_t* ko = k_offsets + (int64_t)bh * (Ck + 2);
  const int32_t* rp = row_ptr + (int64_t)bh * (R + 1);
  // a wave per query cluster, its lanes over the routed key clusters
  for (int a = wave; a < R; a += 4) {
    const int n = qo[a + 1] - qo[a];
    const int32_t* ci = col_idx + (int64_t)bh * R * Cc + rp[a];
    const int ne = rp[a + 1] - rp[a];
    int64_t nr = 0;
    for (int e = lane; e < ne; e += 64) {
      const int b = ci[e];
      const int sz = ko[b + 1] - ko[b];
      nr += sz > 0 ? sz : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) nr += __shfl_xor(nr, o);
    if (lane == 0) {
      const int nt = n > 0 ? (n + BM - 1) / BM : 0;
      item_nt[bh * R + a] = nt;
      item_T[bh * R + a] = nt > 0 ? (int)((nr + BN - 1) / BN) + (a < Cq ? (Ck + BN - 1) / BN : 0) : 0;
    }
  }
}

// Rank of every item by (T descending, index ascending), by counting: a workgroup ranks 64 items,
// each of its four waves counting over a quarter of all items.
constexpr int kRankItems = 64;
__global__ void __launch_bounds__(256)
plan_rank_kernel(const int32_t* __restrict__ item_T, int M, int32_t* __restrict__ by_rank) {
  __shared__ uint64_t keys[4][64];
  __shared__ int rank_sum[kRankItems];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * kRankItems + lane;
  // larger key = earlier: T descending, then index ascending
  auto key_of = [&](int j) {
    return j < M ? ((uint64_t)(uint32_t)item_T[j] << 32) | (uint32_t)(0x7fffffff - j) : (uint64_t)0;
  };
  const uint64_t mine = key_of(i);
  if (threadIdx.x < kRankItems) rank_sum[threadIdx.x] = 0;
  __syncthreads();
  const int quarter = (M + 3) / 4;
  const int j_lo = wave * quarter, j_hi = min(j_lo + quarter, M);
  int rank = 0;
  for (int j0 = j_lo; j0 < j_hi; j0 += 64) {  // the wave's own tile of keys: no workgroup barrier needed
    keys[wave][lane] = j0 + lane < j_hi ? key_of(j0 + lane) : (uint64_t)0;
    __builtin_amdgcn_wave_barrier();
    const int lim = min(64, j_hi - j0);
    for (int u = 0; u < lim; ++u) rank += keys[wave][u] > mine;
    __builtin_amdgcn_wave_barrier();
  }
  atomicAdd(&rank_sum[lane], rank);
  __syncthreads();
  if (wave == 0 && i < M) by_rank[rank_sum[lane]] = i;
}

// rank r -> (list, position): round r/8 deals one item to every list, odd rounds in reverse
__device__ __forceinline__ int list_of_rank(int r) { return ((r >> 3) & 1) ? 7 - (r & 7) : (r & 7); }

__global__ void __launch_bounds__(1024)
plan_lists_kernel(const int32_t* __restrict__ q_offsets, const int32_t* __restrict__ item_nt,
                  const int32_t* __restrict__ by_rank, int M, int Cq, int BM, int32_t* __restrict__ rank_off,
                  int32_t* __restrict__ sched_bh, int32_t* __restrict__ sched_a, int32_t* __restrict__ sched_row0,
                  int32_t* __restrict__ sched_rend, int32_t* __restrict__ sched_x) {
  __shared__ int32_t part[1024];
  __shared__ int32_t total[8], first[8];
  const int tid = threadIdx.x, R = Cq + 1;
  const int rounds = (M + 7) / 8;
  // exclusive offsets of every item inside its list (list xl = ranks 8k + pos(k, xl))
  for (int xl = 0; xl < 8; ++xl) {
    int carry = 0;
    for (int k0 = 0; k0 < rounds; k0 += 1024) {
      const int k = k0 + tid;
      const int r = 8 * k + ((k & 1) ? 7 - xl : xl);
      const int v = (k < rounds && r < M) ? item_nt[by_rank[r]] : 0;
      part[tid] = v;
      __syncthreads();
      for (int o = 1; o < 1024; o <<= 1) {
        const int t = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += t;
        __syncthreads();
      }
      if (k < rounds && r < M) rank_off[r] = carry + part[tid] - v;
      carry += part[1023];
      __syncthreads();
    }
    if (tid == 0) total[xl] = carry;
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int xl = 0; xl < 8; ++xl) {
      first[xl] = run;
      run += total[xl];
    }
  }
  __syncthreads();
  if (tid < 8) {
    sched_x[tid] = first[tid];
    sched_x[8 + tid] = total[tid];
    sched_x[16 + tid] = 0;
  }
  for (int r = tid; r < M; r += 1024) {
    const int i = by_rank[r], bh = i / R, a = i % R;
    const int nt = item_nt[i];
    const int base = first[list_of_rank(r)] + rank_off[r];
    const int q0 = q_offsets[(int64_t)bh * (Cq + 2) + a], q1 = q_offsets[(int64_t)bh * (Cq + 2) + a + 1];
    // The cluster's 32-row wave blocks are dealt evenly to its nt tiles (sizes differ by at most
    // one block): a cluster of 500 rows becomes two tiles of 8 waves rather than one of 12 and
    // one of 4, whose lone wave per SIMD would leave the matrix cores idle most of the time.
    const int blocks = (q1 - q0 + 31) / 32;
    for (int j = 0; j < nt; ++j) {
      sched_bh[base + j] = bh;
      sched_a[base + j] = a;
      sched_row0[base + j] = q0 + 32 * (int)((int64_t)j * blocks / nt);
      sched_rend[base + j] = min(q1, q0 + 32 * (int)((int64_t)(j + 1) * blocks / nt));
    }
  }
}

}  // namespace

// Tile shape of the d = 128 kernel: 12 waves x 32 query rows per workgroup (one workgroup per
// CU, 3 waves per SIMD at 168 VGPRs), 4 K/V tile buffers.
constexpr int kD128Waves = 12;
constexpr int kD128Stages = 4;
constexpr int kD128CopyWaves = 4;

int attn_bf16_bm(int d) { return d == 128 ? 32 * kD128Waves : 32 * kBf16Waves; }

size_t attn_bf16_lds_bytes(int d, int Ck) {
  return d == 128 ? lds_bytes_d128(Ck, kD128Stages) : lds_bytes_generic(d, Ck);
}

size_t plan_d128_workspace(int BH, int Cq, int64_t Nq) {
  const size_t M = (size_t)BH * (Cq + 1);
  const size_t tiles = (size_t)BH * ((size_t)ceil_div(Nq, 32 * kD128Waves) + Cq + 1);
  return 4 * align_up(M * 4, 256) + 4 * align_up(tiles * 4, 256) + align_up(24 * 4, 256);
}

int plan_d128(AttnArgs& a, void* ws, size_t ws_bytes, hipStream_t s) {
  Workspace w(ws, ws_bytes);
  const int M = a.BH * (a.Cq + 1), BM = 32 * kD128Waves;
  const size_t tiles = (size_t)a.BH * ((size_t)ceil_div(a.Nq, BM) + a.Cq + 1);
  int32_t* item_T = w.take<int32_t>(M);
  int32_t* item_nt = w.take<int32_t>(M);
  int32_t* by_rank = w.take<int32_t>(M);
  int32_t* rank_off = w.take<int32_t>(M);
  int32_t* sched_bh = w.take<int32_t>(tiles);
  int32_t* sched_a = w.take<int32_t>(tiles);
  int32_t* sched_row0 = w.take<int32_t>(tiles);
  int32_t* sched_rend = w.take<int32_t>(tiles);
  int32_t* sched_x = w.take<int32_t>(24);
  if (!w.ok()) return SVGEAR_ERR_WORKSPACE;
  plan_items_kernel<<<a.BH, 256, 0, s>>>(a.q_offsets, a.k_offsets, a.row_ptr, a.col_idx, a.Cq, a.Ck, BM, item_T, item_nt);
  SVGEAR_LAUNCH_CHECK();
  plan_rank_kernel<<<(unsigned)ceil_div(M, kRankItems), 256, 0, s>>>(item_T, M, by_rank);
  SVGEAR_LAUNCH_CHECK();
  plan_lists_kernel<<<1, 1024, 0, s>>>(a.q_offsets, item_nt, by_rank, M, a.Cq, BM, rank_off, sched_bh, sched_a, sched_row0,
                                      sched_rend, sched_x);
  SVGEAR_LAUNCH_CHECK();
  a.sched_bh = sched_bh;
  a.sched_a = sched_a;
  a.sched_row0 = sched_row0;
  a.sched_rend = sched_rend;
  a.sched_x = sched_x;
  return SVGEAR_OK;
}

// Merge of two partial softmax results over disjoint key sets (Algorithm 2's merge step):
// one thread per 8 output elements.
__global__ void __launch_bounds__(256)
merge_kernel(const bf16_t* __restrict__ o1, const float* __restrict__ lse1, const bf16_t* __restrict__ o2,
             const float* __restrict__ lse2, int64_t rows, int d, bf16_t* __restrict__ out,
             float* __restrict__ lse) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (row, group of 8 dims)
  const int per_row = d / 8;
  if (i >= rows * per_row) return;
  const int64_t row = i / per_row;
  const float a = lse1[row], b = lse2[row];
  const float m = fmaxf(a, b);
  float w1 = 0.f, w2 = 0.f;
  if (m > -INFINITY) {
    w1 = expf(a - m);
    w2 = expf(b - m);
  }
  const float den = w1 + w2;
  const float s1 = den > 0.f ? w1 / den : 0.f, s2 = den > 0.f ? w2 / den : 0.f;
  const uint4 x = *reinterpret_cast<const uint4*>(o1 + i * 8), y = *reinterpret_cast<const uint4*>(o2 + i * 8);
  const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
  uint32_t r[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float lo = s1 * __uint_as_float(xs[k] << 16) + s2 * __uint_as_float(ys[k] << 16);
    const float hi = s1 * __uint_as_float(xs[k] & 0xffff0000u) + s2 * __uint_as_float(ys[k] & 0xffff0000u);
    r[k] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
  }
  *reinterpret_cast<uint4*>(out + i * 8) = make_uint4(r[0], r[1], r[2], r[3]);
  if (lse && (i % per_row) == 0) lse[row] = den > 0.f ? m + logf(den) : -INFINITY;
}

int launch_merge(const bf16_t* o1, const float* lse1, const bf16_t* o2, const float* lse2, int64_t rows, int d,
                 bf16_t* out, float* lse, hipStream_t s) {
  merge_kernel<<<(unsigned)ceil_div(rows * (d / 8), 256), 256, 0, s>>>(o1, lse1, o2, lse2, rows, d, out, lse);
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

// `total` workgroups: at least the number of tiles (one workgroup per tile; the rest exit).
int launch_attn_bf16(const AttnArgs& a, int d, unsigned total, hipStream_t s) {
  const size_t lds = attn_bf16_lds_bytes(d, a.Ck);
  if (d == 64) {
    auto kern = attn_bf16_kernel<64, kBf16Waves>;
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<total, 64 * kBf16Waves, lds, s>>>(a);
  } else {
    if (!a.sched_x) return SVGEAR_ERR_INVALID;
    auto kern = attn_bf16_d128_kernel<kD128Waves, kD128Stages, kD128CopyWaves>;
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<total, 64 * kD128Waves, lds, s>>>(a);
  }
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

}  // namespace svgear
