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

// 16 bytes per lane from global memory straight into LDS: the wave's 64 lanes fill 1 KB
// starting at LDS byte address `lds_addr` (wave-uniform), lane l at lds_addr + 16 l.
// Written as inline assembly so that the compiler does not treat every later LDS read as
// dependent on the copy (it would drain the copies before the first read of each tile);
// completion is tracked by hand with vmcnt.
__device__ __forceinline__ void async_copy_16B(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory", "m0");
}
// Same copy with the global address given as a wave-uniform base plus a 32-bit byte offset
// per lane (no 64-bit vector arithmetic).
__device__ __forceinline__ void async_copy_16B(const void* gbase, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
               :
               : "v"(byte_off), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)(p);
}

static inline size_t lds_bytes_d128(int Ck, int stages) {
  const size_t kv = (size_t)stages * 2 * BN * 128 * 2;  // K and V, `stages` buffers each
  const size_t lw = (size_t)align_up(Ck, 64) * 4;
  const size_t seg = (size_t)(2 * (Ck + 1) + 1) * 4;
  return kv + (size_t)(stages + 2) * BN * 4 + lw + align_up(seg, 16);
}

// vmcnt(n) with expcnt and lgkmcnt left unconstrained (gfx9 s_waitcnt encoding)
#define SVGEAR_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// NW waves of 32 query rows; NSTAGE K/V tile buffers (tile t+NSTAGE-1 is in flight while
// tile t is computed).
template <int NW, int NSTAGE>
__global__ void __launch_bounds__(64 * NW, 8 / NW)
attn_bf16_d128_kernel(AttnArgs p) {
  constexpr int D = 128;
  constexpr int NT = 64 * NW;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int TILE_BYTES = BN * D * 2;            // 16 KB
  constexpr int INST_PER_TILE = TILE_BYTES / 1024;  // wave-wide 1 KB copies per tensor tile
  constexpr int LOADS_PER_TILE = 2 * INST_PER_TILE / NW;  // copy instructions per wave per tile
  constexpr int RS = NSTAGE + 1;                    // row-map ring
  static_assert(INST_PER_TILE % NW == 0, "copies must split evenly over the waves");

  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  unsigned char* Ks = smem;                        // [NSTAGE][64 rows][256 B], chunk-swizzled
  unsigned char* Vs = smem + NSTAGE * TILE_BYTES;  // [NSTAGE][64 rows][256 B], chunk-swizzled
  int32_t* rowmap = reinterpret_cast<int32_t*>(smem + 2 * NSTAGE * TILE_BYTES);  // [RS][BN]
  float* lw = reinterpret_cast<float*>(rowmap + RS * BN);  // [align64(Ck)] compensation biases
  float* rag_bias = lw + ((p.Ck + 63) & ~63);              // [BN] bias of the ragged routed tile
  int32_t* vstart = reinterpret_cast<int32_t*>(rag_bias + BN);
  int32_t* pstart = vstart + (p.Ck + 2);

  const int total = gridDim.x;
  const int wg = blockIdx.x;
  const int logical = (wg & 7) * (total >> 3) + (wg >> 3);
  const int bh = logical / p.max_tiles, tile = logical % p.max_tiles;
  if (bh >= p.BH || tile >= p.n_tiles[bh]) return;

  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  const int nt_full = n_r / BN;  // routed tiles with all 64 keys valid
  if (tid < BN) rag_bias[tid] = (nt_full * BN + tid < n_r) ? 0.f : -INFINITY;

  const bf16_t* kh = static_cast<const bf16_t*>(p.kp) + (int64_t)bh * p.Nk * D;
  const bf16_t* vh = static_cast<const bf16_t*>(p.vp) + (int64_t)bh * p.Nk * D;
  const bf16_t* kc = p.kbar16 + (int64_t)bh * Ck * D;
  const bf16_t* vc = p.vbar16 + (int64_t)bh * Ck * D;

  int cur = 0;  // segment cursor of threads 0..63 (virtual key position -> permuted row)
  auto map_tile = [&](int t) {
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
  // Copy i of this wave is instruction inst = wave + i*NW of the tile: its tile row, the
  // swizzled 16-byte chunk it fetches and its LDS destination do not depend on the tile.
  constexpr int CPW = INST_PER_TILE / NW;  // copies per tensor per wave per tile
  const int cp_row = lane >> 4, cp_slot = lane & 15;
  const uint32_t lds_k0 = lds_address(Ks), lds_v0 = lds_address(Vs);
  int cp_rr[CPW];
  uint32_t cp_koff[CPW], cp_voff[CPW];
#pragma unroll
  for (int i = 0; i < CPW; ++i) {
    cp_rr[i] = 4 * (wave + i * NW) + cp_row;
    cp_koff[i] = (uint32_t)((cp_slot ^ (cp_rr[i] & 15)) << 4);
    cp_voff[i] = (uint32_t)((cp_slot ^ ((cp_rr[i] & 3) << 2)) << 4);
  }
  // permuted rows (of K/V or of the centroid tables) this lane copies for tile t
  auto fetch_rows = [&](int t, int (&rows)[CPW]) {
    const int32_t* rm = rowmap + (t % RS) * BN;
#pragma unroll
    for (int i = 0; i < CPW; ++i) rows[i] = rm[cp_rr[i]];
  };
  auto issue_copies = [&](int t, const int (&rows)[CPW]) {
    const bf16_t* kb = t < nt_r ? kh : kc;
    const bf16_t* vb = t < nt_r ? vh : vc;
    const uint32_t kdst = lds_k0 + (t % NSTAGE) * TILE_BYTES + wave * 1024;
    const uint32_t vdst = lds_v0 + (t % NSTAGE) * TILE_BYTES + wave * 1024;
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
      const uint32_t rowoff = (uint32_t)rows[i] * (D * 2);
      async_copy_16B(kb, rowoff + cp_koff[i], __builtin_amdgcn_readfirstlane(kdst + i * NW * 1024));
      async_copy_16B(vb, rowoff + cp_voff[i], __builtin_amdgcn_readfirstlane(vdst + i * NW * 1024));
    }
  };
  auto issue_loads = [&](int t) {
    int rows[CPW];
    fetch_rows(t, rows);
    issue_copies(t, rows);
  };

  // per-lane LDS byte offsets of the MFMA operands
  // K row li of a 32-row block, dims 16s + 8lh .. +7: chunk (2s + lh) ^ (li % 16)
  int koff[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) koff[s] = li * 256 + (((2 * s + lh) ^ (li & 15)) << 4);
  int voff[DB];  // transpose read: group = lane/16 -> (dim half, key half); r = lane%16
  {
    const int r = lane & 15, g = lane >> 4, ddhalf = g & 1, khalf = g >> 1;
#pragma unroll
    for (int db = 0; db < DB; ++db)
      voff[db] = (4 * khalf + (r >> 2)) * 256 + ((4 * (db ^ (r >> 2)) + 2 * ddhalf + ((r & 3) >> 1)) << 4) + (r & 1) * 8;
  }

  const int qrow = row0 + 32 * wave + li;
  const bool qvalid = qrow < row_end;
  const bool wave_active = (row0 + 32 * wave) < row_end;
  bf16x8 bq[KS];
  {
    const bf16_t* qr = static_cast<const bf16_t*>(p.qp) + ((int64_t)bh * p.Nq + (qvalid ? qrow : row_end - 1)) * D;
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

  auto rescale = [&](float m_new) {
    const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - m_new);
    l *= alpha;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    m = m_new;
  };

  // One 64-key tile for this wave's 32 queries. BIASED = false: a full routed tile.
  // BIASED = true: per-key additive bias (ragged routed tile: 0 / -inf; compensation tile:
  // log2|k_b| or -inf).
  auto compute_tile = [&](int t, auto biased_tag, auto&& after_scores) {
    constexpr bool BIASED = decltype(biased_tag)::value;
    const unsigned char* Kb = Ks + (t % NSTAGE) * TILE_BYTES;
    const unsigned char* Vb = Vs + (t % NSTAGE) * TILE_BYTES;
    // ---- S^T = K Q^T : 64 keys x 32 queries; register r of block kb is key
    // 32kb + 8(r/4) + 4lh + r%4, query li
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
    {
      // the two 32-key blocks alternate so that consecutive MFMAs are independent; operand
      // reads run four fragments ahead of the MFMAs that consume them
      bf16x8 ak[2 * KS];
#pragma unroll
      for (int i = 0; i < 2 * KS; ++i)
        ak[i] = as_bf16x8(*reinterpret_cast<const uint4*>(Kb + (i & 1) * 32 * 256 + koff[i >> 1]));
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
    }
    after_scores();
    // ---- online softmax in the base-2 domain; the running maximum m is refreshed lazily
    // (only when a score exceeds it by more than 2^kLazyRescale), so O is rarely rescaled
    uint32_t pk[2][8];
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
    // ---- O^T += V^T P^T : k-step ks covers keys 16ks .. 16ks+15; the transpose reads of
    // k-step ks+1 are issued before the MFMAs of k-step ks
    {
      bf16x8 av[4][DB];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int db = 0; db < DB; ++db) av[ks][db] = tr_pair(Vb, ks * 16 * 256 + voff[db]);
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

  // pipeline step around the compute of tile t: the rows of tile t+NSTAGE-1 are looked up
  // first, its copies are issued once the score MFMAs are in flight (the copies have tiles
  // of slack; the wave should not stall on the row lookup before feeding the matrix cores)
  auto run_tile = [&](int t, auto biased_tag) {
    const bool more = t + NSTAGE - 1 < T;
    int rows[CPW];
    if (more) fetch_rows(t + NSTAGE - 1, rows);
    if (wave_active) compute_tile(t, biased_tag, [&] { if (more) issue_copies(t + NSTAGE - 1, rows); });
    else if (more) issue_copies(t + NSTAGE - 1, rows);
    if (t + NSTAGE < T) map_tile(t + NSTAGE);
    // this wave's copies of tile t+1 must have landed; younger tiles may stay in flight
    if (more) SVGEAR_WAIT_VMCNT((NSTAGE - 2) * LOADS_PER_TILE);
    else SVGEAR_WAIT_VMCNT(0);
    __syncthreads();
  };

  // prologue: tiles 0 .. NSTAGE-2 in flight, tile 0 landed
#pragma unroll
  for (int t = 0; t < NSTAGE; ++t)
    if (t < T) map_tile(t);
  __syncthreads();
#pragma unroll
  for (int t = 0; t < NSTAGE - 1; ++t)
    if (t < T) issue_loads(t);
  if (T >= NSTAGE - 1) SVGEAR_WAIT_VMCNT((NSTAGE - 2) * LOADS_PER_TILE);
  else SVGEAR_WAIT_VMCNT(0);
  __syncthreads();

  for (int t = 0; t < nt_full; ++t) run_tile(t, std::false_type{});
  for (int t = nt_full; t < T; ++t) run_tile(t, std::true_type{});

  // ---- epilogue: lane holds query li, dims 32db + 8g + 4lh + 0..3
  if (wave_active) {
    const float lt = l + swap32(l);
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

}  // namespace

// Tile shape of the d = 128 kernel: 8 waves x 32 query rows per workgroup (one workgroup per
// CU, 2 waves per SIMD), 4 K/V tile buffers in flight.
constexpr int kD128Waves = 8;
constexpr int kD128Stages = 4;

int attn_bf16_bm(int d) { return d == 128 ? 32 * kD128Waves : 32 * kBf16Waves; }

size_t attn_bf16_lds_bytes(int d, int Ck) {
  return d == 128 ? lds_bytes_d128(Ck, kD128Stages) : lds_bytes_generic(d, Ck);
}

int launch_attn_bf16(const AttnArgs& a, int d, unsigned total, hipStream_t s) {
  const size_t lds = attn_bf16_lds_bytes(d, a.Ck);
  if (d == 64) {
    auto kern = attn_bf16_kernel<64, kBf16Waves>;
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<total, 64 * kBf16Waves, lds, s>>>(a);
  } else {
    auto kern = attn_bf16_d128_kernel<kD128Waves, kD128Stages>;
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<total, 64 * kD128Waves, lds, s>>>(a);
  }
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

}  // namespace svgear
